// Row-wise kernels of the block-rotation MXFP4 path for gfx950: block Hadamard rotation
// (Sec. 4.3, Eq. 1), MXFP4 quantization (Sec. 4.1) and their fusion, the online step
// that precedes a quantized linear layer.  All of them stream X once from HBM.
//
// Work decomposition.  A "chunk" is 8 consecutive elements of a row (16 bytes of bf16,
// 32 bytes of fp32), held by one lane; 4 consecutive lanes (a DPP quad) hold one
// 32-element MXFP4 group, so the group maximum is two quad-permute steps and the group's
// 8 packed codes per lane form one dword store.  Rotation stages h = 1, 2, 4 run inside
// the lane, h = 8 ... 256 between lanes of the wavefront, larger h through LDS.
#include "brq_device.h"
#include "brq_launch.h"

namespace brq {

enum RowMode { MODE_ROTATE = 0, MODE_QUANT = 1, MODE_FUSED = 2, MODE_STATS = 3 };

struct RowArgs {
    const void* x;      // [M][ldx]
    void* y;            // rotate: [M][ldy]
    uint32_t* codes;    // quant/fused: [M][K/8] dwords
    uint8_t* scales;    // quant/fused: [M][K/32]
    int64_t ldx, ldy;   // in elements
    uint32_t cpr;       // chunks per row = K/8
    uint32_t nchunks;   // M * K/8
    // Tiled output (codes: 64 rows x 64 bytes per (slab, stage) block; scales: 64 rows x 16
    // bytes per (slab, superstage) block): blocks per slab, 0 = row-major output.
    uint32_t stages;    // Kp/128, Kp = K rounded up to a multiple of 512
    uint32_t sstages;   // Kp/512
    const int8_t* signs;   // [K] or null: element k is negated on load where signs[k] < 0
    const void* x2;        // producer kernels: the `up` matrix [M][ldx2] (x is then `gate`)
    int64_t ldx2;
    uint32_t hround;       // producer kernels: the activation passes through bf16
    // MODE_STATS outputs (any may be null) and thresholds
    float* amax;                   // [M][K/32]
    float* sqerr;                  // [M][K/32]
    float* sqerr_bfp4;             // [M][K/32]
    unsigned long long* counts;    // [nt], added to
    uint32_t nt;
    float th[8];
    uint32_t sign_fixed;   // the grid was sized so that a lane's column is the same in every pass
};

// The random sign diagonal of a randomized Hadamard rotation (Sec. 5.1 and the Appendix use
// "randomized"/"stochastic" Hadamard matrices): x_k -> s_k x_k before the butterfly, an exact
// flip of the fp32 sign bit.  `signs` points at the 8 sign bytes of this chunk (8-byte aligned).
// The same flip as 8 ready-made sign-bit masks: kernels whose lanes keep their column from one
// grid-stride pass to the next (the host sizes the grid for that: sign_fixed) expand the sign
// bytes once, and a chunk then costs 8 XORs.
__device__ __forceinline__ void sign_masks(uint32_t (&m)[8], const int8_t* signs) {
    const uint2 sg = *reinterpret_cast<const uint2*>(signs);
#pragma unroll
    for (int i = 0; i < 8; ++i) m[i] = (((i < 4) ? sg.x : sg.y) << (24 - 8 * (i & 3))) & 0x80000000u;
}
__device__ __forceinline__ void flip(float (&v)[8], const uint32_t (&m)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = as_f32(as_u32(v[i]) ^ m[i]);
}
// Byte offsets of chunk kc (8 elements = 4 code bytes) of row `row` in the tiled layout.
__device__ __forceinline__ uint64_t tiled_code_offset(uint32_t row, uint32_t kc, uint32_t stages) {
    return ((uint64_t)(row >> 6) * stages + (kc >> 4)) * 4096u + (row & 63u) * 64u + (kc & 15u) * 4u;
}
__device__ __forceinline__ uint64_t tiled_scale_offset(uint32_t row, uint32_t kc, uint32_t sstages) {
    return ((uint64_t)(row >> 6) * sstages + (kc >> 6)) * 1024u + (row & 63u) * 16u + ((kc >> 2) & 15u);
}

// ---- chunk load / store ---------------------------------------------------------

// X is read exactly once and the outputs are next touched by another kernel: loads and the
// stores of rotated values and codes carry the non-temporal hint, so the stream does not
// displace what the caches hold (on a 16 B in / 4 B out stream this alone is worth about 10% of
// HBM throughput).  The scale bytes are stored plainly: a cache line of scales is completed by
// several wavefronts, and the L2 merges their pieces before the line goes to memory.
template <bool BF16>
__device__ __forceinline__ void store_chunk(void* p, const float (&v)[8]) {
    if constexpr (BF16) {
        v4i w;
        w.x = (int)(f32_to_bf16_bits(v[0]) | (f32_to_bf16_bits(v[1]) << 16));
        w.y = (int)(f32_to_bf16_bits(v[2]) | (f32_to_bf16_bits(v[3]) << 16));
        w.z = (int)(f32_to_bf16_bits(v[4]) | (f32_to_bf16_bits(v[5]) << 16));
        w.w = (int)(f32_to_bf16_bits(v[6]) | (f32_to_bf16_bits(v[7]) << 16));
        __builtin_nontemporal_store(w, reinterpret_cast<v4i*>(p));
    } else {
        __builtin_nontemporal_store(v4f{v[0], v[1], v[2], v[3]}, reinterpret_cast<v4f*>(p));
        __builtin_nontemporal_store(v4f{v[4], v[5], v[6], v[7]}, reinterpret_cast<v4f*>(p) + 1);
    }
}

// fp32 output of the rotation: a lane's 8 values are 32 contiguous bytes, and two 16-byte stores per
// lane would leave the lanes of either instruction 32 bytes apart - the store path then takes them
// one lane at a time (178 us on X 16384 x 8192, where a plain conversion copy of the same traffic takes
// 137).  The four lanes of a quad hold 128 contiguous bytes (consecutive lanes = consecutive chunks of
// one row): the 16-byte pieces are traded inside the quad so that store A writes pieces 0..3 and store
// B pieces 4..7, lane t piece t - 64 contiguous bytes per quad and instruction.  Piece k sits in lane
// k >> 1, half k & 1.  Every lane of the quad must be active.
__device__ __forceinline__ void store_chunk_f32_quad(char* p, const float (&v)[8], uint32_t lane) {
    const uint32_t t = lane & 3u;
    const bool odd = (t & 1u) != 0;
    v4f a, b;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int lo = __builtin_bit_cast(int, v[k]), hi = __builtin_bit_cast(int, v[4 + k]);
        const int a_lo = __builtin_amdgcn_update_dpp(lo, lo, 0x50 /* quad_perm [0,0,1,1] */, 0xF, 0xF, true);
        const int a_hi = __builtin_amdgcn_update_dpp(hi, hi, 0x50, 0xF, 0xF, true);
        const int b_lo = __builtin_amdgcn_update_dpp(lo, lo, 0xFA /* quad_perm [2,2,3,3] */, 0xF, 0xF, true);
        const int b_hi = __builtin_amdgcn_update_dpp(hi, hi, 0xFA, 0xF, 0xF, true);
        a[k] = __builtin_bit_cast(float, odd ? a_hi : a_lo);
        b[k] = __builtin_bit_cast(float, odd ? b_hi : b_lo);
    }
    __builtin_nontemporal_store(a, reinterpret_cast<v4f*>(p - 16 * (int)t));
    __builtin_nontemporal_store(b, reinterpret_cast<v4f*>(p + 64 - 16 * (int)t));
}

// The lane's 8 input values: the chunk at p, or (PROD) the gated activation of the chunks at p
// (gate) and p2 (up), computed here so that it never visits HBM.
template <bool BF16, bool PROD>
__device__ __forceinline__ void load_input(const void* p, const void* p2, bool hround, float (&v)[8]) {
    if constexpr (!PROD) {
        load_chunk<BF16>(p, v);
    } else if constexpr (BF16) {
        // both loads first, then the arithmetic
        const v4i a = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p));
        const v4i b = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p2));
        float w[8];
        v[0] = bf16_lo((uint32_t)a.x); v[1] = bf16_hi((uint32_t)a.x); v[2] = bf16_lo((uint32_t)a.y); v[3] = bf16_hi((uint32_t)a.y);
        v[4] = bf16_lo((uint32_t)a.z); v[5] = bf16_hi((uint32_t)a.z); v[6] = bf16_lo((uint32_t)a.w); v[7] = bf16_hi((uint32_t)a.w);
        w[0] = bf16_lo((uint32_t)b.x); w[1] = bf16_hi((uint32_t)b.x); w[2] = bf16_lo((uint32_t)b.y); w[3] = bf16_hi((uint32_t)b.y);
        w[4] = bf16_lo((uint32_t)b.z); w[5] = bf16_hi((uint32_t)b.z); w[6] = bf16_lo((uint32_t)b.w); w[7] = bf16_hi((uint32_t)b.w);
        swiglu8(v, w, hround);
    } else {
        const v4f a0 = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
        const v4f a1 = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p) + 1);
        const v4f b0 = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p2));
        const v4f b1 = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p2) + 1);
        const float w[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
        v[0] = a0.x; v[1] = a0.y; v[2] = a0.z; v[3] = a0.w; v[4] = a1.x; v[5] = a1.y; v[6] = a1.z; v[7] = a1.w;
        swiglu8(v, w, hround);
    }
}

// Element offset of chunk c.  Contiguous rows (ld == K) need no division.
template <bool CONTIG>
__device__ __forceinline__ int64_t chunk_offset(uint32_t c, uint32_t cpr, int64_t ld) {
    if constexpr (CONTIG) {
        return (int64_t)c * 8;
    } else {
        uint32_t row = c / cpr;
        return (int64_t)row * ld + (int64_t)(c - row * cpr) * 8;
    }
}

// ---- in-wavefront rotation, 32 <= B <= 512 ------------------------------------------

// fl(1/sqrt(2^LOG2B)) as fp32 bits: sqrt(2)/2 = 0x3F3504F3 scaled by a power of two.
__host__ __device__ constexpr uint32_t norm_bits(int log2b) {
    return (log2b & 1) ? (0x3F3504F3u - ((uint32_t)((log2b - 1) / 2) << 23))
                       : (0x3F800000u - ((uint32_t)(log2b / 2) << 23));
}

// Quantize the lane's 8 values (quad = one group) and store codes + scale.
// Chunk kc of row `row`.
__device__ __forceinline__ void quant_store(const float (&y)[8], uint32_t row, uint32_t kc, uint32_t lane,
                                            const RowArgs& a) {
    uint32_t sb = e8m0_from_amax(quad_max(absmax8(y)));
    uint32_t w = encode8_e2m1(y, sb);
    if (a.stages == 0) {
        uint32_t c = row * a.cpr + kc;
        __builtin_nontemporal_store(w, &a.codes[c]);
        if ((lane & 3) == 0) *(&a.scales[c >> 2]) = (uint8_t)sb;
    } else {
        __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(a.codes) +
                                                                   tiled_code_offset(row, kc, a.stages)));
        if ((lane & 3) == 0) *(a.scales + tiled_scale_offset(row, kc, a.sstages)) = (uint8_t)sb;
    }
}

// ---- block statistics (Sec. 4.1, 4.2, Appendix "Rotation Comparison") ----------------------
// For the lane's 8 (rotated) values, quad = one 32-element block: the block-wise scale max|y|, the
// block's MXFP4 quantization loss sum (y - deq(q(y)))^2 (fp32; each difference is exact, the
// squares and the 32-term sum round), and per threshold the number of values with |y| above it.
//
// Counting costs one vector instruction per value and threshold: the comparison writes a lane mask to
// scalar registers, and the scalar unit, which has nothing else to do in this kernel, counts its bits
// and keeps the wavefront's running sums (`cnt`, wavefront-uniform; a wavefront meets fewer than 2^32
// values per launch).  Per-lane counters cost a second vector instruction per value and threshold on a
// kernel whose vector units are the busiest part.
//
// The per-block outputs of a wavefront's 16 blocks sit in lanes 0, 4, 8, ...; stored from there they are
// 16 separate 4-byte accesses.  One lane permute brings them to lanes 0..15, which store 64 contiguous
// bytes.  gidx0 = block index of the wavefront's first chunk; `live` = this lane's chunk exists.
__device__ __forceinline__ float gather_quads(float v, uint32_t lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((int)((lane & 15u) << 4), __builtin_bit_cast(int, v)));
}
__device__ __forceinline__ void stats_chunk(const float (&y)[8], uint32_t gidx0, bool live, uint32_t lane,
                                            const RowArgs& a, uint32_t (&cnt)[8]) {
    typedef float f2 __attribute__((ext_vector_type(2)));
    const float am = quad_max(absmax8(y));
    const uint32_t sb = e8m0_from_amax(am);
    const uint32_t w = encode8_e2m1_signed_zero(y, sb);      // decoded again below: the sign of a zero does not matter
    const float sc = as_f32(sb ? sb << 23 : 0x00400000u);   // 2^(sb - 127); scale byte 0 is the subnormal 2^-127
    float e2 = 0.0f;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        f2 d;   // the two codes of byte p as fp32 (scale 1); value * 2^(sb - 127) is exact, and so is y - that
        if (p == 0) d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, 1.0f, 0);
        if (p == 1) d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, 1.0f, 1);
        if (p == 2) d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, 1.0f, 2);
        if (p == 3) d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, 1.0f, 3);
        const float e0 = __builtin_fmaf(-d.x, sc, y[2 * p]), e1 = __builtin_fmaf(-d.y, sc, y[2 * p + 1]);
        e2 = __builtin_fmaf(e0, e0, e2);
        e2 = __builtin_fmaf(e1, e1, e2);
    }
    e2 = quad_sum(e2);
    // lane j < 16 takes over block j of the wavefront (held by lanes 4 j .. 4 j + 3) and stores it
    const bool blive = __builtin_amdgcn_ds_bpermute((int)((lane & 15u) << 4), (int)live) != 0;
    const bool st = lane < 16u && blive;
    if (a.amax) {   // uniform
        const float g = gather_quads(am, lane);
        if (st) a.amax[gidx0 + lane] = g;
    }
    if (a.sqerr) {
        const float g = gather_quads(e2, lane);
        if (st) a.sqerr[gidx0 + lane] = g;
    }
    if (a.sqerr_bfp4) {   // uniform
        // The FP16-scale counterpart (Sec. 3, 4.1): scale s = half(max / 6), codes = E2M1 rounding of
        // the correctly rounded quotient y / s, loss against code value * s (an exact product).
        const float s = (float)(_Float16)fminf(am / 6.0f, 65504.0f);
        float r[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = (s > 0.0f) ? y[i] / s : 0.0f;
        const uint32_t wb = encode8_e2m1_signed_zero(r, 127u);
        float eb = 0.0f;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            f2 d;
            if (p == 0) d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(wb, 1.0f, 0);
            if (p == 1) d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(wb, 1.0f, 1);
            if (p == 2) d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(wb, 1.0f, 2);
            if (p == 3) d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(wb, 1.0f, 3);
            const float e0 = __builtin_fmaf(-d.x, s, y[2 * p]), e1 = __builtin_fmaf(-d.y, s, y[2 * p + 1]);
            eb = __builtin_fmaf(e0, e0, eb);
            eb = __builtin_fmaf(e1, e1, eb);
        }
        eb = quad_sum(eb);
        const float g = gather_quads(eb, lane);
        if (st) a.sqerr_bfp4[gidx0 + lane] = g;
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        if (t < (int)a.nt) {   // uniform
            const float th = a.th[t];
            // a lane without a chunk carries a copy of the last one: its comparisons are masked out
            const float lim = live ? th : __builtin_inff();
#pragma unroll
            for (int i = 0; i < 8; ++i)
                cnt[t] += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(fabsf(y[i]) > lim));
        }
    }
}

// The wavefront's sums go to LDS (`red`: 8 words, zeroed by the caller before a barrier) through one lane,
// then one lane per threshold adds the workgroup's sum to the global counter.
__device__ __forceinline__ void stats_flush(const uint32_t (&cnt)[8], uint32_t* red, const RowArgs& a) {
    if ((threadIdx.x & 63u) == 0) {
#pragma unroll
        for (int t = 0; t < 8; ++t)
            if (t < (int)a.nt && cnt[t]) atomicAdd(&red[t], cnt[t]);
    }
    __syncthreads();
    if (threadIdx.x < a.nt && red[threadIdx.x]) atomicAdd(&a.counts[threadIdx.x], (unsigned long long)red[threadIdx.x]);
}

// One chunk per lane per step, U steps in flight (the launcher uses U = 1).  LOG2B = 0 means "no rotation":
// the quantizer alone, or (MODE_ROTATE with a producer) the gated activation alone, stored to y.
template <int LOG2B, bool IN_BF16, int MODE, bool OUT_BF16, bool CONTIG, int U, bool PROD>
__global__ void __launch_bounds__(256) k_rowwise(RowArgs a) {
    const uint32_t lane = threadIdx.x & 63;
    constexpr bool ROT = MODE != MODE_QUANT && LOG2B > 0;   // LOG2B = 0 with MODE_ROTATE: the producer alone
    __shared__ uint32_t red[8];
    uint32_t cnt[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (MODE == MODE_STATS) {
        if (threadIdx.x < 8) red[threadIdx.x] = 0;
        __syncthreads();
    }
    constexpr uint32_t inwave_bits = (LOG2B >= 3) ? ((1u << (LOG2B - 3)) - 1u) : 0u;
    const float sigma = (__builtin_popcount(lane & inwave_bits) & 1) ? -1.0f : 1.0f;
    const float cs = as_f32(norm_bits(LOG2B)) * sigma;
    const uint32_t step = gridDim.x * 256u * U;
    uint32_t sm[U][8];
    const bool presigned = ROT && a.signs && a.sign_fixed;   // uniform
    if (presigned) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            sign_masks(sm[u], a.signs + (size_t)((blockIdx.x * 256u * U + u * 256u + threadIdx.x) % a.cpr) * 8);
    }
    // `bb` is uniform over the workgroup and nothing below branches on the lane: chunks past
    // the end re-read the last chunk (clamped index) and only their stores are masked, so
    // every lane exchange sees a full wavefront.
    for (uint32_t bb = blockIdx.x * 256u * U; bb < a.nchunks; bb += step) {
        float v[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t c = min(bb + u * 256u + threadIdx.x, a.nchunks - 1u);
            const char* p = (const char*)a.x + chunk_offset<CONTIG>(c, a.cpr, a.ldx) * (IN_BF16 ? 2 : 4);
            const char* p2 = PROD ? (const char*)a.x2 + chunk_offset<CONTIG>(c, a.cpr, a.ldx2) * (IN_BF16 ? 2 : 4) : nullptr;
            load_input<IN_BF16, PROD>(p, p2, a.hround != 0, v[u]);
            if constexpr (ROT) {
                if (presigned) {
                    flip(v[u], sm[u]);
                } else if (a.signs) {   // uniform
                    uint32_t kc;
                    if ((a.cpr & 63u) == 0) {   // a wavefront's 64 chunks lie in one row: scalar modulo
                        const uint32_t cb = __builtin_amdgcn_readfirstlane(c);
                        kc = cb % a.cpr + (c - cb);
                    } else {
                        kc = c % a.cpr;
                    }
                    apply_signs(v[u], a.signs + (size_t)kc * 8);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = bb + u * 256u + threadIdx.x;
            const bool live = c < a.nchunks;
            if constexpr (ROT) {
                wht_inwave<LOG2B>(v[u], lane);
#pragma unroll
                for (int i = 0; i < 8; ++i) v[u][i] *= cs;
            }
            if constexpr (MODE == MODE_ROTATE) {
                if (live) {
                    char* p = (char*)a.y + chunk_offset<CONTIG>(c, a.cpr, a.ldy) * (OUT_BF16 ? 2 : 4);
                    // (a quad's four chunks are live together: the chunk count is a multiple of 4)
                    if constexpr (OUT_BF16) store_chunk<true>(p, v[u]);
                    else store_chunk_f32_quad(p, v[u], lane);
                }
            } else if constexpr (MODE == MODE_STATS) {
                stats_chunk(v[u], (c - lane) >> 2, live, lane, a, cnt);
            } else {
                uint32_t sb = e8m0_from_amax(quad_max(absmax8(v[u])));
                uint32_t w = encode8_e2m1(v[u], sb);
                if (a.stages == 0) {
                    if (live) {
                        __builtin_nontemporal_store(w, &a.codes[c]);
                        if ((lane & 3) == 0) *(&a.scales[c >> 2]) = (uint8_t)sb;
                    }
                } else if ((a.cpr & 63u) == 0) {
                    // K % 512 == 0: the 64 chunks of a wavefront lie in one row and one scale
                    // superstage, so the row arithmetic is scalar and a lane adds a constant
                    const uint32_t cb = __builtin_amdgcn_readfirstlane(c);       // lane 0's chunk
                    const uint32_t row = cb / a.cpr, kc0 = cb - row * a.cpr;     // kc0 % 64 == 0
                    uint8_t* cbase = reinterpret_cast<uint8_t*>(a.codes) + tiled_code_offset(row, kc0, a.stages);
                    uint8_t* sbase = a.scales + tiled_scale_offset(row, kc0, a.sstages);
                    if (live) {
                        __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(cbase + (lane >> 4) * 4096u + (lane & 15u) * 4u));
                        if ((lane & 3) == 0) *(sbase + (lane >> 2)) = (uint8_t)sb;
                    }
                } else if (live) {
                    const uint32_t row = c / a.cpr, kc = c - row * a.cpr;
                    __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(a.codes) +
                                                                               tiled_code_offset(row, kc, a.stages)));
                    if ((lane & 3) == 0) *(a.scales + tiled_scale_offset(row, kc, a.sstages)) = (uint8_t)sb;
                }
            }
        }
    }
    if constexpr (MODE == MODE_STATS) {
        if (a.counts) stats_flush(cnt, red, a);   // uniform
    }
}

// Quantize / fused rotate+quantize into the tiled layout, B <= 128 and K % 128 == 0.  In that
// layout 128 contiguous bytes of codes are one stage (128 elements) of TWO rows, so the
// row-wise mapping above would write half cache lines.  Here a wavefront takes 4 rows x one
// stage: lane l holds chunk (l & 15) of row 4 rq + (l >> 4), reads 4 x 256 contiguous bytes and
// writes 256 contiguous bytes of codes (two whole lines).  Every address is a wavefront-uniform
// base plus a per-lane constant.  Rotation blocks of up to 16 chunks stay inside one row's lanes.
template <int LOG2B, bool IN_BF16, int MODE, bool PROD>
__global__ void __launch_bounds__(256) k_rowwise_t4(RowArgs a, uint32_t rows, uint32_t nitems) {
    static_assert(LOG2B == 0 || (LOG2B >= 3 && LOG2B <= 7), "a rotation block must fit 16 lanes");
    constexpr int ES = IN_BF16 ? 2 : 4;
    const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr uint32_t inwave_bits = (LOG2B >= 3) ? ((1u << (LOG2B - 3)) - 1u) : 0u;
    const float sigma = (__builtin_popcount(lane & inwave_bits) & 1) ? -1.0f : 1.0f;
    const float cs = as_f32(norm_bits(LOG2B)) * sigma;
    const uint32_t spr = a.cpr >> 4;                                   // stages per row
    const uint32_t lrow = lane >> 4;
    uint32_t sm[8];
    const bool presigned = MODE != MODE_QUANT && a.signs && a.sign_fixed;   // uniform
    if (presigned) sign_masks(sm, a.signs + ((size_t)((blockIdx.x * 4u + wave) % spr) * 16u + (lane & 15u)) * 8);
    // Every address is a wavefront-uniform base plus a per-lane constant (the host checked that
    // 4 rows of pitch fit 32 bits): the loop body spends no vector instruction on addresses.
    const uint32_t in_lane = lrow * (uint32_t)a.ldx * ES + (lane & 15u) * (8u * ES);
    const uint32_t in_lane2 = PROD ? lrow * (uint32_t)a.ldx2 * ES + (lane & 15u) * (8u * ES) : 0u;
    const uint32_t step = gridDim.x * 4u;
    for (uint32_t it = blockIdx.x * 4u + wave; it < nitems; it += step) {
        const uint32_t rq = it / spr, st = it - rq * spr;              // scalar
        const uint32_t row0 = rq * 4u;
        const char* rowbase = (const char*)a.x + ((uint64_t)row0 * (uint64_t)a.ldx + (uint64_t)st * 128u) * ES;   // scalar
        const char* p = rowbase + in_lane;
        const char* p2 = nullptr;
        if constexpr (PROD)
            p2 = (const char*)a.x2 + ((uint64_t)row0 * (uint64_t)a.ldx2 + (uint64_t)st * 128u) * ES + in_lane2;
        if (row0 + 4u > rows) {   // uniform: M % 4 != 0, last item of a column; rows past the end
                                  // re-read the last row, their stores are masked below
            const uint32_t rrow = min(row0 + lrow, rows - 1u);
            p = (const char*)a.x + ((uint64_t)rrow * (uint64_t)a.ldx + (uint64_t)st * 128u + (lane & 15u) * 8u) * ES;
            if constexpr (PROD)
                p2 = (const char*)a.x2 + ((uint64_t)rrow * (uint64_t)a.ldx2 + (uint64_t)st * 128u + (lane & 15u) * 8u) * ES;
        }
        float v[8];
        load_input<IN_BF16, PROD>(p, p2, a.hround != 0, v);
        if constexpr (MODE != MODE_QUANT) {
            if (presigned) flip(v, sm);
            else if (a.signs) apply_signs(v, a.signs + ((size_t)st * 16u + (lane & 15u)) * 8);
            wht_inwave<LOG2B>(v, lane);
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] *= cs;
        }
        const uint32_t sb = e8m0_from_amax(quad_max(absmax8(v)));
        const uint32_t w = encode8_e2m1(v, sb);
        uint8_t* cbase = reinterpret_cast<uint8_t*>(a.codes) + ((uint64_t)(row0 >> 6) * a.stages + st) * 4096u + (row0 & 63u) * 64u;
        uint8_t* sbase = a.scales + ((uint64_t)(row0 >> 6) * a.sstages + (st >> 2)) * 1024u + (row0 & 63u) * 16u + (st & 3u) * 4u;
        if (row0 + lrow < rows) {
            __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(cbase + lane * 4u));
            if ((lane & 3) == 0) *(sbase + lrow * 16u + ((lane >> 2) & 3u)) = (uint8_t)sb;
        }
    }
}

// ---- LDS-staged rotation, 1024 <= B <= 16384 (includes the global, full-K rotation) ----
//
// One workgroup of NT = min(256, B/8) lanes transforms one B-block of one row.  Each
// lane holds CH = B/(8*NT) chunks.  Stages h < 512 run as above; the remaining
// R = log2(B) - 9 stages (h = 512 ... B/2, still ascending) run as one radix-2^R pass
// over LDS: a lane gathers the 2^R elements {g + 512 j}, does the R stages in registers
// and scatters them back.  Then every lane re-reads its own chunks and finishes.
template <int LOG2B, bool IN_BF16, int MODE, bool OUT_BF16, bool PROD>
__global__ void __launch_bounds__(256) k_rowwise_lds(RowArgs a, uint32_t blocks_per_row, uint32_t nblocks) {
    constexpr int B = 1 << LOG2B;
    constexpr int NT = (B / 8 < 256) ? B / 8 : 256;
    constexpr int CH = B / 8 / NT;
    constexpr int R = LOG2B - 9;
    constexpr int RADIX = 1 << R;
    constexpr int GROUPS_PER_LANE = 512 / NT;
    extern __shared__ float lds[];   // B floats

    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const float sigma = (__builtin_popcount(lane) & 1) ? -1.0f : 1.0f;
    __shared__ uint32_t red[8];
    uint32_t cnt[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (MODE == MODE_STATS) {
        if (tid < 8) red[tid] = 0;    // barriers follow below before anyone adds
    }
    // One block per pass; the launcher gives every block its own workgroup except for the
    // statistics, where fewer workgroups mean fewer atomics on the counters.
    for (uint32_t bid = blockIdx.x; bid < nblocks; bid += gridDim.x) {
        const uint32_t row = bid / blocks_per_row, blk = bid - row * blocks_per_row;
        const int64_t xoff = (int64_t)row * a.ldx + (int64_t)blk * B;
        const int64_t xoff2 = PROD ? (int64_t)row * a.ldx2 + (int64_t)blk * B : 0;

#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float v[8];
            uint32_t q = c * NT + tid;   // chunk index inside the block
            load_input<IN_BF16, PROD>((const char*)a.x + (xoff + (int64_t)q * 8) * (IN_BF16 ? 2 : 4),
                                      PROD ? (const char*)a.x2 + (xoff2 + (int64_t)q * 8) * (IN_BF16 ? 2 : 4) : nullptr,
                                      a.hround != 0, v);
            if (a.signs) apply_signs(v, a.signs + ((size_t)blk * B + (size_t)q * 8));
            wht_inwave<9>(v, lane);
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] *= sigma;   // exact: back to the true sign
            float4* dst = reinterpret_cast<float4*>(lds + q * 8);
            dst[0] = make_float4(v[0], v[1], v[2], v[3]);
            dst[1] = make_float4(v[4], v[5], v[6], v[7]);
        }
        __syncthreads();
#pragma unroll
        for (int gi = 0; gi < GROUPS_PER_LANE; ++gi) {
            uint32_t g = gi * NT + tid;   // 0 .. 511
            float r[RADIX];
#pragma unroll
            for (int j = 0; j < RADIX; ++j) r[j] = lds[g + 512 * j];
#pragma unroll
            for (int h = 1; h < RADIX; h *= 2) {
#pragma unroll
                for (int j = 0; j < RADIX; ++j) {
                    if ((j & h) == 0) {
                        float p = r[j], m = r[j + h];
                        r[j] = p + m;
                        r[j + h] = p - m;
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < RADIX; ++j) lds[g + 512 * j] = r[j];
        }
        __syncthreads();
        const float cn = as_f32(norm_bits(LOG2B));
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            uint32_t q = c * NT + tid;
            const float4* src = reinterpret_cast<const float4*>(lds + q * 8);
            float4 lo = src[0], hi = src[1];
            float y[8] = {lo.x * cn, lo.y * cn, lo.z * cn, lo.w * cn, hi.x * cn, hi.y * cn, hi.z * cn, hi.w * cn};
            if constexpr (MODE == MODE_ROTATE) {
                int64_t yoff = (int64_t)row * a.ldy + (int64_t)blk * B + (int64_t)q * 8;
                if constexpr (OUT_BF16) store_chunk<true>((char*)a.y + yoff * 2, y);
                else store_chunk_f32_quad((char*)a.y + yoff * 4, y, lane);
            } else if constexpr (MODE == MODE_STATS) {
                stats_chunk(y, (row * a.cpr + blk * (B / 8) + q - lane) >> 2, true, lane, a, cnt);
            } else {
                quant_store(y, row, blk * (B / 8) + q, lane, a);
            }
        }
        __syncthreads();   // the next pass overwrites the LDS this pass has just read
    }
    if constexpr (MODE == MODE_STATS) {
        if (a.counts) stats_flush(cnt, red, a);   // uniform
    }
}

// ---- host side ---------------------------------------------------------------------

// Workgroups per compute unit of a statistics launch: each ends with up to 8 atomics on the caller's counters.
#ifndef BRQ_STATS_WGS_PER_CU
#define BRQ_STATS_WGS_PER_CU 8
#endif

// Workgroups of a streaming launch.  Measured on X 16384 x 8192 (bf16, B = 32): one chunk in
// flight per lane and many short-lived workgroups beat a persistent grid (8 per CU, two
// chunks in flight: 63 us; 64 per CU, one chunk: 55 us): the dispatcher keeps every CU topped up
// and the loads of a finished workgroup's successor overlap the arithmetic of its neighbours.
// Each workgroup still makes about 3 passes so that small inputs do not pay for launching
// thousands of workgroups (1 pass: 15 % slower; 2, 4 and 8 passes: 1 - 4 % slower than 3, on 32 to 340 MB).
static int rowwise_grid(uint32_t nchunks, int U, int cus) {
    const uint32_t need = (nchunks + 256u * U - 1) / (256u * U);
    uint32_t grid = need / 3;
    const uint32_t lo = (uint32_t)cus * 8, hi = (uint32_t)cus * 64;
    if (grid < lo) grid = lo;
    if (grid > hi) grid = hi;
    return (int)(need < grid ? need : grid);
}

// Signed rotations: round `grid` down to a multiple of period / gcd(period, per_wg), so that one
// grid-stride pass (grid * per_wg work items) is a whole number of rows' worth of columns and
// every lane meets the same column, hence the same signs, in every pass.  Returns 1 if the grid
// could be sized that way (it is left alone, and 0 returned, when that would shrink it by more
// than half).
static uint32_t fix_columns(int& grid, uint32_t period, uint32_t per_wg) {
    uint32_t x = period, y = per_wg;
    while (y) { uint32_t t = x % y; x = y; y = t; }
    const uint32_t unit = period / x;
    const uint32_t g = (uint32_t)grid / unit * unit;
    if (g == 0 || g * 2 < (uint32_t)grid) return 0;
    grid = (int)g;
    return 1;
}

template <int LOG2B, bool IN_BF16, int MODE, bool OUT_BF16, bool PROD = false>
static hipError_t launch_inwave(const RowArgs& a, bool contig, hipStream_t s) {
    int cus = 0;
    if (hipError_t e = device_cus(&cus); e != hipSuccess) return e;
    if constexpr ((MODE == MODE_QUANT || MODE == MODE_FUSED) && LOG2B <= 7) {
        if (a.stages != 0 && (a.cpr & 15u) == 0 && a.ldx * (IN_BF16 ? 2 : 4) * 4 < (int64_t(1) << 32) &&
            (!PROD || a.ldx2 * (IN_BF16 ? 2 : 4) * 4 < (int64_t(1) << 32))) {
            const uint32_t rows = a.nchunks / a.cpr, nitems = ((rows + 3u) / 4u) * (a.cpr >> 4);
            int grid = rowwise_grid(nitems * 64u, 1, cus);
            RowArgs b = a;
            b.sign_fixed = a.signs ? fix_columns(grid, a.cpr >> 4, 4) : 0;
            hipLaunchKernelGGL((k_rowwise_t4<LOG2B, IN_BF16, MODE, PROD>), dim3(grid), dim3(256), 0, s, b, rows, nitems);
            return hipGetLastError();
        }
    }
    constexpr int U = 1;
    int grid = rowwise_grid(a.nchunks, U, cus);
    if constexpr (MODE == MODE_STATS) {   // fewer, longer-lived workgroups: each ends with atomics on the counters
        const int cap = cus * BRQ_STATS_WGS_PER_CU;
        if (grid > cap) grid = cap;
    }
    RowArgs b = a;
    b.sign_fixed = (a.signs && MODE != MODE_QUANT && LOG2B > 0) ? fix_columns(grid, a.cpr, 256 * U) : 0;
    if (contig)
        hipLaunchKernelGGL((k_rowwise<LOG2B, IN_BF16, MODE, OUT_BF16, true, U, PROD>), dim3(grid), dim3(256), 0, s, b);
    else
        hipLaunchKernelGGL((k_rowwise<LOG2B, IN_BF16, MODE, OUT_BF16, false, U, PROD>), dim3(grid), dim3(256), 0, s, b);
    return hipGetLastError();
}

template <int LOG2B, bool IN_BF16, int MODE, bool OUT_BF16, bool PROD = false>
static hipError_t launch_lds(const RowArgs& a, int64_t M, int64_t K, hipStream_t s) {
    constexpr int B = 1 << LOG2B;
    constexpr int NT = (B / 8 < 256) ? B / 8 : 256;
    uint32_t bpr = (uint32_t)(K / B);
    const uint32_t nblocks = (uint32_t)(M * bpr);
    uint32_t grid = nblocks;
    if (MODE == MODE_STATS) {
        int cus = 0;
        if (hipError_t e = device_cus(&cus); e != hipSuccess) return e;
        const uint32_t cap = (uint32_t)cus * (uint32_t)BRQ_STATS_WGS_PER_CU;
        if (grid > cap) grid = cap;
    }
    hipLaunchKernelGGL((k_rowwise_lds<LOG2B, IN_BF16, MODE, OUT_BF16, PROD>), dim3(grid), dim3(NT),
                       B * sizeof(float), s, a, bpr, nblocks);
    return hipGetLastError();
}

template <bool IN_BF16, int MODE, bool OUT_BF16, bool PROD = false>
static hipError_t dispatch_b(int log2b, const RowArgs& a, bool contig, int64_t M, int64_t K, hipStream_t s) {
    switch (log2b) {
        case 3: return launch_inwave<3, IN_BF16, MODE, OUT_BF16, PROD>(a, contig, s);
        case 4: return launch_inwave<4, IN_BF16, MODE, OUT_BF16, PROD>(a, contig, s);
        case 5: return launch_inwave<5, IN_BF16, MODE, OUT_BF16, PROD>(a, contig, s);
        case 6: return launch_inwave<6, IN_BF16, MODE, OUT_BF16, PROD>(a, contig, s);
        case 7: return launch_inwave<7, IN_BF16, MODE, OUT_BF16, PROD>(a, contig, s);
        case 8: return launch_inwave<8, IN_BF16, MODE, OUT_BF16, PROD>(a, contig, s);
        case 9: return launch_inwave<9, IN_BF16, MODE, OUT_BF16, PROD>(a, contig, s);
        case 10: return launch_lds<10, IN_BF16, MODE, OUT_BF16, PROD>(a, M, K, s);
        case 11: return launch_lds<11, IN_BF16, MODE, OUT_BF16, PROD>(a, M, K, s);
        case 12: return launch_lds<12, IN_BF16, MODE, OUT_BF16, PROD>(a, M, K, s);
        case 13: return launch_lds<13, IN_BF16, MODE, OUT_BF16, PROD>(a, M, K, s);
        case 14: return launch_lds<14, IN_BF16, MODE, OUT_BF16, PROD>(a, M, K, s);
        default: return hipErrorInvalidValue;
    }
}

// Tiled layout, K not a multiple of 512: the groups between K and the next multiple of 512 are
// written as zeros (16 zero code bytes, scale byte 0) for every row, so that the persistent
// product kernel can run whole 512-element superstages over tiled operands.  One lane per
// padding group.
__global__ void __launch_bounds__(256) k_zero_kpad(uint8_t* __restrict__ codes, uint8_t* __restrict__ scales,
                                                   uint32_t rows, uint32_t g0, uint32_t gpad, uint32_t stages,
                                                   uint32_t sstages) {
    const uint64_t n = (uint64_t)rows * gpad;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256) {
        const uint32_t row = (uint32_t)(i / gpad), g = g0 + (uint32_t)(i - (uint64_t)row * gpad);
        *reinterpret_cast<v4i*>(codes + tiled_code_offset(row, g * 4, stages)) = v4i{0, 0, 0, 0};
        scales[tiled_scale_offset(row, g * 4, sstages)] = 0;
    }
}

hipError_t launch_zero_kpad(uint8_t* codes, uint8_t* scales, int64_t M, int64_t K, hipStream_t s) {
    const int64_t Kp = (K + 511) / 512 * 512;
    if (Kp == K || M == 0) return hipSuccess;
    const uint32_t gpad = (uint32_t)((Kp - K) / 32);
    const int64_t want = (M * gpad + 255) / 256;
    hipLaunchKernelGGL(k_zero_kpad, dim3((uint32_t)(want < 4096 ? want : 4096)), dim3(256), 0, s, codes, scales,
                       (uint32_t)M, (uint32_t)(K / 32), gpad, (uint32_t)(Kp / 128), (uint32_t)(Kp / 512));
    return hipGetLastError();
}

// mode: RowMode; log2b: 0 for MODE_QUANT, else 3..14.  Arguments are already validated.
hipError_t launch_rowwise(int mode, int log2b, bool in_bf16, bool out_bf16, const void* x, int64_t M,
                          int64_t K, int64_t ldx, void* y, int64_t ldy, uint8_t* codes, uint8_t* scales,
                          bool tiled, const int8_t* signs, const Producer* prod, hipStream_t s, const StatsOut* stats) {
    RowArgs a;
    a.amax = stats ? stats->amax : nullptr;
    a.sqerr = stats ? stats->sqerr : nullptr;
    a.sqerr_bfp4 = stats ? stats->sqerr_bfp4 : nullptr;
    a.counts = stats ? stats->counts : nullptr;
    a.nt = stats ? (uint32_t)stats->nt : 0u;
    for (int t = 0; t < 8; ++t) a.th[t] = (stats && t < stats->nt) ? stats->thresholds[t] : 0.0f;
    a.x2 = prod ? prod->up : nullptr;
    a.ldx2 = prod ? prod->ldu : 0;
    a.hround = (prod && prod->through_bf16) ? 1u : 0u;
    a.signs = signs;
    a.sign_fixed = 0;
    a.x = x; a.y = y; a.codes = reinterpret_cast<uint32_t*>(codes); a.scales = scales;
    a.ldx = ldx; a.ldy = ldy; a.cpr = (uint32_t)(K / 8); a.nchunks = (uint32_t)(M * (K / 8));
    const int64_t Kp = (K + 511) / 512 * 512;
    a.stages = tiled ? (uint32_t)(Kp / 128) : 0u;
    a.sstages = tiled ? (uint32_t)(Kp / 512) : 0u;
    bool contig = (ldx == K) && (mode != MODE_ROTATE || ldy == K) && (!prod || prod->ldu == K);
    if (tiled && Kp != K && mode != MODE_ROTATE) {
        hipError_t e = launch_zero_kpad(codes, scales, M, K, s);
        if (e != hipSuccess) return e;
    }
    if (mode == MODE_STATS) {   // log2b = 0: no rotation
        if (log2b == 0)
            return in_bf16 ? launch_inwave<0, true, MODE_STATS, false>(a, contig, s)
                           : launch_inwave<0, false, MODE_STATS, false>(a, contig, s);
        return in_bf16 ? dispatch_b<true, MODE_STATS, false>(log2b, a, contig, M, K, s)
                       : dispatch_b<false, MODE_STATS, false>(log2b, a, contig, M, K, s);
    }
    if (prod && mode == MODE_ROTATE) {   // the activation alone, written to y (log2b = 0)
        if (in_bf16) return out_bf16 ? launch_inwave<0, true, MODE_ROTATE, true, true>(a, contig, s)
                                     : launch_inwave<0, true, MODE_ROTATE, false, true>(a, contig, s);
        return out_bf16 ? launch_inwave<0, false, MODE_ROTATE, true, true>(a, contig, s)
                        : launch_inwave<0, false, MODE_ROTATE, false, true>(a, contig, s);
    }
    if (mode == MODE_ROTATE) {
        if (in_bf16) return out_bf16 ? dispatch_b<true, MODE_ROTATE, true>(log2b, a, contig, M, K, s)
                                     : dispatch_b<true, MODE_ROTATE, false>(log2b, a, contig, M, K, s);
        return out_bf16 ? dispatch_b<false, MODE_ROTATE, true>(log2b, a, contig, M, K, s)
                        : dispatch_b<false, MODE_ROTATE, false>(log2b, a, contig, M, K, s);
    }
    if (prod) {   // gated-activation producer in front of the quantizer / the fused step
        if (mode == MODE_QUANT)
            return in_bf16 ? launch_inwave<0, true, MODE_QUANT, false, true>(a, contig, s)
                           : launch_inwave<0, false, MODE_QUANT, false, true>(a, contig, s);
        return in_bf16 ? dispatch_b<true, MODE_FUSED, false, true>(log2b, a, contig, M, K, s)
                       : dispatch_b<false, MODE_FUSED, false, true>(log2b, a, contig, M, K, s);
    }
    if (mode == MODE_QUANT)
        return in_bf16 ? launch_inwave<0, true, MODE_QUANT, false>(a, contig, s)
                       : launch_inwave<0, false, MODE_QUANT, false>(a, contig, s);
    return in_bf16 ? dispatch_b<true, MODE_FUSED, false>(log2b, a, contig, M, K, s)
                   : dispatch_b<false, MODE_FUSED, false>(log2b, a, contig, M, K, s);
}

// ---- tiled -> row-major copy of a quantized operand (inspection and parity checks) ----
// One lane per 32-element group: its 16 code bytes and its scale byte.
__global__ void __launch_bounds__(256) k_to_rowmajor(const uint8_t* __restrict__ ct, const uint8_t* __restrict__ st,
                                                     uint32_t rows, uint32_t K, uint32_t stages, uint32_t sstages,
                                                     uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
    const uint32_t gpr = K / 32;                       // groups (16 code bytes, 1 scale byte) per row
    const uint64_t n = (uint64_t)rows * gpr;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256) {
        const uint32_t row = (uint32_t)(i / gpr), g = (uint32_t)(i - (uint64_t)row * gpr);
        const v4i c = *reinterpret_cast<const v4i*>(ct + tiled_code_offset(row, g * 4, stages));
        *reinterpret_cast<v4i*>(codes + i * 16) = c;
        scales[i] = st[tiled_scale_offset(row, g * 4, sstages)];
    }
}

hipError_t launch_to_rowmajor(const uint8_t* codes_t, const uint8_t* scales_t, int64_t rows, int64_t K,
                              uint8_t* codes, uint8_t* scales, hipStream_t s) {
    const int64_t Kp = (K + 511) / 512 * 512;
    const int64_t n = rows * (K / 32);
    const int64_t want = (n + 255) / 256;
    const int grid = (int)(want < 16384 ? want : 16384);
    hipLaunchKernelGGL(k_to_rowmajor, dim3(grid), dim3(256), 0, s, codes_t, scales_t, (uint32_t)rows, (uint32_t)K,
                       (uint32_t)(Kp / 128), (uint32_t)(Kp / 512), codes, scales);
    return hipGetLastError();
}

}  // namespace brq
