// W4A4 product on MXFP4 operands for gfx950 (Sec. 2 and Sec. 4.1 of the paper: the product
// the rotation leaves invariant, evaluated on E2M1 codes with E8M0 group scales).
//
// The contraction runs on CDNA4's block-scaled MFMA.  Operand layout of
// v_mfma_scale_f32_32x32x64_f8f6f4 with fp4 inputs: lane l supplies, for row (l & 31), the
// 32 consecutive K elements of group (l >> 5) as 16 packed bytes (low nibble first), and
// one E8M0 byte for exactly that group; accumulator register i of lane l is element
// (row 8*(i/4) + 4*(l>>5) + i%4, column l & 31).  The 16x16x128 form: row (l & 15), group
// (l >> 4); accumulator i is (row 4*(l>>4) + i, column l & 15).
#include <type_traits>
#include "brq_device.h"
#include "brq_launch.h"

namespace brq {

template <int V>
struct IC { static constexpr int value = V; };

// Addressing of one row of a quantized operand, valid for both layouts: the 16 code bytes of
// group g sit at codes + (g >> 2) * cstep + (g & 3) * 16 and its scale at scales + (g >> 4) * sstep
// + (g & 15), with (cstep, sstep) = (64, 16) for row-major rows and (4096, 1024) for the tiled
// layout (64-row slabs; 64 code bytes per row and stage, 16 scale bytes per row and superstage).
struct RowView {
    const uint8_t* codes;
    const uint8_t* scales;
    uint32_t cstep, sstep;
    __device__ __forceinline__ RowView(const uint8_t* c, const uint8_t* s, bool tiled, int64_t row, int K) {
        if (tiled) {
            const int64_t Kp = ((int64_t)K + 511) / 512 * 512;
            codes = c + (row >> 6) * (Kp / 128) * 4096 + (row & 63) * 64;
            scales = s + (row >> 6) * (Kp / 512) * 1024 + (row & 63) * 16;
            cstep = 4096; sstep = 1024;
        } else {
            codes = c + row * (K / 2);
            scales = s + row * (K / 32);
            cstep = 64; sstep = 16;
        }
    }
    __device__ __forceinline__ v4i group(int g) const {
        return *reinterpret_cast<const v4i*>(codes + (int64_t)(g >> 2) * cstep + (g & 3) * 16);
    }
    __device__ __forceinline__ int scale(int g) const { return scales[(int64_t)(g >> 4) * sstep + (g & 15)]; }
};

__device__ __forceinline__ void store_out(void* y, bool out_bf16, int64_t idx, float v) {
    if (out_bf16) reinterpret_cast<uint16_t*>(y)[idx] = (uint16_t)f32_to_bf16_bits(v);
    else reinterpret_cast<float*>(y)[idx] = v;
}

// ---- general shapes: one 32x32 output tile per wavefront, operands straight from global ----
__global__ void __launch_bounds__(256) k_gemm_direct(const uint8_t* __restrict__ aq, const uint8_t* __restrict__ as,
                                                     int a_tiled, const uint8_t* __restrict__ wq,
                                                     const uint8_t* __restrict__ ws, int w_tiled, int M, int N, int K,
                                                     void* __restrict__ y, int out_bf16, int64_t ldy) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m0 = blockIdx.y * 64 + (wave >> 1) * 32, n0 = blockIdx.x * 64 + (wave & 1) * 32;
    if (m0 >= M || n0 >= N) return;   // whole wavefront leaves together
    const int r = lane & 31, h = lane >> 5;
    const int64_t ra = min(m0 + r, M - 1), rw = min(n0 + r, N - 1);   // clamp: rows past the edge are computed, not stored
    const int groups = K / 32;
    const RowView va(aq, as, a_tiled != 0, ra, K), vw(wq, ws, w_tiled != 0, rw, K);
    v16f acc = {};
    for (int g0 = 0; g0 < groups; g0 += 2) {
        int g = g0 + h;
        v8i a = {}, b = {};
        int sca = 0, scb = 0;
        if (g < groups) {   // odd group count: the last step's second half contributes zeros
            v4i ta = va.group(g);
            v4i tb = vw.group(g);
            a[0] = ta[0]; a[1] = ta[1]; a[2] = ta[2]; a[3] = ta[3];
            b[0] = tb[0]; b[1] = tb[1]; b[2] = tb[2]; b[3] = tb[3];
            sca = va.scale(g); scb = vw.scale(g);
        }
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc, 4, 4, 0, sca, 0, scb);
    }
    const int col = n0 + r;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        int row = m0 + 8 * (i / 4) + 4 * h + (i % 4);
        if (row < M && col < N) store_out(y, out_bf16, (int64_t)row * ldy + col, acc[i]);
    }
}

// ---- M <= 16 (decode): weight streaming, 16 output columns per workgroup -------------------
// Each of the 4 wavefronts takes every 4th 128-wide K step for the same 16 weight rows; the
// partial 16x16 tiles are summed through LDS in a fixed order.
__global__ void __launch_bounds__(256) k_gemm_skinny(const uint8_t* __restrict__ aq, const uint8_t* __restrict__ as,
                                                     int a_tiled, const uint8_t* __restrict__ wq,
                                                     const uint8_t* __restrict__ ws, int w_tiled, int M, int N, int K,
                                                     void* __restrict__ y, int out_bf16, int64_t ldy) {
    __shared__ float part[4][64][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, kq = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int groups = K / 32;
    const int64_t rw = min(n0 + r, N - 1);
    const bool arow = r < M;
    const RowView va(aq, as, a_tiled != 0, arow ? r : 0, K), vw(wq, ws, w_tiled != 0, rw, K);
    v4f acc = {};
    for (int g0 = wave * 4; g0 < groups; g0 += 16) {
        int g = g0 + kq;
        v8i a = {}, b = {};
        int sca = 0, scb = 0;
        if (g < groups) {
            v4i tb = vw.group(g);
            b[0] = tb[0]; b[1] = tb[1]; b[2] = tb[2]; b[3] = tb[3];
            scb = vw.scale(g);
            if (arow) {
                v4i ta = va.group(g);
                a[0] = ta[0]; a[1] = ta[1]; a[2] = ta[2]; a[3] = ta[3];
                sca = va.scale(g);
            }
        }
        acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc, 4, 4, 0, sca, 0, scb);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) part[wave][lane][i] = acc[i];
    __syncthreads();
    if (wave == 0) {
        const int col = n0 + r;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float s = ((part[0][lane][i] + part[1][lane][i]) + part[2][lane][i]) + part[3][lane][i];
            int row = 4 * kq + i;
            if (row < M && col < N) store_out(y, out_bf16, (int64_t)row * ldy + col, s);
        }
    }
}

// ---- M <= 128 (decode batches): weight streaming with the activations in LDS ----------------
// HBM-bound: every weight byte is read exactly once.  A wavefront owns its weight rows for the whole
// of K (no cross-wavefront reduction, fixed summation order) and streams them through registers,
// three 512-element superstages in rotation.  With several tiles of activation rows every wavefront
// would re-read all of A (M x K/2 bytes against its own weight bytes), so the 4 wavefronts of a
// workgroup share the activations: one superstage of A at a time goes into LDS by LDS-DMA (three
// buffers, one barrier per superstage), wavefront w bringing stage w.  The MFMA is the 32x32x64
// one, a wavefront per 32 weight rows and MT tiles of 32 activation rows: with the 16x16x128 form
// every wavefront reads all of A out of LDS for only 16 weight rows and the fragment reads bound the
// kernel (28 us at M = 64, 40 at M = 128 on the 28672 x 8192 decode shape, against 23 and 31 here);
// the persistent tiled kernel at these sizes has one 128 x 256 tile on fewer than half of the CUs,
// each with only its 4-stage ring of weights in flight (44 us), where 4 x N/128 wavefronts here
// each keep two superstages of their own rows in flight.
// Operand fragments (32x32x64: lane (r, h) = (lane & 31, lane >> 5) supplies 32 consecutive K
// elements of row r): within a 128-element stage (64 code bytes per row) lane half h owns bytes
// [32 h, 32 h + 32), MFMA step j of the stage takes bytes 32 h + 16 j, i.e. group 2 h + j of the
// stage, for both operands and both scales.  A in LDS: [stage][row][64 bytes] with the 16-byte
// chunks of row i XOR-swizzled by (i >> 2) & 3 (lanes r = 0..31 of one read then spread over all
// banks), scales [tile][64 rows][16 bytes].  Output: lane (r, h) holds D[8 q + 4 h + i][r] for
// weight row n0 + r, so the 32 lanes of a half store 32 consecutive columns of one output row.

// Weight register sets = LDS buffers of A; SETS - 1 superstages are in flight (4 sets measured no faster).
constexpr int SMALLM_SETS = 3;
constexpr int smallm_lds_bytes(int MT) { return SMALLM_SETS * (MT * 8192 + 4096); }

// TAIL = (K / 512) % SETS: the superstages left after the main loop, which takes them SETS at a time in
// one basic block (no load behind a branch: the compiler's count of the outstanding weight loads is
// then exact; with early exits inside the loop it falls back to waiting for all of them).
template <int MT, int TAIL>
__global__ void __launch_bounds__(256) k_gemm_smallm(const uint8_t* __restrict__ aq, const uint8_t* __restrict__ as,
                                                     int a_tiled, const uint8_t* __restrict__ wq,
                                                     const uint8_t* __restrict__ ws, int w_tiled, int M, int N, int K,
                                                     void* __restrict__ y, int out_bf16, int64_t ldy) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int STG = MT * 2048;                      // one stage of A codes: MT * 32 rows x 64 bytes
    constexpr int BUF = 4 * STG + 4096;                 // codes [4 stages][MT * 32 rows][64], then scales [4 tiles][64 rows][16]
    constexpr int NA = 2 * MT + 1;                      // LDS-DMA instructions per wavefront and superstage
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, h = lane >> 5;
    const int n0 = blockIdx.x * 128 + wave * 32;
    const int nss = (K + 511) / 512;                    // tiled operands are zero-padded to whole superstages
    const int64_t Kp = (int64_t)nss * 512;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    const RowView vw(wq, ws, w_tiled != 0, min(n0 + r, N - 1), K);

    const uint32_t a_cstep = a_tiled ? 4096u : 64u, a_sstep = a_tiled ? 1024u : 16u;
    auto row_off_c = [&](int row) -> uint32_t {
        row = min(row, M - 1);
        return a_tiled ? (uint32_t)((row >> 6) * (Kp / 128) * 4096 + (row & 63) * 64) : (uint32_t)((int64_t)row * (K / 2));
    };
    auto row_off_s = [&](int row) -> uint32_t {
        row = min(row, M - 1);
        return a_tiled ? (uint32_t)((row >> 6) * (Kp / 512) * 1024 + (row & 63) * 16) : (uint32_t)((int64_t)row * (K / 32));
    };
    // one DMA instruction = 16 rows x 64 bytes; lane i brings chunk (i & 3) ^ ((i >> 4) & 3) of row i >> 2
    uint32_t voc[2 * MT];
#pragma unroll
    for (int j = 0; j < 2 * MT; ++j)
        voc[j] = row_off_c(16 * j + (lane >> 2)) + (uint32_t)((lane & 3) ^ ((lane >> 4) & 3)) * 16u;
    // ... and one more the scale rows of 32-row tile `wave` (lanes 32..63 repeat them into the second half of
    // the tile's 1 KB slot; a wavefront without a tile of its own repeats row M - 1): every wavefront
    // issues the same number of loads, which the counted waits below rely on
    const uint32_t vos = row_off_s(32 * wave + r);
    // wavefront `wave` brings stage `wave` of the superstage
    auto dma_a = [&](int ss, uint32_t buf) {
        const uint8_t* cb = uniform_ptr(aq + (int64_t)(4 * ss + wave) * a_cstep);
        const uint32_t lb = lds0 + buf * BUF + (uint32_t)wave * STG;
#pragma unroll
        for (int j = 0; j < 2 * MT; ++j) {
            if (j == 0) dma16<0>(lb, cb, voc[0]);
            if (j == 1) dma16<1024>(lb, cb, voc[1]);
            if (j == 2) dma16<2048>(lb, cb, voc[j]);
            if (j == 3) dma16<3072>(lb, cb, voc[j]);
            if (j == 4) dma16<4096>(lb, cb, voc[j]);
            if (j == 5) dma16<5120>(lb, cb, voc[j]);
            if (j == 6) dma16<6144>(lb, cb, voc[j]);
            if (j == 7) dma16<7168>(lb, cb, voc[j]);
        }
        dma16<0>(lds0 + buf * BUF + 4 * STG + (uint32_t)wave * 1024, uniform_ptr(as + (int64_t)ss * a_sstep), vos);
    };
    // a superstage of this lane's weight row: per stage t its two steps (32 bytes at 32 h), and the 16 scale bytes.
    // Plain loads: one instruction takes half of every cache line it touches and the next one the other half,
    // and a streaming load does not leave the line in the cache for it (the weights would cross HBM twice).
    auto load_w = [&](int ss, v4i (&c)[8], v4i& sc) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                c[2 * t + j] = *reinterpret_cast<const v4i*>(vw.codes + (int64_t)(4 * ss + t) * vw.cstep + h * 32 + j * 16);
        sc = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(vw.scales + (int64_t)ss * vw.sstep));
    };
    v16f acc[MT];
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[j] = v16f{};
    const uint32_t sw = (uint32_t)(r >> 2) & 3u;
    // The 8 steps (stage t, half-step j) of a superstage, each over the MT row tiles: consecutive MFMAs go
    // to different accumulators, and the A fragments of step s + 1 are read while those of step s multiply.
    auto superstage = [&](uint32_t buf, const v4i (&c)[8], const v4i& sc) {
        const uint8_t* cb = lds + buf * BUF + r * 64;
        const uint8_t* sb = lds + buf * BUF + 4 * STG + r * 16;
        v4i asc[MT], af[2][MT];
#pragma unroll
        for (int jt = 0; jt < MT; ++jt) asc[jt] = *reinterpret_cast<const v4i*>(sb + jt * 1024);
        auto read_step = [&](int st, v4i (&f)[MT]) {
            const int t = st >> 1, j = st & 1;
#pragma unroll
            for (int jt = 0; jt < MT; ++jt)
                f[jt] = *reinterpret_cast<const v4i*>(cb + t * STG + jt * 2048 + (((uint32_t)(2 * h + j) ^ sw) << 4));
        };
        read_step(0, af[0]);
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            const int t = st >> 1, j = st & 1;
            if (st + 1 < 8) read_step(st + 1, af[(st + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);   // keeps the reads ahead of this step's MFMAs
            // group 4 t + 2 h + j of the superstage: byte 2 h + j of scale dword t
            const int scb = (int)(((uint32_t)sc[t] >> (16 * h + 8 * j)) & 0xffu);
            v8i b = {};
            b[0] = c[st][0]; b[1] = c[st][1]; b[2] = c[st][2]; b[3] = c[st][3];
#pragma unroll
            for (int jt = 0; jt < MT; ++jt) {
                v8i a = {};
                a[0] = af[st & 1][jt][0]; a[1] = af[st & 1][jt][1]; a[2] = af[st & 1][jt][2]; a[3] = af[st & 1][jt][3];
                const int sca = (int)(((uint32_t)asc[jt][t] >> (16 * h + 8 * j)) & 0xffu);
                acc[jt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[jt], 4, 4, 0, sca, 0, scb);
            }
        }
    };
    // D = SETS - 1 superstages ahead.  Issue order per wavefront: A(0), W(0), .., A(D - 1), W(D - 1); then turn
    // ss issues A(ss + D), W(ss + D) - A into the LDS buffer, W into the register set that turn ss - 1
    // consumed - and computes superstage ss.  Loads return in order: at the top of turn ss everything
    // younger than W(ss) is the (D - 1) x (NA + 9) loads of the superstages after it, so waiting until at
    // most that many are outstanding means A(ss) and W(ss) have landed while D - 1 superstages stay in
    // flight across the barrier.  Every turn of the main loop issues its loads, past the end of K those of
    // the last superstage once more (into a free buffer and register set, and out of the L2), so the turns
    // are all alike; the TAIL turns after it issue none.
    constexpr int SETS = SMALLM_SETS, D = SETS - 1;
    v4i c[SETS][8], s4[SETS];
#pragma unroll
    for (int i = 0; i < D; ++i) {
        dma_a(min(i, nss - 1), (uint32_t)i);
        load_w(min(i, nss - 1), c[i], s4[i]);
    }
    // k = the turn's register set and LDS buffer (superstage mod SETS), G = superstages in flight behind it
    auto turn = [&](auto Kc, auto Gc, auto Issue, int ss) {
        constexpr int k = decltype(Kc)::value, G = decltype(Gc)::value, kn = (k + D) % SETS;
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::"n"(G * (NA + 9)) : "memory");
        // The compiler counts only the weight loads it can see, not the LDS-DMA ones: where it first needs
        // W(ss) it waits until no more loads are outstanding than the weight loads it knows to be younger.
        // Asking for W(ss) here, before this turn's loads are issued, makes that count the 9 G of the
        // superstages in flight (which also asks for their A shares, fetched from the L2 long ago); asked
        // for after this turn's loads it would be 9 more, fewer than are really outstanding, and the oldest
        // superstage in flight would have to land first.
        asm volatile("" ::"v"(c[k][0]), "v"(c[k][1]), "v"(c[k][2]), "v"(c[k][3]), "v"(c[k][4]), "v"(c[k][5]), "v"(c[k][6]),
                     "v"(c[k][7]), "v"(s4[k]));
        // (scheduling fences: without them the compiler sinks the weight loads below the turn's MFMAs and
        // lifts the next turn's scale arithmetic, which needs the youngest load, up into this one)
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (decltype(Issue)::value) {
            const int nx = min(ss + D, nss - 1);
            dma_a(nx, (uint32_t)kn);
            load_w(nx, c[kn], s4[kn]);
        }
        __builtin_amdgcn_sched_barrier(0);
        superstage((uint32_t)k, c[k], s4[k]);
        __builtin_amdgcn_sched_barrier(0);
    };
    using Yes = std::true_type;
    using No = std::false_type;
    int ss = 0;
    for (; ss + SETS <= nss; ss += SETS) {
        turn(IC<0>{}, IC<D - 1>{}, Yes{}, ss);
        turn(IC<1>{}, IC<D - 1>{}, Yes{}, ss + 1);
        turn(IC<2>{}, IC<D - 1>{}, Yes{}, ss + 2);
        if constexpr (SETS > 3) turn(IC<3 % SETS>{}, IC<D - 1>{}, Yes{}, ss + 3);
    }
    // TAIL superstages are left; the loads of the D - 1 after superstage ss, real or repeated, are in flight
    if constexpr (TAIL >= 1) turn(IC<0>{}, IC<D - 1>{}, No{}, ss);
    if constexpr (TAIL >= 2) turn(IC<1>{}, IC<(D >= 2 ? D - 2 : 0)>{}, No{}, ss + 1);
    if constexpr (TAIL >= 3) turn(IC<2>{}, IC<(D >= 3 ? D - 3 : 0)>{}, No{}, ss + 2);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the repeated loads land before the LDS is released
    const int col = n0 + r;
#pragma unroll
    for (int jt = 0; jt < MT; ++jt)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = 32 * jt + 8 * q + 4 * h + i;
                if (row < M && col < N) store_out(y, out_bf16, (int64_t)row * ldy + col, acc[jt][4 * q + i]);
            }
}

// ---- M <= 16 with the online step inside (Sec. 4.3: the rotation R_4 and the quantizer in front of the
// quantized layer, here folded into the product's own prologue) ---------------------------------------
// Every workgroup first rotates (B = 32) and quantizes ALL of the activations, M <= 16 rows x K, into LDS -
// the same arithmetic as the row-wise kernels, a quad of lanes per 32-element group - in the layout the
// weight-streaming loop reads: codes [stage][16 rows][64 bytes] with the 16-byte chunks of row i XOR-swizzled
// by (i >> 2) & 3, scales [superstage][16 rows][16 bytes].  Then it streams its 128 weight rows exactly like
// k_gemm_smallm with one tile, without any barrier (the activations never change), so the result is bit
// for bit that of brq_mxfp4_gemm on the output of brq_rotate_quantize_fused.  The first superstages of
// weights are requested before the prologue and arrive under it.  What this saves is one small launch; what
// it costs is that every one of the N / 128 workgroups repeats the quantization of the same activations.
constexpr int decode_fused_lds_bytes(int64_t K) { return (int)(K / 128 * 1024 + K / 512 * 256); }

template <bool IN_BF16, int TAIL>
__global__ void __launch_bounds__(256) k_gemm_decode_fused(const void* __restrict__ x, int64_t ldx, const int8_t* __restrict__ signs,
                                                           const uint8_t* __restrict__ wq, const uint8_t* __restrict__ ws,
                                                           int w_tiled, int M, int N, int K, void* __restrict__ y, int out_bf16,
                                                           int64_t ldy) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, h = lane >> 5;
    const int n0 = blockIdx.x * 128 + wave * 32;
    const int nss = K / 512;
    uint8_t* const scl = lds + (K / 128) * 1024;          // scales behind the codes
    const RowView vw(wq, ws, w_tiled != 0, min(n0 + r, N - 1), K);
    auto load_w = [&](int ss, v4i (&c)[8], v4i& sc) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                c[2 * t + j] = *reinterpret_cast<const v4i*>(vw.codes + (int64_t)(4 * ss + t) * vw.cstep + h * 32 + j * 16);
        sc = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(vw.scales + (int64_t)ss * vw.sstep));
    };
    constexpr int SETS = SMALLM_SETS, D = SETS - 1;
    v4i c[SETS][8], s4[SETS];
#pragma unroll
    for (int i = 0; i < D; ++i) load_w(min(i, nss - 1), c[i], s4[i]);

    // ---- prologue: the online step on all M rows.  A wavefront takes 64 chunks (512 elements: one
    // superstage of one row) at a time; chunk kc of a row lies in stage kc / 16, 16-byte chunk (kc % 16) / 4.
    {
        const uint32_t cpr = (uint32_t)K / 8u, nchunks = (uint32_t)M * cpr;
        const float sigma = (__builtin_popcount(lane & 3) & 1) ? -1.0f : 1.0f;
        const float cs = as_f32(0x3E3504F3u) * sigma;      // fl(1 / sqrt(32)), sign of the cross-lane stages folded in
        // four passes' loads are issued before the first is used: a wavefront is alone on its SIMD, and nothing
        // else would hide their latency
        constexpr uint32_t U = 4;
        for (uint32_t cb0 = (uint32_t)wave * 64u; cb0 < nchunks; cb0 += 256u * U) {
            float v[U][8];
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                const uint32_t cb = min(cb0 + 256u * u, nchunks - 64u);      // past the end: the last pass again, not written
                const uint32_t row = cb / cpr, kc = cb - row * cpr + (uint32_t)lane;
                load_chunk<IN_BF16>((const char*)x + ((int64_t)row * ldx + (int64_t)kc * 8) * (IN_BF16 ? 2 : 4), v[u]);
            }
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                const uint32_t cb = cb0 + 256u * u;
                if (cb >= nchunks) break;                                     // uniform
                const uint32_t row = cb / cpr, kc = cb - row * cpr + (uint32_t)lane;
                if (signs) apply_signs(v[u], signs + (size_t)kc * 8);   // uniform
                wht_inwave<5>(v[u], (uint32_t)lane);
#pragma unroll
                for (int i = 0; i < 8; ++i) v[u][i] *= cs;
                const uint32_t sb = e8m0_from_amax(quad_max(absmax8(v[u])));
                const uint32_t w = encode8_e2m1(v[u], sb);
                const uint32_t st = kc >> 4, q16 = (kc >> 2) & 3u;
                *reinterpret_cast<uint32_t*>(lds + st * 1024u + row * 64u + ((q16 ^ ((row >> 2) & 3u)) << 4) + (kc & 3u) * 4u) = w;
                if ((lane & 3) == 0) scl[(kc >> 6) * 256u + row * 16u + ((kc >> 2) & 15u)] = (uint8_t)sb;
            }
        }
    }
    __syncthreads();

    v16f acc = {};
    const uint32_t ra = (uint32_t)(r & 15);               // lanes 16..31 of a half repeat rows 0..15: never stored
    const uint32_t sw = (ra >> 2) & 3u;
    auto superstage = [&](int ss, const v4i (&cw)[8], const v4i& sc) {
        const uint8_t* cbase = lds + (uint32_t)ss * 4096u + ra * 64u;
        const v4i asc = *reinterpret_cast<const v4i*>(scl + (uint32_t)ss * 256u + ra * 16u);
        v4i af[2];
        af[0] = *reinterpret_cast<const v4i*>(cbase + (((uint32_t)(2 * h) ^ sw) << 4));
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            const int t = st >> 1, j = st & 1;
            if (st + 1 < 8) af[(st + 1) & 1] = *reinterpret_cast<const v4i*>(cbase + ((st + 1) >> 1) * 1024 + (((uint32_t)(2 * h + ((st + 1) & 1)) ^ sw) << 4));
            __builtin_amdgcn_sched_barrier(0);
            const int scb = (int)(((uint32_t)sc[t] >> (16 * h + 8 * j)) & 0xffu);
            const int sca = (int)(((uint32_t)asc[t] >> (16 * h + 8 * j)) & 0xffu);
            v8i a = {}, b = {};
            b[0] = cw[st][0]; b[1] = cw[st][1]; b[2] = cw[st][2]; b[3] = cw[st][3];
            a[0] = af[st & 1][0]; a[1] = af[st & 1][1]; a[2] = af[st & 1][2]; a[3] = af[st & 1][3];
            acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc, 4, 4, 0, sca, 0, scb);
        }
    };
    // Register sets in rotation, SETS - 1 superstages of weights in flight; the loop body is one basic block of
    // SETS turns and every load is visible to the compiler, whose wait counts are then exact.
    auto turn = [&](auto Kc, auto Issue, int ss) {
        constexpr int k = decltype(Kc)::value, kn = (k + D) % SETS;
        if constexpr (decltype(Issue)::value) load_w(min(ss + D, nss - 1), c[kn], s4[kn]);
        __builtin_amdgcn_sched_barrier(0);
        superstage(ss, c[k], s4[k]);
        __builtin_amdgcn_sched_barrier(0);
    };
    using Yes = std::true_type;
    using No = std::false_type;
    int ss = 0;
    for (; ss + SETS <= nss; ss += SETS) {
        turn(IC<0>{}, Yes{}, ss);
        turn(IC<1>{}, Yes{}, ss + 1);
        turn(IC<2>{}, Yes{}, ss + 2);
    }
    if constexpr (TAIL >= 1) turn(IC<0>{}, No{}, ss);
    if constexpr (TAIL >= 2) turn(IC<1>{}, No{}, ss + 1);
    const int col = n0 + r;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 8 * q + 4 * h + i;
            if (row < M && col < N) store_out(y, out_bf16, (int64_t)row * ldy + col, acc[4 * q + i]);
        }
}

// ---- measurement aid: the block-scaled fp4 MFMA back to back from registers ------------------
// 4 wavefronts per workgroup, one per SIMD, the register tile of the large-shape product kernel: 4 W
// fragments x 4 A fragments -> 16 independent 32x32 accumulators, every MFMA on another pair of fragments
// (so that the operand registers switch between consecutive instructions as they do in the product).  The
// fragments are 16 bytes per lane from `operands`: W fragment t from bytes [1024 t, 1024 t + 1024), A fragment
// t from [4096 + 1024 t, ...); scale bytes 127.  What a launch of this sustains is the ceiling of any product
// kernel on the same operand bit patterns: it includes the instruction's own issue overhead and whatever
// clock the chip holds under that load, and nothing else.
__global__ void __launch_bounds__(256, 1) k_mfma_ceiling(const uint8_t* __restrict__ operands, int iters,
                                                         float* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    v8i w8[4], a8[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const v4i w = *reinterpret_cast<const v4i*>(operands + t * 1024 + lane * 16);
        const v4i a = *reinterpret_cast<const v4i*>(operands + 4096 + t * 1024 + lane * 16);
        w8[t] = v8i{};
        a8[t] = v8i{};
        w8[t][0] = w[0]; w8[t][1] = w[1]; w8[t][2] = w[2]; w8[t][3] = w[3];
        a8[t][0] = a[0]; a8[t][1] = a[1]; a8[t][2] = a[2]; a8[t][3] = a[3];
    }
    v16f acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = v16f{};
    // Shader-clock cycles and 100 MHz reference ticks around the loop give the clock the chip held.
    // The loop bound passes through an asm statement after the first pair of timestamps and the
    // accumulators' sum through one before the second, so the loop cannot move across either.
    const uint64_t c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
    asm volatile("" : "+s"(iters) : "s"(c0), "s"(r0));
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(w8[i >> 2], a8[i & 3], acc[i], 4, 4, 0, 127, 0, 127);
    }
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) t += acc[i][j];
    asm volatile("" : "+v"(t));
    const uint64_t c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
    if (blockIdx.x == 0 && threadIdx.x < 2) t = (float)(threadIdx.x == 0 ? c1 - c0 : r1 - r0);
    sink[blockIdx.x * 256 + threadIdx.x] = t;
}

hipError_t launch_mfma_ceiling(const uint8_t* operands, int iters, int workgroups, float* sink, hipStream_t s) {
    hipLaunchKernelGGL(k_mfma_ceiling, dim3(workgroups), dim3(256), 0, s, operands, iters, sink);
    return hipGetLastError();
}

using SmallmKern = void (*)(const uint8_t*, const uint8_t*, int, const uint8_t*, const uint8_t*, int, int, int, int, void*,
                            int, int64_t);
static const SmallmKern smallm_kern[4][4] = {
    {k_gemm_smallm<1, 0>, k_gemm_smallm<1, 1>, k_gemm_smallm<1, 2>, k_gemm_smallm<1, 3 % SMALLM_SETS>},
    {k_gemm_smallm<2, 0>, k_gemm_smallm<2, 1>, k_gemm_smallm<2, 2>, k_gemm_smallm<2, 3 % SMALLM_SETS>},
    {k_gemm_smallm<3, 0>, k_gemm_smallm<3, 1>, k_gemm_smallm<3, 2>, k_gemm_smallm<3, 3 % SMALLM_SETS>},
    {k_gemm_smallm<4, 0>, k_gemm_smallm<4, 1>, k_gemm_smallm<4, 2>, k_gemm_smallm<4, 3 % SMALLM_SETS>}};

// The weight-streaming kernels use up to 108 KB of LDS per workgroup: declared once per device.
hipError_t setup_gemm_smallm() {
    for (int m = 0; m < 4; ++m)
        for (int t = 0; t < 4; ++t)
            if (hipError_t e = hipFuncSetAttribute((const void*)smallm_kern[m][t], hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   smallm_lds_bytes(1 + m)); e != hipSuccess) return e;
    return hipSuccess;
}

static_assert(SMALLM_SETS == 3, "k_gemm_decode_fused writes its turns out for three register sets");

hipError_t setup_gemm_decode_fused() {
    const void* kernels[6] = {(const void*)k_gemm_decode_fused<true, 0>, (const void*)k_gemm_decode_fused<true, 1>,
                              (const void*)k_gemm_decode_fused<true, 2>, (const void*)k_gemm_decode_fused<false, 0>,
                              (const void*)k_gemm_decode_fused<false, 1>, (const void*)k_gemm_decode_fused<false, 2>};
    for (const void* k : kernels)
        if (hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, decode_fused_lds_bytes(DECODE_FUSED_MAX_K));
            e != hipSuccess) return e;
    return hipSuccess;
}

hipError_t launch_gemm_decode_fused(const void* x, bool in_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* signs,
                                    const Operand& w, int64_t N, void* y, bool out_bf16, int64_t ldy, hipStream_t s) {
    int cus = 0;
    if (hipError_t e = device_cus(&cus); e != hipSuccess) return e;
    const int tail = (int)((K / 512) % SMALLM_SETS);
    const dim3 grid((uint32_t)((N + 127) / 128)), block(256);
    const int ldsb = decode_fused_lds_bytes(K);
#define BRQ_LAUNCH_DF(BF, T) hipLaunchKernelGGL((k_gemm_decode_fused<BF, T>), grid, block, ldsb, s, x, ldx, signs, w.codes, w.scales, \
                                                (int)w.tiled, (int)M, (int)N, (int)K, y, (int)out_bf16, ldy)
    if (in_bf16) { if (tail == 0) BRQ_LAUNCH_DF(true, 0); else if (tail == 1) BRQ_LAUNCH_DF(true, 1); else BRQ_LAUNCH_DF(true, 2); }
    else { if (tail == 0) BRQ_LAUNCH_DF(false, 0); else if (tail == 1) BRQ_LAUNCH_DF(false, 1); else BRQ_LAUNCH_DF(false, 2); }
#undef BRQ_LAUNCH_DF
    return hipGetLastError();
}

hipError_t launch_mxfp4_gemm(const Operand& a, const Operand& w, int64_t M, int64_t N, int64_t K, void* y,
                             bool out_bf16, int64_t ldy, hipStream_t s) {
    const int64_t Kp = (K + 511) / 512 * 512;
    int cus = 0;
    if (hipError_t e = device_cus(&cus); e != hipSuccess) return e;      // (also the per-device kernel set-up)
    if (M <= 128 && (K == Kp || (a.tiled && w.tiled)) && Kp < (int64_t(1) << 26)) {
        // decode batches: weight streaming with the activations shared through LDS
        const auto& kern = smallm_kern;
        const int mi = (int)((M - 1) / 32), tail = (int)((Kp / 512) % SMALLM_SETS);
        const dim3 grid((uint32_t)((N + 127) / 128)), block(256);
        hipLaunchKernelGGL(kern[mi][tail], grid, block, smallm_lds_bytes(1 + mi), s, a.codes, a.scales, (int)a.tiled,
                           w.codes, w.scales, (int)w.tiled, (int)M, (int)N, (int)K, y, (int)out_bf16, ldy);
        return hipGetLastError();
    }
    if (M > 16 && tiled_gemm_supported(M, N, K, out_bf16, ldy, a.tiled && w.tiled)) {
        return launch_gemm_tiled(a, w, M, N, K, y, out_bf16, ldy, s);
    } else if (M <= 16) {
        dim3 grid((uint32_t)((N + 15) / 16));
        hipLaunchKernelGGL(k_gemm_skinny, grid, dim3(256), 0, s, a.codes, a.scales, (int)a.tiled, w.codes, w.scales,
                           (int)w.tiled, (int)M, (int)N, (int)K, y, (int)out_bf16, ldy);
    } else {
        dim3 grid((uint32_t)((N + 63) / 64), (uint32_t)((M + 63) / 64));
        hipLaunchKernelGGL(k_gemm_direct, grid, dim3(256), 0, s, a.codes, a.scales, (int)a.tiled, w.codes, w.scales,
                           (int)w.tiled, (int)M, (int)N, (int)K, y, (int)out_bf16, ldy);
    }
    return hipGetLastError();
}

}  // namespace brq
