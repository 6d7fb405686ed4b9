// Large-shape W4A4 MXFP4 product for gfx950: persistent 256 x 256 output tiles, operands
// staged through LDS, contraction on v_mfma_scale_f32_32x32x64_f8f6f4 (the product of Sec. 2
// on the MXFP4 operands of Sec. 4.1).
//
// Workgroup = 4 wavefronts (2 x 2), one per SIMD, each owning a 128 x 128 piece of the tile
// as 4 x 4 MFMA tiles of 32 x 32: 256 accumulator registers per lane.  The weights are the
// MFMA's row operand and the activations its column operand, so that a lane ends up with 4
// consecutive output COLUMNS of one output row.
//
// K is consumed in stages of 128 elements (64 code bytes per row).  Within a stage lane half
// h = lane >> 5 owns groups 2h and 2h+1: MFMA step j in {0,1} contracts group 2h+j of every
// row.  Any assignment of K groups to lane halves is valid as long as both operands and
// their scales use the same one; this one lets a lane's two steps read 32 contiguous bytes
// and one 16-bit pair of scale bytes (selected with the instruction's op_sel).
//
// Operands travel HBM -> LDS with global_load_lds_dwordx4 (no VGPR staging): the 64 lanes of
// one such instruction fill 1 KB of LDS linearly (lane i -> base + 16 i) from per-lane global
// addresses.  Lane i fetches 16-byte chunk (i & 3) ^ ((i >> 4) & 3) of row i >> 2: 4 lanes
// read one contiguous 64-byte row segment, and the XOR spreads rows over the LDS banks for
// the MFMA-side ds_read_b128 (16 consecutive rows of one chunk -> 16 distinct 16-byte bank
// groups).  Scales travel the same way, 16 bytes (the 16 groups of 512 K elements) of one
// row per lane.  Both operands may come row-major or in the tiled layout of brq.h (64-row
// slabs, one contiguous 4 KB block per slab and stage): only the per-lane global offsets and
// the stage-to-stage pointer steps differ, the LDS image is the same.
//
// A ring of 4 code stages and 2 scale buffers runs continuously across the tiles a
// workgroup processes: the next tile's first stages are loading during the current tile's
// epilogue.  With one wavefront per SIMD nothing hides a stall, and the SIMD issues one
// instruction per 4 cycles while a 32x32x64 fp4 MFMA occupies the matrix core for 32: every
// gap between two MFMAs takes at most ~4 other instructions.  The stage body is therefore
// laid out by hand as 32 slots of (1 MFMA + a few LDS reads / LDS-DMA loads), pinned with
// scheduling barriers, and the K loop is unrolled by 4 so that every LDS address is an
// immediate offset.
//
// The output leaves through a 4 KB LDS block per wavefront that turns the accumulator layout
// (neighbouring lanes = different rows) into whole 128-byte row segments per 8 lanes.  M and N
// may be ragged: the last tile row (column) clamps its A (W) loads into the operand and masks its stores, rows
// one by one and columns by 16-byte chunk (so N is a multiple of 8 for bf16 and of 4 for fp32 output).
//
// LDS map (bytes): [0, 128K) 4 stages x (W rows 16K | A rows 16K); [128K, 144K) 2 scale
// buffers x (W 4K | A 4K); [144K, 160K) 4 epilogue blocks.
#include "brq_device.h"
#include "brq_launch.h"

namespace brq {
namespace tiled {

constexpr int TM = 256, TN = 256, KS = 128;
constexpr int STAGE_BYTES = 32768, OPER_BYTES = 16384;
constexpr int SCALE_BASE = 4 * STAGE_BYTES, SCALE_BUF = 8192, SCALE_OPER = 4096;
constexpr int EPI_BASE = SCALE_BASE + 2 * SCALE_BUF;    // 147456: one 4 KB output block per wavefront
constexpr int LDS_BYTES = EPI_BASE + 4 * 4096;          // 163840, all of the CU's 160 KB

template <int V>
struct IC { static constexpr int value = V; };

// Wait until at most N of this wavefront's vector-memory operations are outstanding and all
// its LDS reads have returned, then meet the other wavefronts.
template <int N>
__device__ __forceinline__ void wait_vm_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier\n\t" ::"n"(N) : "memory");
}
// Elements O .. O + 7 of an accumulator, copied to vector registers by instructions that stay where they
// are written (volatile, ordered with the MFMAs).
template <int O>
__device__ __forceinline__ void read_acc8(const v16f& a, IC<O>, float (&c)[16]) {
    asm volatile("v_accvgpr_read_b32 %0, %8\n\tv_accvgpr_read_b32 %1, %9\n\tv_accvgpr_read_b32 %2, %10\n\t"
                 "v_accvgpr_read_b32 %3, %11\n\tv_accvgpr_read_b32 %4, %12\n\tv_accvgpr_read_b32 %5, %13\n\t"
                 "v_accvgpr_read_b32 %6, %14\n\tv_accvgpr_read_b32 %7, %15"
                 : "=v"(c[O]), "=v"(c[O + 1]), "=v"(c[O + 2]), "=v"(c[O + 3]), "=v"(c[O + 4]), "=v"(c[O + 5]), "=v"(c[O + 6]), "=v"(c[O + 7])
                 : "a"(a[O]), "a"(a[O + 1]), "a"(a[O + 2]), "a"(a[O + 3]), "a"(a[O + 4]), "a"(a[O + 5]), "a"(a[O + 6]), "a"(a[O + 7]));
}

// The same without a wait for global memory: the caller has already seen its loads land.
__device__ __forceinline__ void lds_wait_and_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier\n\t" ::: "memory");
}

// Pair order of the NACC = 4 * MB accumulators of a wavefront (the order in which a tile's first stage
// starts them and the output path takes them): index X -> W tile 2 * ((X / 2) / MB) + X % 2, A tile
// (X / 2) % MB: the two W tiles of one 128-byte bf16 output block are neighbours.
template <int X, int MB>
struct PairA { static constexpr int value = 2 * ((X >> 1) / MB) + (X & 1); };
template <int X, int MB>
struct PairB { static constexpr int value = (X >> 1) % MB; };

// f(IC<-1>), f(IC<0>), ..., f(IC<N>)
template <class F, int N, int S = -1>
__device__ __forceinline__ void static_for_drain(F& f, IC<N> n, IC<S> = {}) {
    f(IC<S>{});
    if constexpr (S < N) static_for_drain(f, n, IC<S + 1>{});
}

// Tiles of one workgroup.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its
// own L2: XCD x takes the contiguous id range [x*per_xcd, (x+1)*per_xcd), and ids run down 8
// tile rows before moving to the next tile column, so the 32 tiles an XCD works on at one
// time form an 8 x 4 patch and share operand panels in its L2.
struct TileWalk {
    int first, end, stride, tiles_m, tiles_n;
    __device__ __forceinline__ void tile(int i, int& tm, int& tn) const {
        int id = first + i * stride;
        int group = id / (8 * tiles_n), rem = id - group * 8 * tiles_n;
        int rows = min(8, tiles_m - group * 8);
        tm = group * 8 + rem % rows;
        tn = rem / rows;
    }
};

// The MFMAs are issued through volatile inline assembly: the compiler treats pure intrinsic
// calls as freely movable and sinks all of a stage's MFMAs behind its memory operations,
// which is the opposite of the interleaving this kernel lives on.  Volatile asm statements
// keep their source order relative to each other and to the LDS reads.  The accumulator is
// an AGPR tuple ("a"), the fragments are 4-register VGPR tuples; SEL picks scale byte 0 / 1.
__device__ __forceinline__ void mfma_fp4(v16f& acc, const v4i& wf, const v4i& af, IC<0>, int sw, int sa) {
    asm volatile("v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, %0, %3, %4 op_sel_hi:[0,0,0] cbsz:4 blgp:4"
                 : "+a"(acc) : "v"(wf), "v"(af), "v"(sw), "v"(sa));
}
__device__ __forceinline__ void mfma_fp4(v16f& acc, const v4i& wf, const v4i& af, IC<1>, int sw, int sa) {
    asm volatile("v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, %0, %3, %4 op_sel:[1,1,0] op_sel_hi:[0,0,0] cbsz:4 blgp:4"
                 : "+a"(acc) : "v"(wf), "v"(af), "v"(sw), "v"(sa));
}
// The same with C = 0: the first MFMA of a tile on its accumulator (step 0 of the tile's first stage)
// starts the sum, so the 256 accumulator registers are never cleared by separate instructions.
__device__ __forceinline__ void mfma_fp4_init(v16f& acc, const v4i& wf, const v4i& af, int sw, int sa) {
    asm volatile("v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, 0, %3, %4 op_sel_hi:[0,0,0] cbsz:4 blgp:4"
                 : "+a"(acc) : "v"(wf), "v"(af), "v"(sw), "v"(sa));     // (tied like the others; the old value is not read)
}
#define BRQ_MFMA(ACC, WF, AF, SEL, SW, SA) mfma_fp4(ACC, WF, AF, IC<SEL>{}, SW, SA)
#define BRQ_SLOT_END() __builtin_amdgcn_sched_barrier(0)
// Refill loads are spread over the whole stage, one every fourth slot, for all four wavefronts alike: the
// texture-address unit takes ~27 cycles per load and the workgroup's four wavefronts issue theirs in the same
// slot, so four loads keep it busy for most of four slots.  (Staggering the wavefronts over the slots instead
// needs a branch per slot, and the taken branches cost more - 5% of the kernel - than the short queue does.)
#define BRQ_DMA_TAIL(I) do { if constexpr (!LAST && DIAG != 2) dma_step(Uc, IC<(I)>{}); } while (0)
#define BRQ_DMA_HEAD(I) do { if constexpr (MODE != 1 && !(LAST && U != 0) && DIAG != 2) dma_step(IC<PU>{}, IC<(I)>{}); } while (0)
// (LAST = the last superstage of the workgroup: only its first stage still has loads to issue, the tail of its own
// last stage's; no superstage follows, so nothing is loaded, no scale row and no next fragment is read for one)
#define BRQ_N0(X) do { if constexpr (!(LAST && U == 3)) { X; } } while (0)
#define BRQ_LD_SCALES(I) do { if constexpr (!LAST) ld_scales(Uc, IC<(I)>{}); } while (0)

// Where the measurement instantiation reports its clock; the product instantiation's is empty.
template <bool TIMED>
struct ClockOut {};
template <>
struct ClockOut<true> { unsigned long long* p; };

// MB = A tiles (32 rows) per wavefront: 4 -> 256 x 256 output tile, 2 -> 128 x 256 (for shapes
// with too few 256 x 256 tiles to fill the chip; the stage is then 16 MFMA slots long).
// DIAG != 0 = the measurement aids of brq_diag.h: workgroup 0 also reports the shader-clock cycles and the
// 100 MHz ticks it ran for, and how the cycles split into prologue, K loops and epilogues.  DIAG == 2 in
// addition issues no refill loads in the K loops: the ring keeps the first superstage the prologue brought, every
// MFMA, LDS read, barrier and output store runs as in the product, and the result is NOT the product - what
// the kernel would cost if its operands moved themselves.  The product (DIAG == 0) has no such code.
template <bool OUT_BF16, int MB, int DIAG>
__global__ void __launch_bounds__(256, 1) k_gemm_tiled(const uint8_t* __restrict__ aq, const uint8_t* __restrict__ as,
                                                       const uint8_t* __restrict__ wq, const uint8_t* __restrict__ ws,
                                                       int M, int N, int K, void* __restrict__ y, int64_t ldy, int a_tiled, int w_tiled,
                                                       ClockOut<DIAG != 0> clk) {
    constexpr bool TIMED = DIAG != 0;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned long long t_c0 = 0, t_r0 = 0, t_loop = 0, t_epi = 0, t_pro = 0, t_mark = 0;
    if constexpr (TIMED) {
        if (blockIdx.x == 0) { t_c0 = __builtin_readcyclecounter(); t_r0 = __builtin_amdgcn_s_memrealtime(); }
    }
    const int r = lane & 31, h = lane >> 5;
    const int wn = wave >> 1, wm = wave & 1;   // this wavefront's 128 W rows / 32 MB A rows inside the tile
    constexpr int TMv = 64 * MB;               // output rows per tile
    constexpr int ARW = 16 * MB;               // A rows each wavefront loads per stage (its share of the tile's)

    TileWalk tw;
    tw.tiles_m = (M + TMv - 1) / TMv;            // the last tile row may be ragged: loads clamp, stores mask
    tw.tiles_n = (N + TN - 1) / TN;            // ... and so may the last tile column
    {
        const int T = tw.tiles_m * tw.tiles_n, G = gridDim.x;   // G is a multiple of 8
        const int per_xcd = (T + 7) / 8, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        tw.first = xcd * per_xcd + slot;
        tw.end = min((xcd + 1) * per_xcd, T);
        tw.stride = G >> 3;
    }
    const int ntiles = tw.first < tw.end ? (tw.end - tw.first + tw.stride - 1) / tw.stride : 0;
    if (ntiles == 0) return;                  // uniform over the workgroup
    const int KQ = K / (4 * KS);              // 512-element superstages (4 stages) per tile
    const int64_t cpitch = K / 2, spitch = K / 32;

    // ---- producer state.  The producer runs one superstage (4 stages) ahead of the MFMAs.
    // A wavefront loads its own 64-row slab of each operand: per stage 4 loads of 16 rows x 64
    // bytes, which land in LDS as rows of 64 bytes with the 16-byte chunks of row i XOR-swizzled by
    // (i >> 2) & 3.  Row-major operand: lane offset ((lane >> 2) + 16 q) rows, a stage is 64
    // bytes further along K.  Tiled operand: the slab's stage is one contiguous 4096-byte block
    // (16 rows per KB), the next stage the next block: a load then touches 8 cache lines
    // instead of 16, which is what the texture-address unit charges for.
    const uint32_t swz16 = (uint32_t)(((lane & 3) ^ ((lane >> 4) & 3)) << 4);
    uint32_t vqw[4], vqa[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        vqw[q] = w_tiled ? (uint32_t)(q * 1024 + (lane >> 2) * 64) + swz16
                         : (uint32_t)(((lane >> 2) + 16 * q) * cpitch) + swz16;
        vqa[q] = a_tiled ? (uint32_t)(q * 1024 + (lane >> 2) * 64) + swz16
                         : (uint32_t)(((lane >> 2) + 16 * q) * cpitch) + swz16;
    }
    const int alane = lane & (ARW - 1);       // MB = 2: lanes 32..63 of the A scale load repeat rows 0..31
    uint32_t vscw = w_tiled ? (uint32_t)(lane * 16) : (uint32_t)(lane * spitch);
    uint32_t vsca = a_tiled ? (uint32_t)(alane * 16) : (uint32_t)(alane * spitch);
    bool a_clamped = false, w_clamped = false;   // row-major operand: the per-lane offsets currently hold clamped rows
    // byte steps: stage to stage, superstage to superstage (codes), superstage to superstage (scales)
    const int w_stage = w_tiled ? 4096 : 64, w_super = w_tiled ? 16384 : 256, w_ssuper = w_tiled ? 1024 : 16;
    const int a_stage = a_tiled ? 4096 : 64, a_super = a_tiled ? 16384 : 256, a_ssuper = a_tiled ? 1024 : 16;
    const uint32_t dma_lds = lds0 + wave * 4096;             // this wavefront's 64-row W slab in a stage
    const uint32_t dma_lds_a = lds0 + wave * (ARW * 64);      // ... and its 16 MB-row A slab
    const uint32_t dma_sc = lds0 + SCALE_BASE + wave * 1024; // ... and in a scale buffer
    int p_tile = 0, p_kq = 0;                                 // producer position: tile index, superstage in tile
    uint32_t p_buf = 0;                                       // byte offset of the scale buffer the producer fills next
    const uint8_t *p_w[4] = {}, *p_a[4] = {}, *p_ws = nullptr, *p_as = nullptr;   // [stage of the superstage]
    // The stream ends with the workgroup's last superstage: while the consumer works on that one the producer
    // issues nothing (the LAST instantiation of the stages, whose waits count the fewer loads in flight).
    auto producer_next = [&]() {   // pointers of the next superstage; once per 128 MFMAs
        if (p_kq == 0) {
            int tm, tn;
            tw.tile(min(p_tile, ntiles - 1), tm, tn);      // (K = 512: past the end the last tile again)
            const int64_t wrow = (int64_t)tn * TN + wave * 64, arow = (int64_t)tm * TMv + wave * ARW;   // slab rows
            // Slabs of the ragged last tile row / column: rows past M - 1 (N - 1) are never stored, but
            // their loads must stay inside the operand.  Tiled: the buffer has whole 64-row slabs, so a
            // slab index past the last one is clamped.  Row-major: the slab base moves back to at most
            // M - 64 and every lane clamps its row to M - 1.
            const uint8_t *bw, *bws;
            if (w_tiled) {
                const int64_t slab = min(wrow >> 6, (int64_t)(N + 63) / 64 - 1);
                bw = wq + slab * (cpitch / 64) * 4096;
                bws = ws + slab * (spitch / 16) * 1024;
            } else {
                const int64_t wbase = min(wrow, max((int64_t)N - 64, (int64_t)0));
                bw = wq + wbase * cpitch;
                bws = ws + wbase * spitch;
                if (wrow + 64 > N || w_clamped) {         // uniform; also restores the plain offsets afterwards
                    w_clamped = wrow + 64 > N;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        vqw[q] = (uint32_t)((min(wrow + (lane >> 2) + 16 * q, (int64_t)N - 1) - wbase) * cpitch) + swz16;
                    vscw = (uint32_t)((min(wrow + lane, (int64_t)N - 1) - wbase) * spitch);
                }
            }
            p_ws = uniform_ptr(bws);
            const uint8_t *ba, *bas;
            if (a_tiled) {
                // (for MB = 2 a wavefront's 32 rows are one half of a 64-row slab)
                const int64_t slab = min(arow >> 6, (int64_t)(M + 63) / 64 - 1);
                ba = aq + slab * (cpitch / 64) * 4096 + (arow & 63) * 64;
                bas = as + slab * (spitch / 16) * 1024 + (arow & 63) * 16;
            } else {
                const int64_t abase = min(arow, max((int64_t)M - ARW, (int64_t)0));
                ba = aq + abase * cpitch;
                bas = as + abase * spitch;
                if (arow + ARW > M || a_clamped) {        // uniform; also restores the plain offsets afterwards
                    a_clamped = arow + ARW > M;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        vqa[q] = (uint32_t)((min(arow + (lane >> 2) + 16 * q, (int64_t)M - 1) - abase) * cpitch) + swz16;
                    vsca = (uint32_t)((min(arow + alane, (int64_t)M - 1) - abase) * spitch);
                }
            }
            p_as = uniform_ptr(bas);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                p_w[u] = uniform_ptr(bw + u * w_stage);
                p_a[u] = uniform_ptr(ba + u * a_stage);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) { p_w[u] += w_super; p_a[u] += a_super; }
            p_ws += w_ssuper; p_as += a_ssuper;
        }
        if (++p_kq == KQ) { p_kq = 0; ++p_tile; }
    };
    // loads of stage U of the producer's superstage: I = 0, 1 the scale rows (U == 0 only, and
    // first, so that they are older than the stage's code loads), I = 2..9 the code slabs
    // (W and A alternating, 16 rows x 64 bytes each; with MB = 2 the A slab has 2 loads, not 4)
    auto dma_step = [&](auto Uc, auto Ic) {
        constexpr int U = decltype(Uc)::value, I = decltype(Ic)::value;
        if constexpr (I == 0) {
            if constexpr (U == 0) dma16<0>(dma_sc + p_buf, p_ws, vscw);
        } else if constexpr (I == 1) {
            if constexpr (U == 0) dma16<SCALE_OPER>(dma_sc + p_buf, p_as, vsca);
        } else {
            constexpr int q = (I - 2) >> 1;
            if constexpr (((I - 2) & 1) == 0) dma16<U * STAGE_BYTES + q * 1024>(dma_lds, p_w[U], vqw[q]);
            else if constexpr (q < MB) dma16<U * STAGE_BYTES + OPER_BYTES + q * 1024>(dma_lds_a, p_a[U], vqa[q]);
        }
    };
    auto dma_stage = [&](auto Uc) {
        dma_step(Uc, IC<0>{}); dma_step(Uc, IC<1>{}); dma_step(Uc, IC<2>{}); dma_step(Uc, IC<3>{});
        dma_step(Uc, IC<4>{}); dma_step(Uc, IC<5>{}); dma_step(Uc, IC<6>{}); dma_step(Uc, IC<7>{});
        dma_step(Uc, IC<8>{}); dma_step(Uc, IC<9>{});
    };

    // ---- consumer: per-lane LDS read pointers.  [0]: stages 0-1, [1]: stages 2-3 (the
    // immediate offset of a ds_read reaches 64 KB).
    const int sw = (r >> 2) & 3;
    const uint8_t *wp[2][2], *ap[2][2];     // [stage pair][step j]
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint32_t c16 = ((2 * h + j) ^ sw) << 4;
        wp[0][j] = lds + (wn * 128 + r) * 64 + c16;
        ap[0][j] = lds + OPER_BYTES + (wm * 32 * MB + r) * 64 + c16;
        wp[1][j] = wp[0][j] + 2 * STAGE_BYTES;
        ap[1][j] = ap[0][j] + 2 * STAGE_BYTES;
    }
    const uint8_t* wsp = lds + SCALE_BASE + (wn * 128 + r) * 16;                 // scale rows, buffer 0
    // A scale rows sit at 1 KB per loading wavefront: row i of the tile at (i / ARW) * 1024 + (i % ARW) * 16
    constexpr int ASC_TILE = (MB == 4) ? 512 : 1024;     // from one 32-row A tile of a wavefront to the next
    const uint8_t* asp = lds + SCALE_BASE + SCALE_OPER + (MB == 4 ? (wm * 128 + r) * 16 : wm * 2048 + r * 16);
    uint32_t c_buf = 0;                  // byte offset of the consumer's scale buffer
    const int hshift = h * 16;

    v4i w0[4], a0[MB], w1[4], a1[MB];    // step-0 / step-1 operand fragments
    int scw[2][4], sca[2][MB];           // scale registers, [stage parity][MFMA tile]
    v4i srw[4], sra[MB];                 // a superstage's 16 scale bytes of this lane's row in each MFMA tile
    v16f acc[4][MB];                     // [W tile][A tile]

    auto ld_w = [&](auto Uc, auto Jc, auto Tc) -> v4i {
        constexpr int U = decltype(Uc)::value, J = decltype(Jc)::value, T = decltype(Tc)::value;
        return *reinterpret_cast<const v4i*>(wp[U >> 1][J] + (U & 1) * STAGE_BYTES + T * 2048);
    };
    auto ld_a = [&](auto Uc, auto Jc, auto Tc) -> v4i {
        constexpr int U = decltype(Uc)::value, J = decltype(Jc)::value, T = decltype(Tc)::value;
        return *reinterpret_cast<const v4i*>(ap[U >> 1][J] + (U & 1) * STAGE_BYTES + T * 2048);
    };

    // ---- output path.  Lane (r, h) holds, for W tile a and A tile b, output row m = 32 b + r and
    // columns n = 32 a + 8 q + 4 h + {0..3}, q = 0..3: neighbouring lanes hold different rows.
    // The store path merges the 16-byte accesses of neighbouring lanes only, so storing from
    // this layout costs one cycle per lane (64 per instruction, 8K per tile).  Each wavefront
    // therefore turns its output round in a private 4 KB LDS block, 32 rows x 128 bytes at a
    // time: written as 16-byte chunks from the accumulator layout, read back with 8
    // consecutive lanes per row, stored as 8 rows x 128 contiguous bytes per instruction.
    // Chunk c of row i sits at i * 128 + ((c ^ (i & 7)) << 4): 8 lanes that write (8 rows, one
    // chunk) or read (one row, 8 chunks) then cover all 32 banks.  LDS operations of one
    // wavefront execute in order, so write -> read -> next write need no waits.
    //
    // A block is 32 rows x 128 bytes: bf16 -> the accumulators of two neighbouring W tiles and one
    // A tile; fp32 -> one accumulator.  Accumulators are taken in "pair order": index x ->
    // W tile 2 * ((x / 2) / MB) + x % 2, A tile (x / 2) % MB, so that the two accumulators of a bf16
    // block are consecutive.  Three steps per block: pack + write to LDS (per accumulator), read
    // back, store.  They are spread over the MFMA slots of the NEXT tile's first stage (drain_slot
    // below): the matrix cores start the next tile while the vector units move this one out, and
    // only a workgroup's last tile pays for its output on its own.
    constexpr int ES = OUT_BF16 ? 2 : 4;
    constexpr int NACC = 4 * MB, XPB = OUT_BF16 ? 2 : 1;     // accumulators per wavefront, per block
    const int64_t pitch = ldy * ES;
    uint8_t* const ybytes = reinterpret_cast<uint8_t*>(y);
    uint8_t* const ebuf = lds + EPI_BASE + wave * 4096;
    uint8_t* ytile = ybytes;        // the finished tile's corner for this wavefront
    int mrem = 0, nrem = 0;         // this lane stores rows row + 8 j < mrem of the blocks whose first column is < nrem
    uint32_t st_off = 0, wsw = 0;
    uint8_t* ewr = ebuf;
    const uint8_t* erd = ebuf;
    uint4 ob[2][4];                 // two blocks read back: rows (lane >> 3) + 8 j, j = 0..3
    auto out_begin = [&](int ti_done) __attribute__((always_inline)) {
        int ti_e = ti_done;
        asm volatile("" : "+s"(ti_e));    // keeps the address arithmetic below out of the K loop
        int tm, tn;
        tw.tile(ti_e, tm, tn);
        ytile = ybytes + ((int64_t)tm * TMv + wm * 32 * MB) * pitch + ((int64_t)tn * TN + wn * 128) * ES;
        // The per-lane offsets do not depend on the tile; passing the lane through an empty asm
        // statement makes them be recomputed here (a dozen instructions per tile) instead of living in
        // registers across the K loop.
        int le = lane;
        asm volatile("" : "+v"(le));
        const int re = le & 31, he = le >> 5;
        st_off = (uint32_t)(le >> 3) * (uint32_t)pitch + (le & 7) * 16;
        ewr = ebuf + re * 128;                                   // this lane's row for writing
        wsw = (uint32_t)((re & 7) ^ he) << 4;                    // its chunk swizzle, h folded in
        erd = ebuf + (le >> 3) * 128 + (((le & 7) ^ ((le >> 3) & 7)) << 4);
        mrem = M - (tm * TMv + wm * 32 * MB) - (le >> 3);
        nrem = N - (tn * TN + wn * 128) - (le & 7) * (16 / ES);     // N is a multiple of the 16-byte chunk's columns
    };
    auto out_pack_write = [&](auto Xc) __attribute__((always_inline)) {
        constexpr int X = decltype(Xc)::value;
        const v16f& cacc = acc[PairA<X, MB>::value][PairB<X, MB>::value];
        if constexpr (OUT_BF16) {
            // The accumulator is read HERE, by instructions the compiler cannot move: left to itself it copies
            // every accumulator that a stage will move out into vector registers at the top of the stage
            // (the copies depend on nothing), which takes more registers than there are.
            float c[16];
            read_acc8(cacc, IC<0>{}, c);
            read_acc8(cacc, IC<8>{}, c);
            // v_permlane32_swap trades q between the lane halves: a lane then holds columns
            // 32 a + 16 p + 8 h + {0..7}, p = 0, 1, as one chunk, index (a & 1) * 4 + 2 p + h within the row
            constexpr int a1 = X & 1;
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                uint32_t x0 = pack_bf16x2(c[8 * p + 0], c[8 * p + 1]), x1 = pack_bf16x2(c[8 * p + 2], c[8 * p + 3]);
                uint32_t y0 = pack_bf16x2(c[8 * p + 4], c[8 * p + 5]), y1 = pack_bf16x2(c[8 * p + 6], c[8 * p + 7]);
                auto s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
                auto s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
                *reinterpret_cast<uint4*>(ewr + (wsw ^ (uint32_t)((a1 * 4 + 2 * p) << 4))) = make_uint4(s0[0], s1[0], s0[1], s1[1]);
            }
        } else {
            // chunk index 2 q + h
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<float4*>(ewr + (wsw ^ (uint32_t)(q << 5))) = make_float4(cacc[4 * q], cacc[4 * q + 1], cacc[4 * q + 2], cacc[4 * q + 3]);
        }
    };
    auto out_read = [&](auto Kc) __attribute__((always_inline)) {
        constexpr int Kb = decltype(Kc)::value & 1;
        ob[Kb][0] = *reinterpret_cast<const uint4*>(erd);
        ob[Kb][1] = *reinterpret_cast<const uint4*>(erd + 1024);
        ob[Kb][2] = *reinterpret_cast<const uint4*>(erd + 2048);
        ob[Kb][3] = *reinterpret_cast<const uint4*>(erd + 3072);
    };
    auto out_store = [&](auto Kc) __attribute__((always_inline)) {
        constexpr int Kk = decltype(Kc)::value, Kb = Kk & 1, X = Kk * XPB;
        constexpr int row = PairB<X, MB>::value * 32;
        constexpr int colbytes = (OUT_BF16 ? PairA<X, MB>::value / 2 : PairA<X, MB>::value) * 128;
        uint8_t* dst = ytile + row * pitch + colbytes + st_off;
        // whole 128-byte lines that this kernel never reads back: with the streaming hint the output does not
        // displace the operand panels that the other XCDs are about to fetch from the memory-side cache
        typedef unsigned int u4 __attribute__((ext_vector_type(4)));
        const int mr = (colbytes / ES < nrem) ? mrem : 0;     // a chunk past column N - 1 is not stored
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (row + 8 * j < mr)
                __builtin_nontemporal_store(u4{ob[Kb][j].x, ob[Kb][j].y, ob[Kb][j].z, ob[Kb][j].w}, reinterpret_cast<u4*>(dst + 8 * j * pitch));
    };
    // What the output path does after MFMA slot S of the next tile's first stage (S = -1: before slot 0;
    // S = NACC: the first slot of that stage's second step): accumulator S + 1 is packed and written (the
    // MFMA of slot S + 1 overwrites it), a completed block is read back, and the block read two slots
    // earlier is stored.
    auto drain_slot = [&](auto Sc) __attribute__((always_inline)) {
        constexpr int X = decltype(Sc)::value + 1, XR = X - 2;
        if constexpr (X < NACC) out_pack_write(IC<X>{});
        if constexpr (XR >= 0 && XR < NACC && XR % XPB == XPB - 1) out_store(IC<XR / XPB>{});
        if constexpr (X < NACC && X % XPB == XPB - 1) out_read(IC<X / XPB>{});
    };

    // One stage (U = stage & 3).  Slots m0..m31 = MFMAs in (W tile a, A tile b) order, step 0
    // then step 1.  F1 = step-1 fragments of this stage, N0 = step-0 fragments of the next.
    //   m0..m7    one F1 read each (this stage landed before the previous barrier)
    //   m8..m11   stage 3 only: the next superstage's scale rows (ld_scales)
    //   m11|m12   wait (next stage landed) + barrier (everyone is done reading this stage)
    //   m12..m15  N0 W-fragments 0..2 (registers last used by m3, m7, m11)
    //   m16..m20  N0 W-fragment 3 and the A-fragments (registers free after m15)
    //   m12..m31  the loads that refill this stage's buffer with stage + 4, every other slot
    //   m26..m29  next stage's scale registers
    // MODE 0: any stage but a tile's first.  MODE 1, 2: a tile's first stage (U = 0): its step-0 MFMAs take
    // C = 0 (nothing ever clears the accumulators) and run in pair order; MODE 2 also moves the previous
    // tile out (drain_slot after every step-0 MFMA).  The order of MFMAs on different accumulators does not
    // change any sum; the read schedule above still holds in pair order (W fragments 0, 1 are last used by
    // m6, m7, fragment 2 by m14, fragment 3 and the A fragments by m12..m15).
    // Scales.  A row's 16 scale bytes of a superstage are read ONCE, as one 16-byte access per MFMA tile
    // (32 rows x 16 bytes: every bank once), in the last stage of the superstage before, slots 8..11 (MB = 2:
    // 4..7), which carry no other LDS read: the buffer landed two barriers earlier, and the registers' old
    // contents were last used when this stage's scale registers were made during the stage before.  Reading
    // the dword of one stage at a time instead costs four accesses per tile and superstage, each of them a
    // 4-way bank conflict (32 rows, 16 bytes apart, 4 bytes wide).  Dword NU of the row holds stage NU's four
    // groups; lane half h takes bytes 2h, 2h + 1 of it.
    auto ld_scales = [&](auto Uc, auto Ic) __attribute__((always_inline)) {
        constexpr int U = decltype(Uc)::value, I = decltype(Ic)::value;
        if constexpr (U == 3) {
            const uint32_t nb = c_buf ^ SCALE_BUF;
            if constexpr (MB == 4) {
                srw[I] = *reinterpret_cast<const v4i*>(wsp + nb + I * 512);
                sra[I] = *reinterpret_cast<const v4i*>(asp + nb + I * ASC_TILE);
            } else {
                srw[I] = *reinterpret_cast<const v4i*>(wsp + nb + I * 512);
                if constexpr (I < MB) sra[I] = *reinterpret_cast<const v4i*>(asp + nb + I * ASC_TILE);
            }
        }
    };
    auto next_scale = [&](const v4i& row, auto Nc) __attribute__((always_inline)) -> int {
        return (int)((uint32_t)row[decltype(Nc)::value] >> hshift);
    };
    auto stage = [&](auto Uc, auto Modec, auto Lastc) __attribute__((always_inline)) {
        constexpr int U = decltype(Uc)::value, P = U & 1, NU = (U + 1) & 3, PU = (U + 3) & 3;
        constexpr int MODE = decltype(Modec)::value;
        constexpr bool LAST = decltype(Lastc)::value != 0;
        // loads younger than the stage a wait is for: two stages' worth, fewer once the last superstage has stopped issuing
        constexpr int VMW = (MB == 4) ? (!LAST || U == 0 ? 16 : U == 1 ? 8 : 0) : (!LAST || U == 0 ? 12 : U == 1 ? 6 : 0);
        static_assert(MODE == 0 || U == 0, "a tile starts with stage 0");
        using N_ = IC<NU>;
        using J0 = IC<0>;
        using J1 = IC<1>;
        int (&csw)[4] = scw[P];
        int (&csa)[MB] = sca[P];
        int (&nsw)[4] = scw[P ^ 1];
        int (&nsa)[MB] = sca[P ^ 1];
        // step-0 MFMA of slot S: plain order + accumulate, or pair order + C = 0 (+ the output path's share)
#define BRQ_STEP0(S, A, B_)                                                                                          \
        do {                                                                                                         \
            if constexpr (MODE == 0) BRQ_MFMA(acc[A][B_], w0[A], a0[B_], 0, csw[A], csa[B_]);                        \
            else {                                                                                                   \
                mfma_fp4_init(acc[PairA<S, MB>::value][PairB<S, MB>::value], w0[PairA<S, MB>::value],               \
                              a0[PairB<S, MB>::value], csw[PairA<S, MB>::value], csa[PairB<S, MB>::value]);          \
                if constexpr (MODE == 2) drain_slot(IC<S>{});                                                        \
            }                                                                                                        \
        } while (0)
        if constexpr (MODE == 2) {
            // The next stage's loads are waited for HERE, before the output path issues its first store: from
            // now on stores and loads are mixed in the counter, and a count is only safe against loads.  (Its
            // younger loads are the 2 stages after it; nothing older than a tile ago is still outstanding.)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(MB == 4 ? 13 : 10) : "memory");
            drain_slot(IC<-1>{});
            BRQ_SLOT_END();
        }

        if constexpr (MB == 4) {
            BRQ_STEP0(0, 0, 0); w1[0] = ld_w(Uc, J1{}, IC<0>{}); BRQ_DMA_HEAD(7); BRQ_SLOT_END();
            BRQ_STEP0(1, 0, 1); a1[0] = ld_a(Uc, J1{}, IC<0>{}); BRQ_SLOT_END();
            BRQ_STEP0(2, 0, 2); a1[1] = ld_a(Uc, J1{}, IC<1>{}); BRQ_SLOT_END();
            BRQ_STEP0(3, 0, 3); a1[2] = ld_a(Uc, J1{}, IC<2>{}); BRQ_SLOT_END();
            BRQ_STEP0(4, 1, 0); a1[3] = ld_a(Uc, J1{}, IC<3>{}); BRQ_DMA_HEAD(8); BRQ_SLOT_END();
            BRQ_STEP0(5, 1, 1); w1[1] = ld_w(Uc, J1{}, IC<1>{}); BRQ_SLOT_END();
            BRQ_STEP0(6, 1, 2); w1[2] = ld_w(Uc, J1{}, IC<2>{}); BRQ_SLOT_END();
            BRQ_STEP0(7, 1, 3); w1[3] = ld_w(Uc, J1{}, IC<3>{}); BRQ_SLOT_END();
            BRQ_STEP0(8, 2, 0); BRQ_LD_SCALES(0); BRQ_DMA_HEAD(9);
            if constexpr (U == 0 && !LAST) { producer_next(); p_buf ^= SCALE_BUF; }      // the previous superstage's loads are all issued
            BRQ_SLOT_END();
            BRQ_STEP0(9, 2, 1); BRQ_LD_SCALES(1); BRQ_SLOT_END();
            BRQ_STEP0(10, 2, 2); BRQ_LD_SCALES(2); BRQ_SLOT_END();
            BRQ_STEP0(11, 2, 3); BRQ_LD_SCALES(3); BRQ_SLOT_END();
            // The next stage's loads have landed once at most 16 vector-memory operations are outstanding:
            // the LOADS younger than them are two stages' worth, 8 code loads each (this stage's buffer
            // was refilled by slots 12..31 of the stage three back and slots 0..8 of the one after it; since
            // then came that stage's slots 12..31, all of the stage before this one, and this stage's slots
            // 0..8: 5 + 3 + 5 + 3, and 2 more when a stage 0 with its scale loads is among them).  The output
            // path's stores share the counter and complete out of order with the loads, but loads complete in
            // order among themselves: if a load of the next stage were still outstanding, so would be its 16
            // younger ones, 17 in all.  The count is therefore safe whatever the stores do; stores still in
            // flight only make the wait stricter, which is why MODE 2 has waited before its first store (there
            // with this stage's own 3 loads not yet issued: 13) and only meets the others here.
            if constexpr (MODE == 2) lds_wait_and_barrier();
            else wait_vm_and_barrier<VMW>();
            // refill of this stage's buffer: the scale rows first (stage 0; the wait two stages on then covers
            // them: 5 + 8 + 3 younger loads), a code load every fourth slot, the last three in the next stage
            BRQ_STEP0(12, 3, 0); BRQ_N0(w0[0] = ld_w(N_{}, J0{}, IC<0>{})); BRQ_DMA_TAIL(0); BRQ_SLOT_END();
            BRQ_STEP0(13, 3, 1); BRQ_N0(w0[1] = ld_w(N_{}, J0{}, IC<1>{})); BRQ_DMA_TAIL(1); BRQ_SLOT_END();
            BRQ_STEP0(14, 3, 2); BRQ_N0(w0[2] = ld_w(N_{}, J0{}, IC<2>{})); BRQ_DMA_TAIL(2); BRQ_SLOT_END();
            BRQ_STEP0(15, 3, 3); BRQ_SLOT_END();

            BRQ_MFMA(acc[0][0], w1[0], a1[0], 1, csw[0], csa[0]); BRQ_N0(w0[3] = ld_w(N_{}, J0{}, IC<3>{}));
            if constexpr (MODE == 2) drain_slot(IC<NACC>{});
            BRQ_SLOT_END();
            BRQ_MFMA(acc[0][1], w1[0], a1[1], 1, csw[0], csa[1]); BRQ_N0(a0[0] = ld_a(N_{}, J0{}, IC<0>{})); BRQ_SLOT_END();
            BRQ_MFMA(acc[0][2], w1[0], a1[2], 1, csw[0], csa[2]); BRQ_N0(a0[1] = ld_a(N_{}, J0{}, IC<1>{})); BRQ_DMA_TAIL(3); BRQ_SLOT_END();
            BRQ_MFMA(acc[0][3], w1[0], a1[3], 1, csw[0], csa[3]); BRQ_N0(a0[2] = ld_a(N_{}, J0{}, IC<2>{})); BRQ_SLOT_END();
            BRQ_MFMA(acc[1][0], w1[1], a1[0], 1, csw[1], csa[0]); BRQ_N0(a0[3] = ld_a(N_{}, J0{}, IC<3>{})); BRQ_SLOT_END();
            BRQ_MFMA(acc[1][1], w1[1], a1[1], 1, csw[1], csa[1]); BRQ_SLOT_END();
            BRQ_MFMA(acc[1][2], w1[1], a1[2], 1, csw[1], csa[2]); BRQ_DMA_TAIL(4); BRQ_SLOT_END();
            BRQ_MFMA(acc[1][3], w1[1], a1[3], 1, csw[1], csa[3]); BRQ_SLOT_END();
            BRQ_MFMA(acc[2][0], w1[2], a1[0], 1, csw[2], csa[0]); BRQ_SLOT_END();
            BRQ_MFMA(acc[2][1], w1[2], a1[1], 1, csw[2], csa[1]); BRQ_SLOT_END();
            BRQ_MFMA(acc[2][2], w1[2], a1[2], 1, csw[2], csa[2]); nsw[0] = next_scale(srw[0], N_{}); nsw[1] = next_scale(srw[1], N_{}); BRQ_DMA_TAIL(5); BRQ_SLOT_END();
            BRQ_MFMA(acc[2][3], w1[2], a1[3], 1, csw[2], csa[3]); nsw[2] = next_scale(srw[2], N_{}); nsw[3] = next_scale(srw[3], N_{}); BRQ_SLOT_END();
            BRQ_MFMA(acc[3][0], w1[3], a1[0], 1, csw[3], csa[0]); nsa[0] = next_scale(sra[0], N_{}); nsa[1] = next_scale(sra[1], N_{}); BRQ_SLOT_END();
            BRQ_MFMA(acc[3][1], w1[3], a1[1], 1, csw[3], csa[1]); nsa[2] = next_scale(sra[2], N_{}); nsa[3] = next_scale(sra[3], N_{}); BRQ_SLOT_END();
            BRQ_MFMA(acc[3][2], w1[3], a1[2], 1, csw[3], csa[2]); BRQ_DMA_TAIL(6); BRQ_SLOT_END();
            BRQ_MFMA(acc[3][3], w1[3], a1[3], 1, csw[3], csa[3]); BRQ_SLOT_END();
        } else {
            // 128 x 256 tile: 16 slots.  m0..m5 F1 reads, m4..m7 scale rows (stage 3), m7|m8 wait + barrier,
            // m8..m13 N0 reads, m13..m15 scale registers.  Refill: 6 code loads per stage, 4 of them in
            // m10..m15 and 2 in the next stage's m1, m5; the scale loads of stage 0 in m8, m9.  Two stages'
            // worth of loads, 12, are younger than the stage the wait is for (10 before MODE 2's first store).
            BRQ_STEP0(0, 0, 0); w1[0] = ld_w(Uc, J1{}, IC<0>{}); BRQ_SLOT_END();
            BRQ_STEP0(1, 0, 1); a1[0] = ld_a(Uc, J1{}, IC<0>{}); BRQ_DMA_HEAD(6); BRQ_SLOT_END();
            BRQ_STEP0(2, 1, 0); a1[1] = ld_a(Uc, J1{}, IC<1>{}); BRQ_SLOT_END();
            BRQ_STEP0(3, 1, 1); w1[1] = ld_w(Uc, J1{}, IC<1>{}); BRQ_SLOT_END();
            BRQ_STEP0(4, 2, 0); w1[2] = ld_w(Uc, J1{}, IC<2>{}); BRQ_LD_SCALES(0); BRQ_SLOT_END();
            BRQ_STEP0(5, 2, 1); w1[3] = ld_w(Uc, J1{}, IC<3>{}); BRQ_LD_SCALES(1); BRQ_DMA_HEAD(8);
            if constexpr (U == 0 && !LAST) { producer_next(); p_buf ^= SCALE_BUF; }
            BRQ_SLOT_END();
            BRQ_STEP0(6, 3, 0); BRQ_LD_SCALES(2); BRQ_SLOT_END();
            BRQ_STEP0(7, 3, 1); BRQ_LD_SCALES(3); BRQ_SLOT_END();
            if constexpr (MODE == 2) lds_wait_and_barrier();
            else wait_vm_and_barrier<VMW>();
            BRQ_MFMA(acc[0][0], w1[0], a1[0], 1, csw[0], csa[0]); BRQ_N0(w0[0] = ld_w(N_{}, J0{}, IC<0>{})); BRQ_DMA_TAIL(0);
            if constexpr (MODE == 2) drain_slot(IC<NACC>{});
            BRQ_SLOT_END();
            BRQ_MFMA(acc[0][1], w1[0], a1[1], 1, csw[0], csa[1]); BRQ_N0(a0[0] = ld_a(N_{}, J0{}, IC<0>{})); BRQ_DMA_TAIL(1); BRQ_SLOT_END();
            BRQ_MFMA(acc[1][0], w1[1], a1[0], 1, csw[1], csa[0]); BRQ_N0(a0[1] = ld_a(N_{}, J0{}, IC<1>{})); BRQ_DMA_TAIL(2); BRQ_SLOT_END();
            BRQ_MFMA(acc[1][1], w1[1], a1[1], 1, csw[1], csa[1]); BRQ_N0(w0[1] = ld_w(N_{}, J0{}, IC<1>{})); BRQ_SLOT_END();
            BRQ_MFMA(acc[2][0], w1[2], a1[0], 1, csw[2], csa[0]); BRQ_N0(w0[2] = ld_w(N_{}, J0{}, IC<2>{})); BRQ_DMA_TAIL(3); BRQ_SLOT_END();
            BRQ_MFMA(acc[2][1], w1[2], a1[1], 1, csw[2], csa[1]); BRQ_N0(w0[3] = ld_w(N_{}, J0{}, IC<3>{})); BRQ_SLOT_END();
            BRQ_MFMA(acc[3][0], w1[3], a1[0], 1, csw[3], csa[0]); nsw[0] = next_scale(srw[0], N_{}); nsw[1] = next_scale(srw[1], N_{}); BRQ_DMA_TAIL(4); BRQ_SLOT_END();
            BRQ_MFMA(acc[3][1], w1[3], a1[1], 1, csw[3], csa[1]); nsw[2] = next_scale(srw[2], N_{}); nsw[3] = next_scale(srw[3], N_{});
            nsa[0] = next_scale(sra[0], N_{}); nsa[1] = next_scale(sra[1], N_{}); BRQ_DMA_TAIL(5); BRQ_SLOT_END();
        }
#undef BRQ_STEP0
    };

    // ---- prologue: superstage 0 in flight, its first fragments in registers
    producer_next();
    dma_stage(IC<0>{});
    dma_stage(IC<1>{});
    dma_stage(IC<2>{});
    dma_stage(IC<3>{});
    // Stage 0 and the scale rows have landed once only the three later stages' loads are outstanding; the stages'
    // own waits take it from there (their counts hold from the start: the prologue's later stages stand in for the
    // loads a running ring would have issued).
    wait_vm_and_barrier<(MB == 4 ? 24 : 18)>();
    w0[0] = ld_w(IC<0>{}, IC<0>{}, IC<0>{}); w0[1] = ld_w(IC<0>{}, IC<0>{}, IC<1>{});
    w0[2] = ld_w(IC<0>{}, IC<0>{}, IC<2>{}); w0[3] = ld_w(IC<0>{}, IC<0>{}, IC<3>{});
    a0[0] = ld_a(IC<0>{}, IC<0>{}, IC<0>{}); a0[1] = ld_a(IC<0>{}, IC<0>{}, IC<1>{});
    if constexpr (MB == 4) { a0[2] = ld_a(IC<0>{}, IC<0>{}, IC<2>{}); a0[3] = ld_a(IC<0>{}, IC<0>{}, IC<3>{}); }
#pragma unroll
    for (int t = 0; t < 4; ++t) { srw[t] = *reinterpret_cast<const v4i*>(wsp + t * 512); scw[0][t] = (int)((uint32_t)srw[t][0] >> hshift); }
#pragma unroll
    for (int t = 0; t < MB; ++t) { sra[t] = *reinterpret_cast<const v4i*>(asp + t * ASC_TILE); sca[0][t] = (int)((uint32_t)sra[t][0] >> hshift); }

    // One superstage = 4 stages of MFMAs on the consumer side, and the loads of the producer's
    // superstage (the next one of the stream) on the other.
    auto superstage = [&](auto Modec, auto Lastc) __attribute__((always_inline)) {
        stage(IC<0>{}, Modec, Lastc);
        stage(IC<1>{}, IC<0>{}, Lastc);
        stage(IC<2>{}, IC<0>{}, Lastc);
        stage(IC<3>{}, IC<0>{}, Lastc);
        c_buf ^= SCALE_BUF;
    };
    // The accumulators are one read-modify-write chain from here to the end (no instruction: each tile's
    // first MFMAs take C = 0).
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < MB; ++b) asm volatile("" : "=a"(acc[a][b]));
    if constexpr (TIMED) { t_mark = __builtin_readcyclecounter(); t_pro = t_mark - t_c0; }
    // The workgroup's first tile has no predecessor to move out; every later tile's first stage carries the
    // output of the tile before it.
    // The workgroup's superstages in order: tile 0 starts in mode 1, every later tile in mode 2 (after out_begin
    // for the tile before it), all others are plain.  The very last one is peeled off and issues no loads for a
    // successor (LAST) - unless K is a single superstage: then it is a tile's first stage as well, runs like any
    // other, and the loads it issues for a successor that does not exist are waited for at the end.
    {
        const int peel = KQ > 1 ? 1 : 0;
        superstage(IC<1>{}, IC<0>{});
        for (int kq = 1; kq < KQ - (ntiles == 1 ? peel : 0); ++kq) superstage(IC<0>{}, IC<0>{});
        for (int ti = 1; ti < ntiles; ++ti) {
            out_begin(ti - 1);
            superstage(IC<2>{}, IC<0>{});
            for (int kq = 1; kq < KQ - (ti == ntiles - 1 ? peel : 0); ++kq) superstage(IC<0>{}, IC<0>{});
        }
        if (peel) superstage(IC<0>{}, IC<1>{});
    }
    if constexpr (TIMED) { const unsigned long long t = __builtin_readcyclecounter(); t_loop += t - t_mark; t_mark = t; }
    // ---- the last tile's output, with nothing to overlap it.  Its accumulators were last written by MFMAs
    // hidden in inline assembly: the compiler does not know to keep the 18 wait states between a 16-pass
    // MFMA and a read of its result.
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    out_begin(ntiles - 1);
    static_for_drain(drain_slot, IC<NACC>{});
    if constexpr (TIMED) { const unsigned long long t = __builtin_readcyclecounter(); t_epi += t - t_mark; t_mark = t; }
    // K > 512: every load into LDS landed before the last superstage's third barrier; only output stores are in
    // flight, and those may outlive the workgroup.  K = 512: the successor's loads must land before the LDS is released.
    if (KQ == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if constexpr (TIMED) {
        if (blockIdx.x == 0) {
            const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
            if (tid == 0) {
                clk.p[0] = c1 - t_c0; clk.p[1] = r1 - t_r0; clk.p[2] = t_loop; clk.p[3] = t_epi;
                clk.p[4] = (unsigned long long)ntiles; clk.p[5] = t_pro;
            }
        }
    }
}

#undef BRQ_MFMA
#undef BRQ_SLOT_END
#undef BRQ_DMA_TAIL
#undef BRQ_DMA_HEAD
#undef BRQ_N0
#undef BRQ_LD_SCALES

}  // namespace tiled

// K must be whole 512-element superstages; tiled operands are zero-padded to that by the
// quantizers, so with both operands tiled any K will do.
bool tiled_gemm_supported(int64_t M, int64_t N, int64_t K, bool out_bf16, int64_t ldy, bool both_tiled) {
    const int64_t Kp = (K + 511) / 512 * 512;
    return M > 0 && N > 0 && N % (out_bf16 ? 8 : 4) == 0 && (K == Kp || both_tiled) &&
           (ldy * (out_bf16 ? 2 : 4)) % 16 == 0 && ldy * (out_bf16 ? 2 : 4) < (int64_t(1) << 28) &&
           (Kp / 2) * 64 < (int64_t(1) << 31);
}

template <bool OUT_BF16, int MB, int DIAG>
static void launch_one(dim3 g, hipStream_t s, const Operand& a, const Operand& w, int M, int N, int K, void* y, int64_t ldy,
                       unsigned long long* clk) {
    tiled::ClockOut<DIAG != 0> c;
    if constexpr (DIAG != 0) c.p = clk;
    hipLaunchKernelGGL((tiled::k_gemm_tiled<OUT_BF16, MB, DIAG>), g, dim3(256), tiled::LDS_BYTES, s, a.codes, a.scales, w.codes,
                       w.scales, M, N, K, y, ldy, (int)a.tiled, (int)w.tiled, c);
}

// The kernels use all 160 KB of the CU's LDS: declared once per device.
hipError_t setup_gemm_tiled() {
    const void* kernels[9] = {(const void*)tiled::k_gemm_tiled<true, 4, 0>, (const void*)tiled::k_gemm_tiled<false, 4, 0>,
                              (const void*)tiled::k_gemm_tiled<true, 2, 0>, (const void*)tiled::k_gemm_tiled<false, 2, 0>,
                              (const void*)tiled::k_gemm_tiled<true, 4, 1>, (const void*)tiled::k_gemm_tiled<false, 4, 1>,
                              (const void*)tiled::k_gemm_tiled<true, 2, 1>, (const void*)tiled::k_gemm_tiled<false, 2, 1>,
                              (const void*)tiled::k_gemm_tiled<true, 4, 2>};
    for (const void* k : kernels)
        if (hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, tiled::LDS_BYTES); e != hipSuccess) return e;
    return hipSuccess;
}

hipError_t launch_gemm_tiled(const Operand& a, const Operand& w, int64_t M, int64_t N, int64_t K, void* y,
                             bool out_bf16, int64_t ldy, hipStream_t s, unsigned long long* clk, bool no_loads) {
    int cus = 0;
    if (hipError_t e = device_cus(&cus); e != hipSuccess) return e;
    cus = cus >= 8 ? (cus & ~7) : 8;     // whole rounds of the 8 XCDs
    K = (K + 511) / 512 * 512;   // padded K of tiled operands (a no-op otherwise)
    // 256 x 256 tiles unless there are too few of them to give every CU one: then 128 x 256
    const int64_t tn = (N + tiled::TN - 1) / tiled::TN;
    const int64_t T4 = ((M + 255) / 256) * tn, T2 = ((M + 127) / 128) * tn;
    const bool half = T4 < cus && T2 > T4;
    const int T = (int)(half ? T2 : T4);
    const int grid = T < cus ? ((T + 7) & ~7) : cus;
    const dim3 g(grid);
    const int Mi = (int)M, Ni = (int)N, Ki = (int)K;
    if (no_loads) {    // brq_diag_mxfp4_gemm_no_loads: one instantiation only
        if (!clk || half || !out_bf16) return hipErrorInvalidValue;
        launch_one<true, 4, 2>(g, s, a, w, Mi, Ni, Ki, y, ldy, clk);
    } else if (clk) {     // the measurement instantiation (brq_diag_mxfp4_gemm_clock)
        if (half) out_bf16 ? launch_one<true, 2, 1>(g, s, a, w, Mi, Ni, Ki, y, ldy, clk) : launch_one<false, 2, 1>(g, s, a, w, Mi, Ni, Ki, y, ldy, clk);
        else out_bf16 ? launch_one<true, 4, 1>(g, s, a, w, Mi, Ni, Ki, y, ldy, clk) : launch_one<false, 4, 1>(g, s, a, w, Mi, Ni, Ki, y, ldy, clk);
    } else {
        if (half) out_bf16 ? launch_one<true, 2, 0>(g, s, a, w, Mi, Ni, Ki, y, ldy, clk) : launch_one<false, 2, 0>(g, s, a, w, Mi, Ni, Ki, y, ldy, clk);
        else out_bf16 ? launch_one<true, 4, 0>(g, s, a, w, Mi, Ni, Ki, y, ldy, clk) : launch_one<false, 4, 0>(g, s, a, w, Mi, Ni, Ki, y, ldy, clk);
    }
    return hipGetLastError();
}

}  // namespace brq
