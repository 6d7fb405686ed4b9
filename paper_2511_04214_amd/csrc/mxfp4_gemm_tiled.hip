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
// row per lane.
//
// A ring of 4 code stages and 2 scale buffers runs continuously across the tiles a
// workgroup processes: the next tile's first stages are loading during the current tile's
// epilogue.  Per stage: the step-1 fragments are read from LDS while the 16 step-0 MFMAs
// run; then one s_barrier (next stage has landed everywhere, this stage's buffer is free);
// then the step-0 fragments of the next stage are read and the 10 loads that refill the
// freed buffer are issued, one between each pair of the 16 step-1 MFMAs.
//
// LDS map (bytes): [0, 128K) 4 stages x (W rows 16K | A rows 16K); [128K, 144K) 2 scale
// buffers x (W 4K | A 4K); [144K, 160K) epilogue staging, 4K per wavefront.
#include "brq_device.h"
#include "brq_launch.h"

namespace brq {
namespace tiled {

constexpr int TM = 256, TN = 256, KS = 128;
constexpr int STAGE_BYTES = 32768, OPER_BYTES = 16384;
constexpr int SCALE_BASE = 4 * STAGE_BYTES, SCALE_BUF = 8192, SCALE_OPER = 4096;
constexpr int EPI_BASE = SCALE_BASE + 2 * SCALE_BUF, EPI_WAVE = 4096;
constexpr int LDS_BYTES = EPI_BASE + 4 * EPI_WAVE;   // 163840 = all of a CU's LDS

// One LDS-DMA load: 64 lanes x 16 bytes from base + voff(lane) to LDS lds_addr + 16 * lane.
// lds_addr and base must be wavefront-uniform (they travel in scalar registers / M0).
__device__ __forceinline__ void load_lds16(uint32_t lds_addr, const uint8_t* base, uint32_t voff) {
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    uint64_t b = (uint64_t)base;
    uint32_t blo = __builtin_amdgcn_readfirstlane((uint32_t)b), bhi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    base = (const uint8_t*)(((uint64_t)bhi << 32) | blo);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2\n\t" ::"s"(lds_addr), "v"(voff), "s"(base) : "memory");
}

// Wait until at most N of this wavefront's vector-memory operations are outstanding and all
// its LDS reads have returned, then meet the other wavefronts.
template <int N>
__device__ __forceinline__ void wait_vm_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier\n\t" ::"n"(N) : "memory");
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

#define BRQ_MFMA(ACC, WF, AF, SEL, SW, SA)                                                                  \
    ACC = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(v8i{WF[0], WF[1], WF[2], WF[3], 0, 0, 0, 0},     \
                                                          v8i{AF[0], AF[1], AF[2], AF[3], 0, 0, 0, 0}, ACC, \
                                                          4, 4, SEL, SW, SEL, SA)

template <bool OUT_BF16>
__global__ void __launch_bounds__(256, 1) k_gemm_tiled(const uint8_t* __restrict__ aq, const uint8_t* __restrict__ as,
                                                       const uint8_t* __restrict__ wq, const uint8_t* __restrict__ ws,
                                                       int M, int N, int K, void* __restrict__ y, int64_t ldy) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, h = lane >> 5;
    const int wn = wave >> 1, wm = wave & 1;   // this wavefront's 128 W rows / 128 A rows inside the tile

    TileWalk tw;
    tw.tiles_m = M / TM;
    tw.tiles_n = N / TN;
    {
        const int T = tw.tiles_m * tw.tiles_n, G = gridDim.x;   // G is a multiple of 8
        const int per_xcd = (T + 7) / 8, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        tw.first = xcd * per_xcd + slot;
        tw.end = min((xcd + 1) * per_xcd, T);
        tw.stride = G >> 3;
    }
    const int ntiles = tw.first < tw.end ? (tw.end - tw.first + tw.stride - 1) / tw.stride : 0;
    const int KT = K / KS;                    // stages per tile, a multiple of 4
    const int64_t cpitch = K / 2, spitch = K / 32;

    // per-lane constant parts of the global offsets
    const uint32_t code_voff = (uint32_t)((lane >> 2) * cpitch + (((lane & 3) ^ ((lane >> 4) & 3)) << 4));
    const uint32_t scale_voff = (uint32_t)(lane * spitch);

    // ---- producer: the stage whose loads are issued next, as (stream index, tile, stage in tile)
    int ig = 0, iti = 0, ikt = 0;
    const uint8_t *t_w = nullptr, *t_a = nullptr, *t_ws = nullptr, *t_as = nullptr;   // rows of the producer's tile
    const uint8_t *p_w = nullptr, *p_a = nullptr, *p_ws = nullptr, *p_as = nullptr;   // ... at the producer's stage
    uint32_t p_lds = 0, p_sc = 0;
    bool p_scales = false;
    // Past the end of the stream (iti >= ntiles) the last tile is loaded again: 4 throw-away
    // stages that nobody reads keep the number of loads in flight the same in every iteration.
    auto issue_begin = [&]() {
        if (ikt == 0) {   // new tile: the only place with an integer division
            int tm, tn;
            tw.tile(min(iti, ntiles - 1), tm, tn);
            t_w = wq + ((int64_t)tn * TN + wave * 64) * cpitch;
            t_a = aq + ((int64_t)tm * TM + wave * 64) * cpitch;
            t_ws = ws + ((int64_t)tn * TN + wave * 64) * spitch;
            t_as = as + ((int64_t)tm * TM + wave * 64) * spitch;
        }
        p_lds = lds0 + (ig & 3) * STAGE_BYTES + wave * 4096;
        p_w = t_w + ikt * 64;
        p_a = t_a + ikt * 64;
        p_scales = (ikt & 3) == 0;
        p_sc = lds0 + SCALE_BASE + ((ig >> 2) & 1) * SCALE_BUF + wave * 1024;
        p_ws = t_ws + (ikt >> 2) * 16;
        p_as = t_as + (ikt >> 2) * 16;
        ++ig;
        if (++ikt == KT) { ikt = 0; ++iti; }
    };
    // step 0..7: 16 rows x 64 bytes of codes each (W, A alternating); 8, 9: the scale rows
    auto issue_step = [&](int i) {
        if (i < 8) {
            const int q = i >> 1;
            if (i & 1) load_lds16(p_lds + OPER_BYTES + q * 1024, p_a + q * 16 * cpitch, code_voff);
            else load_lds16(p_lds + q * 1024, p_w + q * 16 * cpitch, code_voff);
        } else if (i == 8) {
            load_lds16(p_sc, p_ws, scale_voff);
        } else {
            load_lds16(p_sc + SCALE_OPER, p_as, scale_voff);
        }
    };
    auto issue_all = [&]() {
        issue_begin();
        if (p_scales) {   // scales first: they are then older than the stage's code loads
            issue_step(8);
            issue_step(9);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) issue_step(i);
    };

    // ---- consumer: MFMA-side LDS offsets (bytes) inside a stage / scale buffer
    const int sw = (r >> 2) & 3;
    uint32_t woff[2], aoff[2];   // chunk of step j, rows of MFMA tile 0; tile t adds 32 rows = 2048 bytes
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        woff[j] = (wn * 128 + r) * 64 + (((2 * h + j) ^ sw) << 4);
        aoff[j] = OPER_BYTES + (wm * 128 + r) * 64 + (((2 * h + j) ^ sw) << 4);
    }
    const uint32_t wsoff = SCALE_BASE + (wn * 128 + r) * 16, asoff = SCALE_BASE + SCALE_OPER + (wm * 128 + r) * 16;
    const int hshift = h * 16;

    v4i w0[4], a0[4], w1[4], a1[4];     // step-0 / step-1 operand fragments
    int sws[4], sas[4], nws[4], nas[4]; // scale registers of the current / next stage
    auto read_frags = [&](int stage, int j, v4i (&wf)[4], v4i (&af)[4]) {
        const uint8_t* st = lds + (stage & 3) * STAGE_BYTES;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            wf[t] = *reinterpret_cast<const v4i*>(st + woff[j] + t * 2048);
            af[t] = *reinterpret_cast<const v4i*>(st + aoff[j] + t * 2048);
        }
    };
    auto read_scales = [&](int stage, int (&sw_)[4], int (&sa_)[4]) {
        const uint8_t* sc = lds + ((stage >> 2) & 1) * SCALE_BUF + (stage & 3) * 4;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            sw_[t] = (int)(*reinterpret_cast<const uint32_t*>(sc + wsoff + t * 512) >> hshift);
            sa_[t] = (int)(*reinterpret_cast<const uint32_t*>(sc + asoff + t * 512) >> hshift);
        }
    };

    if (ntiles == 0) return;   // uniform over the workgroup

    // ---- prologue: 4 stages in flight, first fragments in registers
    issue_all();
    issue_all();
    issue_all();
    issue_all();
    wait_vm_and_barrier<24>();        // the 3 younger stages: 8 code loads each
    read_frags(0, 0, w0, a0);
    read_scales(0, sws, sas);

    int g = 0;
    for (int ti = 0; ti < ntiles; ++ti) {
        v16f acc[4][4];   // [W tile][A tile]
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[a][b] = v16f{};

        for (int kt = 0; kt < KT; ++kt, ++g) {
            // first half: step-1 fragments of this stage stream in behind the step-0 MFMAs
            read_frags(g, 1, w1, a1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) BRQ_MFMA(acc[a][b], w0[a], a0[b], 0, sws[a], sas[b]);
            __builtin_amdgcn_sched_barrier(0);

            // This wavefront has read stage g completely; the next stage must have landed.  The
            // stream is padded with 4 throw-away stages at its end (see issue_begin), so exactly
            // two younger stages (16 code loads) are in flight here, always.
            wait_vm_and_barrier<16>();
            read_frags(g + 1, 0, w0, a0);
            read_scales(g + 1, nws, nas);
            __builtin_amdgcn_sched_barrier(0);

            // second half: step-1 MFMAs, the refill loads spread between them
#pragma unroll
            for (int a = 0; a < 4; ++a) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    BRQ_MFMA(acc[a][b], w1[a], a1[b], 1, sws[a], sas[b]);
                    const int idx = a * 4 + b;
                    if (idx == 0) {
                        issue_begin();                            // stage g+4 goes into stage g's buffer
                        if (p_scales) { issue_step(8); issue_step(9); }
                        __builtin_amdgcn_sched_barrier(0);
                    } else if (idx <= 8) {
                        issue_step(idx - 1);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) { sws[t] = nws[t]; sas[t] = nas[t]; }
        }

        // ---- epilogue: lane (r, h) holds, for W tile a / A tile b, output row m = b*32 + r and
        // columns n = a*32 + 8q + 4h + {0..3}, q = 0..3.  Each wavefront transposes through its
        // own 4 KB of LDS into full 128-byte row segments.
        int ti_e = ti;
        asm volatile("" : "+s"(ti_e));    // keeps the address arithmetic below out of the K loop
        int tm, tn;
        tw.tile(ti_e, tm, tn);
        uint8_t* ep = lds + EPI_BASE + wave * EPI_WAVE;
        const int64_t row0 = (int64_t)tm * TM + wm * 128, col0 = (int64_t)tn * TN + wn * 128;
        const int rr0 = lane >> 3, ck = lane & 7;     // read-back: 16-byte chunk ck of rows rr0 + 8p
        if constexpr (OUT_BF16) {
            // pass = 32 output rows x 64 columns (two W tiles) = 32 x 128 bytes
            uint8_t* yb = reinterpret_cast<uint8_t*>(y) + ((row0 + rr0) * ldy + col0 + ck * 8) * 2;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
#pragma unroll
                for (int ap = 0; ap < 2; ++ap) {
#pragma unroll
                    for (int a2 = 0; a2 < 2; ++a2) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const v16f& c = acc[ap * 2 + a2][b];
                            uint2 pk;
                            pk.x = pack_bf16x2(c[4 * q + 0], c[4 * q + 1]);
                            pk.y = pack_bf16x2(c[4 * q + 2], c[4 * q + 3]);
                            const int c8 = a2 * 8 + 2 * q + h;           // 8-byte column index 0..15
                            *reinterpret_cast<uint2*>(ep + r * 128 + ((c8 ^ ((r & 7) << 1)) << 3)) = pk;
                        }
                    }
                    // staging is private to the wavefront: only its own writes are read back
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const int rr = p * 8 + rr0;
                        uint4 v = *reinterpret_cast<const uint4*>(ep + rr * 128 + ((ck ^ (rr & 7)) << 4));
                        *reinterpret_cast<uint4*>(yb + ((int64_t)(b * 32 + p * 8) * ldy + ap * 64) * 2) = v;
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_sched_barrier(0);    // one pass at a time: keeps register pressure flat
                }
            }
        } else {
            // pass = 32 output rows x 32 columns (one W tile) = 32 x 128 bytes
            uint8_t* yb = reinterpret_cast<uint8_t*>(y) + ((row0 + rr0) * ldy + col0 + ck * 4) * 4;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
#pragma unroll
                for (int a = 0; a < 4; ++a) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const v16f& c = acc[a][b];
                        const int c16 = 2 * q + h;
                        *reinterpret_cast<float4*>(ep + r * 128 + ((c16 ^ (r & 7)) << 4)) =
                            make_float4(c[4 * q], c[4 * q + 1], c[4 * q + 2], c[4 * q + 3]);
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const int rr = p * 8 + rr0;
                        float4 v = *reinterpret_cast<const float4*>(ep + rr * 128 + ((ck ^ (rr & 7)) << 4));
                        *reinterpret_cast<float4*>(yb + ((int64_t)(b * 32 + p * 8) * ldy + a * 32) * 4) = v;
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }
    // the throw-away stages are still in flight: let them land before the LDS is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

#undef BRQ_MFMA

}  // namespace tiled

bool tiled_gemm_supported(int64_t M, int64_t N, int64_t K, bool out_bf16, int64_t ldy) {
    return M > 0 && N > 0 && M % tiled::TM == 0 && N % tiled::TN == 0 && K % 512 == 0 &&
           (ldy * (out_bf16 ? 2 : 4)) % 16 == 0 && (K / 2) * 16 < (int64_t(1) << 31);
}

hipError_t launch_gemm_tiled(const uint8_t* aq, const uint8_t* as, const uint8_t* wq, const uint8_t* ws,
                             int64_t M, int64_t N, int64_t K, void* y, bool out_bf16, int64_t ldy,
                             hipStream_t s) {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        int n = 256;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v >= 8)
            n = v & ~7;
        hipError_t e = hipFuncSetAttribute((const void*)tiled::k_gemm_tiled<true>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, tiled::LDS_BYTES);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void*)tiled::k_gemm_tiled<false>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, tiled::LDS_BYTES);
        if (e != hipSuccess) return e;
        cus = n;
    }
    const int T = (int)((M / tiled::TM) * (N / tiled::TN));
    const int grid = T < cus ? ((T + 7) & ~7) : cus;
    if (out_bf16)
        hipLaunchKernelGGL(tiled::k_gemm_tiled<true>, dim3(grid), dim3(256), tiled::LDS_BYTES, s, aq, as, wq, ws,
                           (int)M, (int)N, (int)K, y, ldy);
    else
        hipLaunchKernelGGL(tiled::k_gemm_tiled<false>, dim3(grid), dim3(256), tiled::LDS_BYTES, s, aq, as, wq, ws,
                           (int)M, (int)N, (int)K, y, ldy);
    return hipGetLastError();
}

}  // namespace brq
