// Block rotation with caller-supplied orthogonal 32 x 32 blocks (Sec. 4.3, Eq. 1 in full:
// R_block = diag(R_1, ..., R_n), every R_i orthogonal; the Hadamard block of the other kernels
// is one choice, learned blocks are what the conclusion proposes for the online step), alone or
// fused with the MXFP4 quantizer of Sec. 4.1.  A dense contraction, so it runs on the matrix
// cores: y_b = x_b R_b is computed as D = R_b^T X_b^T with v_mfma_f32_32x32x16_bf16.
//
// Precision.  bf16 activations are exact MFMA operands.  The fp32 entries of R are split into
// three bf16 parts (hi + mid + lo = R up to 2^-27 relative; each remainder is exact in fp32), fp32
// activations likewise, and the partial products are accumulated in fp32 from the smallest to
// the largest: the result is within a few fp32 roundings of the exact sum, |err| <= 2^-20 *
// sum_i |x_i| |R_ij|.  The order of the additions inside an MFMA is the hardware's, so the
// last bits are not reproducible elsewhere; parity for this kernel is stated with that bound.
//
// Work decomposition.  A wavefront owns 128 columns (four blocks, one stage of the tiled layout) for
// the whole launch and keeps the three bf16 parts of their R (96 VGPRs) in registers; it walks down
// the rows in tiles of 32.
// Operand layout of the 32x32x16 MFMA: lane (m = lane & 31, h = lane >> 5) supplies, as the
// column operand, 8 consecutive k of token row m; MFMA step t = 0, 1 of a block takes
// k = 16 h + 8 t + {0..7} (any assignment of k to lanes and steps is valid as long as R^T uses
// the same one), so a lane reads 32 contiguous bytes of its row per block.  The result leaves
// the matrix core with lane (m, h) holding outputs j = 8 q + 4 h + {0..3}, q = 0..3, of row m:
// half of a 32-element quantization group; the group maximum and the packed codes are
// completed with v_permlane32_swap.
#include "brq_device.h"
#include "brq_launch.h"

namespace brq {
namespace matrot {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct Args {
    const void* x;          // [M][ldx]
    int64_t ldx;
    const float* R;         // [nR][32][32]
    uint32_t shared;        // nR == 1
    uint32_t M, K;
    void* y;                // rotate: [M][ldy] fp32 or bf16
    int64_t ldy;
    uint8_t* codes;
    uint8_t* scales;
    uint32_t stages, sstages;   // tiled output: blocks per slab; 0 = row-major
    uint32_t ntiles, nsplits, ncols;   // row tiles of 32, row walkers per column group, column groups (32 NB columns each)
};

// fp32 -> three bf16 (bits) with hi + mid + lo = f up to 2^-27 |f|; every remainder is exact
__device__ __forceinline__ void split3(float f, uint32_t& hi, uint32_t& mid, uint32_t& lo) {
    hi = f32_to_bf16_bits(f);
    const float r1 = f - as_f32(hi << 16);
    mid = f32_to_bf16_bits(r1);
    const float r2 = r1 - as_f32(mid << 16);
    lo = f32_to_bf16_bits(r2);
}

// 8 fp32 -> three MFMA operands (8 bf16 each, element kk in half (kk & 1) of dword kk >> 1)
__device__ __forceinline__ void split3x8(const float (&f)[8], v4i (&part)[3]) {
    uint32_t p[3][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) split3(f[i], p[0][i], p[1][i], p[2][i]);
#pragma unroll
    for (int s = 0; s < 3; ++s)
        part[s] = v4i{(int)(p[s][0] | (p[s][1] << 16)), (int)(p[s][2] | (p[s][3] << 16)),
                      (int)(p[s][4] | (p[s][5] << 16)), (int)(p[s][6] | (p[s][7] << 16))};
}

__device__ __forceinline__ v16f mfma_bf16(const v4i& a, const v4i& b, const v16f& c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// LDS of one wavefront with NB blocks (32 NB columns): two operand buffers of 32 rows x 64 NB bytes and
// the block the packed codes pass through (32 rows x 16 NB bytes)
constexpr int wave_lds(int NB) { return 2 * (2048 * NB) + 512 * NB; }

// MODE 0: rotation alone (y out), MODE 2: fused with the quantizer.  NB: blocks per wavefront.
//
// Data movement of the bf16 path.  The texture-address unit charges a 64-lane access by the
// cache lines it touches and merges only neighbouring lanes, and in the MFMA's operand layout
// neighbouring lanes are different rows: loading operands straight into that layout (32 lines
// per instruction) and storing codes from it (8 bytes per lane, rows apart) made this kernel
// address-bound at half the memory rate.  So a tile's 32 rows x 64 NB bytes come in by LDS-DMA, 8
// whole lines per instruction (a lane fetches 16-byte chunk p ^ (row & 15) of its row into slot p,
// the XOR spreading the MFMA-side reads over the banks), one tile ahead of the arithmetic; and
// the packed codes go through an LDS block so that NB consecutive lanes store the 16 NB contiguous
// code bytes of a row.  With NB = 4 a wavefront owns a whole 128-element stage: in the tiled
// layout its 32 rows x 64 code bytes are 2 KB of contiguous, whole cache lines (with two blocks it
// wrote half lines that the L2 had to merge with a neighbour's).  All LDS is private to the
// wavefront: no barriers.  Loads and stores share one counter and complete out of order with each
// other, so the wait for the next tile's data is a wait for everything, placed just before this
// tile's stores: by then the loads are a whole tile old and the previous stores older still.
template <bool IN_BF16, int MODE, bool OUT_BF16, int NB>
__global__ void __launch_bounds__(256) k_matrot(Args a) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr uint32_t ROWB = 64u * NB;               // bytes of a tile row (bf16)
    constexpr uint32_t CPR = 4u * NB;                 // 16-byte chunks per tile row
    constexpr uint32_t RPI = 64u / CPR;               // rows per LDS-DMA instruction
    constexpr int NDMA = 32 / RPI;                    // instructions per tile
    constexpr uint32_t TILE = 32u * ROWB;
    constexpr uint32_t SWZ = CPR - 1u;                // chunk p of row i sits in slot p ^ (i & SWZ): 16 consecutive
                                                      // rows of one chunk then cover all 64 banks
    const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t m = lane & 31, h = lane >> 5;
    const uint32_t wid = blockIdx.x * 4u + wave;
    if (wid >= a.ncols * a.nsplits) return;          // uniform per wavefront; no barrier below
    const uint32_t colgrp = wid % a.ncols, split = wid / a.ncols;
    const uint32_t col0 = colgrp * (32u * NB);
    constexpr int ES = IN_BF16 ? 2 : 4;
    uint8_t* const wl = lds + wave * wave_lds(NB);
    const uint32_t wl0 = (uint32_t)(uintptr_t)wl;
    uint8_t* const ep = wl + 2 * TILE;

    // R^T operands of the wavefront's blocks: lane (j = m, h), step t: R[b][16 h + 8 t + kk][j], kk = 0..7
    v4i rp[NB][2][3];
#pragma unroll
    for (int bb = 0; bb < NB; ++bb) {
        const float* Rb = a.R + (a.shared ? 0u : (size_t)(col0 / 32u + bb) * 1024u);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            float f[8];
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) f[kk] = Rb[(16u * h + 8u * t + kk) * 32u + m];
            split3x8(f, rp[bb][t]);
        }
    }

    // bf16: LDS-DMA of a tile into buffer `buf`.  Instruction i brings rows RPI i + lane / CPR; the
    // host checked that 32 rows of pitch fit 32 bits.  Rows past the end re-read the last row.
    const uint32_t pitch = (uint32_t)a.ldx * ES;
    const uint32_t rin = lane / CPR, pos = lane % CPR;
    auto lane_off = [&](uint32_t i, uint32_t last) -> uint32_t {
        const uint32_t row = RPI * i + rin;
        return min(row, last) * pitch + ((pos ^ (row & SWZ)) << 4);
    };
    uint32_t voff[NDMA];
#pragma unroll
    for (int i = 0; i < NDMA; ++i) voff[i] = lane_off(i, 31u);
    auto dma_tile = [&](uint32_t tile, uint32_t buf) {
        const uint8_t* base = uniform_ptr((const uint8_t*)a.x + ((uint64_t)tile * 32u * (uint64_t)a.ldx + col0) * ES);
        const uint32_t lb = wl0 + buf * TILE;
        const bool whole = tile * 32u + 32u <= a.M;   // uniform
        const uint32_t last = whole ? 31u : a.M - 1u - tile * 32u;
#pragma unroll
        for (int i = 0; i < NDMA; ++i) {
            const uint32_t vo = whole ? voff[i] : lane_off(i, last);
            if (i == 0) dma16_stream<0>(lb, base, vo);
            if (i == 1) dma16_stream<1024>(lb, base, vo);
            if (i == 2) dma16_stream<2048>(lb, base, vo);
            if (i == 3) dma16_stream<3072>(lb, base, vo);
            if (i == 4) dma16_stream<4096>(lb, base, vo);
            if (i == 5) dma16_stream<5120>(lb, base, vo);
            if (i == 6) dma16_stream<6144>(lb, base, vo);
            if (i == 7) dma16_stream<7168>(lb, base, vo);
        }
    };
    uint32_t buf = 0;
    if constexpr (IN_BF16) {
        dma_tile(split, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }

    for (uint32_t tile = split; tile < a.ntiles; tile += a.nsplits) {
        const uint32_t row = tile * 32u + m;
        if constexpr (IN_BF16) {
            if (tile + a.nsplits < a.ntiles) dma_tile(tile + a.nsplits, buf ^ 1u);   // uniform
        }
        uint32_t sbv[NB];
        v16f accs[MODE == 0 ? NB : 1];
#pragma unroll
        for (int bb = 0; bb < NB; ++bb) {
            sbv[bb] = 0;
            v16f acc = {};
            if constexpr (IN_BF16) {
                const uint8_t* src = wl + buf * TILE + m * ROWB;
                const v4i x0 = *reinterpret_cast<const v4i*>(src + (((uint32_t)(bb * 4) + 2u * h) ^ (m & SWZ)) * 16u);
                const v4i x1 = *reinterpret_cast<const v4i*>(src + (((uint32_t)(bb * 4) + 2u * h + 1u) ^ (m & SWZ)) * 16u);
#pragma unroll
                for (int s = 2; s >= 0; --s) {        // smallest part first
                    acc = mfma_bf16(rp[bb][0][s], x0, acc);
                    acc = mfma_bf16(rp[bb][1][s], x1, acc);
                }
            } else {
                // fp32 activations (not the fast path): straight from global into the operand layout
                const uint32_t lrow = min(row, a.M - 1u);
                const char* xp = (const char*)a.x + ((uint64_t)lrow * (uint64_t)a.ldx + col0 + 16u * h) * ES;
                v4i xs[2][3];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const v4f lo = *reinterpret_cast<const v4f*>(xp + bb * 128 + t * 32);
                    const v4f hi = *reinterpret_cast<const v4f*>(xp + bb * 128 + t * 32 + 16);
                    const float f[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    split3x8(f, xs[t]);
                }
                // the six products whose parts' orders add up to at most 2 (the rest is below 2^-27)
                constexpr int PX[6] = {2, 0, 1, 1, 0, 0}, PR[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
                for (int i = 0; i < 6; ++i) {
                    acc = mfma_bf16(rp[bb][0][PR[i]], xs[0][PX[i]], acc);
                    acc = mfma_bf16(rp[bb][1][PR[i]], xs[1][PX[i]], acc);
                }
            }
            // acc[4 q + i] = y[row][col0 + 32 bb + 8 q + 4 h + i]
            const uint32_t cb = col0 + 32u * bb;
            if constexpr (MODE == 0) {
                accs[bb] = acc;
            } else {
                const float lo8[8] = {acc[0], acc[1], acc[2], acc[3], acc[4], acc[5], acc[6], acc[7]};
                const float hi8[8] = {acc[8], acc[9], acc[10], acc[11], acc[12], acc[13], acc[14], acc[15]};
                // group maximum: own 16 values, then the other half of the row's group (lane ^ 32);
                // non-negative floats order like their bit patterns
                const uint32_t am = as_u32(fmaxf(absmax8(lo8), absmax8(hi8)));
                const auto ex = __builtin_amdgcn_permlane32_swap(am, am, false, false);
                const uint32_t sb = e8m0_from_amax(as_f32(max(ex[0], ex[1])));
                sbv[bb] = sb;
                // U: codes of q = 0, 1 (two 16-bit pieces), V: of q = 2, 3.  After the swap lane h = 0
                // holds both lanes' U (group bytes 0..7), lane h = 1 both lanes' V (bytes 8..15);
                // piece (q, h) belongs at byte 4 q + 2 h of the group
                const uint32_t U = encode8_e2m1(lo8, sb), V = encode8_e2m1(hi8, sb);
                const auto sw = __builtin_amdgcn_permlane32_swap(U, V, false, false);
                const uint2 o = make_uint2((sw[0] & 0xffffu) | (sw[1] << 16), (sw[0] >> 16) | (sw[1] & 0xffff0000u));
                // row m, block bb, half h.  A row of the code block is 16 NB bytes: rows 4 apart would meet in
                // the same banks (8 of a wavefront's 32 rows per bank group), so the 16-byte piece of block bb
                // sits in slot bb ^ (m >> 2) of its row
                *reinterpret_cast<uint2*>(ep + m * (16u * NB) + (((uint32_t)bb ^ ((m >> 2) & (NB - 1u))) << 4) + 8u * h) = o;
            }
        }
        if constexpr (MODE == 0) {
            // The rotated values leave through LDS too: in the accumulator layout a lane holds 4 consecutive
            // columns of its own row, rows apart between neighbouring lanes (stored from there the kernel ran
            // at a third of the memory rate).  The tile goes, 256 bytes of every row at a time (all 128 bf16
            // columns, or 64 fp32 columns = two of the four blocks), into the operand buffer that this tile's
            // MFMAs have finished reading (LDS operations of a wavefront execute in order; fp32 input has no
            // operand buffers), 16-byte piece p of row i at i * 256 + ((p ^ (i & 15)) << 4); it is read back
            // with 16 consecutive lanes per row and stored as 4 rows x 256 contiguous bytes per instruction.
            static_assert(NB == 4, "the staging below is laid out for 128 columns per wavefront");
            uint8_t* const st = wl + (IN_BF16 ? buf * TILE : 0u);
            constexpr int ROUNDS = OUT_BF16 ? 1 : 2;
            constexpr int OES = OUT_BF16 ? 2 : 4;
            const uint32_t rrow = lane >> 4, rp16 = lane & 15u;
#pragma unroll
            for (int rd = 0; rd < ROUNDS; ++rd) {
#pragma unroll
                for (int b2 = 0; b2 < NB / ROUNDS; ++b2) {
                    const v16f& c = accs[rd * (NB / ROUNDS) + b2];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if constexpr (OUT_BF16) {      // 8 bytes: half h of piece 4 b2 + q
                            const uint2 o = make_uint2(pack_bf16x2(c[4 * q], c[4 * q + 1]), pack_bf16x2(c[4 * q + 2], c[4 * q + 3]));
                            *reinterpret_cast<uint2*>(st + m * 256u + ((((uint32_t)(4 * b2 + q)) ^ (m & 15u)) << 4) + 8u * h) = o;
                        } else {                       // 16 bytes: piece 8 b2 + 2 q + h
                            *reinterpret_cast<float4*>(st + m * 256u + ((((uint32_t)(8 * b2 + 2 * q) + h) ^ (m & 15u)) << 4)) =
                                make_float4(c[4 * q], c[4 * q + 1], c[4 * q + 2], c[4 * q + 3]);
                        }
                    }
                }
                v4i o[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t r = rrow + 4u * j;
                    o[j] = *reinterpret_cast<const v4i*>(st + r * 256u + ((rp16 ^ (r & 15u)) << 4));
                }
                // next tile landed, earlier stores done (loads and stores share one counter)
                if constexpr (IN_BF16) { if (rd == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t orow = tile * 32u + rrow + 4u * j;
                    if (orow < a.M) {
                        char* dst = (char*)a.y + ((uint64_t)orow * (uint64_t)a.ldy + col0) * OES + rd * 256 + rp16 * 16u;
                        __builtin_nontemporal_store(o[j], reinterpret_cast<v4i*>(dst));
                    }
                }
            }
        }
        if constexpr (MODE == 2) {
            // 16-byte piece L of the code block is row L / NB, block L % NB: lane l takes pieces l, l + 64, ...
            v4i wv[NB / 2];
#pragma unroll
            for (int k = 0; k < NB / 2; ++k) {      // (the reader undoes the slot swizzle: NB lanes read one whole row)
                const uint32_t piece = lane + 64u * k, prow = piece / NB, pb = piece % NB;
                wv[k] = *reinterpret_cast<const v4i*>(ep + prow * (16u * NB) + ((pb ^ ((prow >> 2) & (NB - 1u))) << 4));
            }
            if constexpr (IN_BF16) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // next tile landed, earlier stores done
            const uint32_t g0 = col0 / 32u;
#pragma unroll
            for (int k = 0; k < NB / 2; ++k) {
                const uint32_t piece = lane + 64u * k;
                const uint32_t srow = tile * 32u + piece / NB, g = g0 + piece % NB;
                if (srow < a.M) {
                    uint8_t* dst = a.stages == 0
                                       ? a.codes + (uint64_t)srow * (a.K / 2u) + g * 16u
                                       : a.codes + ((uint64_t)(srow >> 6) * a.stages + (g >> 2)) * 4096u + (srow & 63u) * 64u + (g & 3u) * 16u;
                    if constexpr (NB == 4) __builtin_nontemporal_store(wv[k], reinterpret_cast<v4i*>(dst));   // whole lines
                    else *reinterpret_cast<v4i*>(dst) = wv[k];
                }
            }
            if (h == 0 && row < a.M) {
                uint8_t* dst = a.stages == 0 ? a.scales + (uint64_t)row * (a.K / 32u) + g0
                                             : a.scales + ((uint64_t)(row >> 6) * a.sstages + (g0 >> 4)) * 1024u + (row & 63u) * 16u + (g0 & 15u);
                if constexpr (NB == 4)
                    *reinterpret_cast<uint32_t*>(dst) = sbv[0] | (sbv[1] << 8) | (sbv[2 % NB] << 16) | (sbv[3 % NB] << 24);
                else
                    *reinterpret_cast<uint16_t*>(dst) = (uint16_t)(sbv[0] | (sbv[1] << 8));
            }
        }
        buf ^= 1u;
    }
}

}  // namespace matrot

// The kernels use 72 KB of LDS per workgroup: declared once per device.
hipError_t setup_matrix_rotate() {
    constexpr int NB = 4, LDS = 4 * matrot::wave_lds(NB);
    const void* kernels[6] = {(const void*)matrot::k_matrot<true, 0, true, NB>, (const void*)matrot::k_matrot<true, 0, false, NB>,
                              (const void*)matrot::k_matrot<false, 0, true, NB>, (const void*)matrot::k_matrot<false, 0, false, NB>,
                              (const void*)matrot::k_matrot<true, 2, false, NB>, (const void*)matrot::k_matrot<false, 2, false, NB>};
    for (const void* k : kernels)
        if (hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, LDS); e != hipSuccess) return e;
    return hipSuccess;
}

// mode 0: rotation alone into y; mode 2: fused with the quantizer into codes / scales.
// K % 128 == 0 (checked by the caller), nR = 1 or K / 32.
hipError_t launch_matrix_rotate(int mode, bool in_bf16, bool out_bf16, const void* x, int64_t M, int64_t K, int64_t ldx,
                                const float* R, int64_t nR, void* y, int64_t ldy, uint8_t* codes, uint8_t* scales,
                                bool tiled, hipStream_t s) {
    int cus = 0;
    if (hipError_t e = device_cus(&cus); e != hipSuccess) return e;
    matrot::Args a;
    a.x = x; a.ldx = ldx; a.R = R; a.shared = nR == 1 ? 1u : 0u;
    a.M = (uint32_t)M; a.K = (uint32_t)K; a.y = y; a.ldy = ldy; a.codes = codes; a.scales = scales;
    const int64_t Kp = (K + 511) / 512 * 512;
    a.stages = tiled ? (uint32_t)(Kp / 128) : 0u;
    a.sstages = tiled ? (uint32_t)(Kp / 512) : 0u;
    a.ntiles = (uint32_t)((M + 31) / 32);
    constexpr int NB = 4;                                  // blocks per wavefront: one 128-element stage
    a.ncols = (uint32_t)(K / (32 * NB));
    // about 8 wavefronts per CU (two workgroups fit its LDS); a wavefront keeps its R for at least 4 row
    // tiles when there are that many
    uint32_t want = (uint32_t)cus * 8u / a.ncols;
    if (want < 1) want = 1;
    const uint32_t most = (a.ntiles + 3u) / 4u;
    a.nsplits = want < most ? want : most;
    if (mode == 2 && tiled && Kp != K) {
        hipError_t e = launch_zero_kpad(codes, scales, M, K, s);
        if (e != hipSuccess) return e;
    }
    constexpr int LDS = 4 * matrot::wave_lds(NB);          // 72 KB: above the default limit (setup_matrix_rotate)
    const dim3 grid((a.ncols * a.nsplits + 3u) / 4u), block(256);
    if (mode == 0) {
        if (in_bf16) {
            if (out_bf16) hipLaunchKernelGGL((matrot::k_matrot<true, 0, true, NB>), grid, block, LDS, s, a);
            else hipLaunchKernelGGL((matrot::k_matrot<true, 0, false, NB>), grid, block, LDS, s, a);
        } else {
            if (out_bf16) hipLaunchKernelGGL((matrot::k_matrot<false, 0, true, NB>), grid, block, LDS, s, a);
            else hipLaunchKernelGGL((matrot::k_matrot<false, 0, false, NB>), grid, block, LDS, s, a);
        }
    } else {
        if (in_bf16) hipLaunchKernelGGL((matrot::k_matrot<true, 2, false, NB>), grid, block, LDS, s, a);
        else hipLaunchKernelGGL((matrot::k_matrot<false, 2, false, NB>), grid, block, LDS, s, a);
    }
    return hipGetLastError();
}

}  // namespace brq
