// Host-side launch entry points of the kernel translation units (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace brq {

// Per-device facts and one-time set-up.  The launchers size their grids by the number of compute units
// and three kernel families ask for more than the default 64 KB of LDS, which HIP wants declared per
// function and device before the first launch.  device_cus() returns the CU count of the CURRENT device and
// on its first call for that device (under a lock, keyed by the device id) runs the three set-up routines;
// brq_init() is that call made ahead of time.  Nothing else in the library outlives a call.
hipError_t device_cus(int* cus);
hipError_t setup_gemm_tiled();     // mxfp4_gemm_tiled.hip
hipError_t setup_gemm_smallm();    // mxfp4_gemm.hip
hipError_t setup_matrix_rotate();  // matrix_rotate_quant.hip
hipError_t setup_gemm_decode_fused();   // mxfp4_gemm.hip

// mode: 0 rotate, 1 quantize, 2 fused rotate+quantize.  log2b: 0 for quantize, else 3..14.
// tiled: codes and scales go out in the tiled operand layout instead of row-major.
// signs: [K] sign bytes of a randomized rotation (element k negated where signs[k] < 0) or null.
// prod: null, or the gated-activation producer in front of a quantize / fused launch: x is then
// `gate`, prod->up the second matrix, and the kernel works on silu(gate) * up.
struct Producer {
    const void* up;      // [M][ldu], same element type as x
    int64_t ldu;
    bool through_bf16;   // the activation is rounded to bf16 before the rotation
};
// stats: outputs of mode 3 (block statistics of the transformed activation), else null.
struct StatsOut {
    float* amax;                  // [M][K/32] or null
    float* sqerr;                 // [M][K/32] or null
    float* sqerr_bfp4;            // [M][K/32] or null
    unsigned long long* counts;   // [nt], added to, or null
    int nt;                       // 0..8
    const float* thresholds;      // host, nt values
};
// mode 3: statistics (log2b = 0 for "no rotation").
hipError_t launch_rowwise(int mode, int log2b, bool in_bf16, bool out_bf16, const void* x, int64_t M,
                          int64_t K, int64_t ldx, void* y, int64_t ldy, uint8_t* codes, uint8_t* scales,
                          bool tiled, const int8_t* signs, const Producer* prod, hipStream_t s,
                          const StatsOut* stats = nullptr);

// Reduction of per-block statistics (block_summary.hip): histogram of the block scales over `nedges` <= 32
// host-side edges, class counts and fp64 sums split by reference scale > outlier.  Outputs are added to.
hipError_t launch_block_summary(const float* amax, const float* sqerr, const float* ref, int64_t n, float outlier,
                                const float* edges, int nedges, unsigned long long* hist, unsigned long long* counts,
                                double* sums, hipStream_t s);

// Tiled operand whose K is not a multiple of 512: writes the K padding of rows 0..M-1 as zeros.
hipError_t launch_zero_kpad(uint8_t* codes, uint8_t* scales, int64_t M, int64_t K, hipStream_t s);

// Rotation by caller-supplied 32 x 32 blocks R[nR][32][32] (nR = 1 or K/32) on the matrix cores.
// mode 0: y = x R_block (y fp32 or bf16); mode 2: fused with the quantizer.  K % 128 == 0.
hipError_t launch_matrix_rotate(int mode, bool in_bf16, bool out_bf16, const void* x, int64_t M, int64_t K, int64_t ldx,
                                const float* R, int64_t nR, void* y, int64_t ldy, uint8_t* codes, uint8_t* scales,
                                bool tiled, hipStream_t s);

// A quantized [rows][K] operand as the product kernels see it.
struct Operand {
    const uint8_t* codes;
    const uint8_t* scales;
    bool tiled;
};

hipError_t launch_mxfp4_gemm(const Operand& a, const Operand& w, int64_t M, int64_t N, int64_t K, void* y,
                             bool out_bf16, int64_t ldy, hipStream_t s);

// The decode-size product with the online step (B = 32 rotation + quantizer) of its activations in its own
// prologue: x [M <= 16][ldx] bf16 or fp32, K % 512 == 0, K <= DECODE_FUSED_MAX_K (the quantized activations of
// all of K stay in LDS).
constexpr int64_t DECODE_FUSED_MAX_K = 16384;
hipError_t launch_gemm_decode_fused(const void* x, bool in_bf16, int64_t M, int64_t K, int64_t ldx, const int8_t* signs,
                                    const Operand& w, int64_t N, void* y, bool out_bf16, int64_t ldy, hipStream_t s);

// Persistent LDS-staged kernel for large shapes (N a multiple of 256, any M; K a multiple of 512,
// or any K when both operands are tiled, whose K padding is zero).
bool tiled_gemm_supported(int64_t M, int64_t N, int64_t K, bool out_bf16, int64_t ldy, bool both_tiled);
// clk (optional, device): receives the clock read-out of workgroup 0's first wavefront (brq_diag.h).
// no_loads: the measurement variant without refill loads (needs clk, bf16 out and 256 x 256 tiles).
// True if the launcher would take 256 x 256 tiles for this shape on the current device.
hipError_t launch_gemm_tiled(const Operand& a, const Operand& w, int64_t M, int64_t N, int64_t K, void* y,
                             bool out_bf16, int64_t ldy, hipStream_t s, unsigned long long* clk = nullptr,
                             bool no_loads = false);

// Tiled -> row-major copy of a quantized operand.
hipError_t launch_to_rowmajor(const uint8_t* codes_t, const uint8_t* scales_t, int64_t rows, int64_t K,
                              uint8_t* codes, uint8_t* scales, hipStream_t s);

// Measurement aid: `workgroups` x 4 wavefronts, each iters x 16 block-scaled fp4 MFMAs (32x32x64).
hipError_t launch_mfma_ceiling(const uint8_t* operands, int iters, int workgroups, float* sink, hipStream_t s);

}  // namespace brq
