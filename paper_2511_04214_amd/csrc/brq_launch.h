// Host-side launch entry points of the kernel translation units (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace brq {

// mode: 0 rotate, 1 quantize, 2 fused rotate+quantize.  log2b: 0 for quantize, else 5..14.
hipError_t launch_rowwise(int mode, int log2b, bool in_bf16, bool out_bf16, const void* x, int64_t M,
                          int64_t K, int64_t ldx, void* y, int64_t ldy, uint8_t* codes, uint8_t* scales,
                          hipStream_t s);

hipError_t launch_mxfp4_gemm(const uint8_t* aq, const uint8_t* as, const uint8_t* wq, const uint8_t* ws,
                             int64_t M, int64_t N, int64_t K, void* y, bool out_bf16, int64_t ldy,
                             hipStream_t s);

// Persistent LDS-staged kernel for large shapes (M, N multiples of 256, K a multiple of 512).
bool tiled_gemm_supported(int64_t M, int64_t N, int64_t K, bool out_bf16, int64_t ldy);
hipError_t launch_gemm_tiled(const uint8_t* aq, const uint8_t* as, const uint8_t* wq, const uint8_t* ws,
                             int64_t M, int64_t N, int64_t K, void* y, bool out_bf16, int64_t ldy,
                             hipStream_t s);

}  // namespace brq
