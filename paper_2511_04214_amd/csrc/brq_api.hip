// extern "C" boundary of the library: argument validation on the host, then a kernel launch
// on the caller's stream.  No allocation, no host synchronisation; the only state is the per-device
// set-up record below.
#include <mutex>

#include "../../include/brq.h"
#include "../../include/brq_diag.h"
#include "brq_launch.h"

namespace brq {

namespace {
std::mutex g_device_mu;
struct DeviceSlot { bool ready; int cus; } g_device[64];
}  // namespace

hipError_t device_cus(int* cus) {
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_device_mu);
    DeviceSlot& slot = g_device[dev];
    if (!slot.ready) {
        int v = 0;
        if (hipError_t e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev); e != hipSuccess) return e;
        if (v <= 0) return hipErrorInvalidDevice;
        if (hipError_t e = setup_gemm_tiled(); e != hipSuccess) return e;
        if (hipError_t e = setup_gemm_smallm(); e != hipSuccess) return e;
        if (hipError_t e = setup_matrix_rotate(); e != hipSuccess) return e;
        if (hipError_t e = setup_gemm_decode_fused(); e != hipSuccess) return e;
        slot.cus = v;
        slot.ready = true;
    }
    *cus = slot.cus;
    return hipSuccess;
}

}  // namespace brq

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
int dtype_size(brq_dtype d) { return d == BRQ_F32 ? 4 : (d == BRQ_BF16 ? 2 : 0); }

// log2 of the rotation block, or -1 if B is not an accepted block size for this K
int block_log2(int64_t B, int64_t K) {
    if (B < 8 || B > 16384 || (B & (B - 1)) != 0 || K % B != 0) return -1;
    int l = 0;
    while ((int64_t(1) << l) < B) ++l;
    return l;
}

// An empty matrix (M == 0) may come with a NULL pointer; everything else is still checked.
brq_status check_rows(const void* x, brq_dtype dt, int64_t M, int64_t K, int64_t ld) {
    int es = dtype_size(dt);
    if (es == 0) return BRQ_ERR_DTYPE;
    if (M < 0 || K <= 0 || K % 32 != 0 || ld < K) return BRQ_ERR_SHAPE;
    if (K >= (int64_t(1) << 31) || M >= (int64_t(1) << 31) || M * (K / 8) >= (int64_t(1) << 31)) return BRQ_ERR_SHAPE;
    if (M > 0 && !x) return BRQ_ERR_NULL;
    if (!aligned16(x) || (ld * es) % 16 != 0) return BRQ_ERR_ALIGN;
    return BRQ_OK;
}

brq_status check_out(const uint8_t* codes, const uint8_t* scales, int64_t M) {
    if (M > 0 && (!codes || !scales)) return BRQ_ERR_NULL;
    if (!aligned16(codes) || !aligned16(scales)) return BRQ_ERR_ALIGN;
    return BRQ_OK;
}

bool layout_ok(brq_layout l) { return l == BRQ_LAYOUT_ROWMAJOR || l == BRQ_LAYOUT_TILED; }

brq_status launched(hipError_t e) { return e == hipSuccess ? BRQ_OK : BRQ_ERR_LAUNCH; }

}  // namespace

extern "C" {

brq_status brq_init(void) {
    int cus = 0;
    return brq::device_cus(&cus) == hipSuccess ? BRQ_OK : BRQ_ERR_DEVICE;
}

brq_status brq_block_rotate(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx, int64_t B,
                            const int8_t* signs, void* y, brq_dtype ydt, int64_t ldy, void* stream) {
    brq_status st = check_rows(x, xdt, M, K, ldx);
    if (st != BRQ_OK) return st;
    st = check_rows(y, ydt, M, K, ldy);
    if (st != BRQ_OK) return st;
    if (!aligned16(signs)) return BRQ_ERR_ALIGN;
    int l2 = block_log2(B, K);
    if (l2 < 0) return BRQ_ERR_BLOCK;
    if (M == 0) return BRQ_OK;
    return launched(brq::launch_rowwise(0, l2, xdt == BRQ_BF16, ydt == BRQ_BF16, x, M, K, ldx, y, ldy, nullptr,
                                        nullptr, false, signs, nullptr, static_cast<hipStream_t>(stream)));
}

brq_status brq_operand_bytes(int64_t rows, int64_t K, brq_layout layout, int64_t* codes_bytes,
                             int64_t* scales_bytes) {
    if (rows < 0 || K <= 0 || K % 32 != 0) return BRQ_ERR_SHAPE;
    if (!layout_ok(layout)) return BRQ_ERR_LAYOUT;
    int64_t r = rows, k = K;
    if (layout == BRQ_LAYOUT_TILED) {
        r = (rows + 63) / 64 * 64;
        k = (K + 511) / 512 * 512;
    }
    if (codes_bytes) *codes_bytes = r * (k / 2);
    if (scales_bytes) *scales_bytes = r * (k / 32);
    return BRQ_OK;
}

brq_status brq_mxfp4_quantize(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx, uint8_t* codes,
                              uint8_t* scales, brq_layout layout, void* stream) {
    brq_status st = check_rows(x, xdt, M, K, ldx);
    if (st != BRQ_OK) return st;
    if (!layout_ok(layout)) return BRQ_ERR_LAYOUT;
    st = check_out(codes, scales, M);
    if (st != BRQ_OK) return st;
    if (M == 0) return BRQ_OK;
    return launched(brq::launch_rowwise(1, 0, xdt == BRQ_BF16, false, x, M, K, ldx, nullptr, 0, codes, scales,
                                        layout == BRQ_LAYOUT_TILED, nullptr, nullptr, static_cast<hipStream_t>(stream)));
}

brq_status brq_rotate_quantize_fused(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx, int64_t B,
                                     const int8_t* signs, uint8_t* codes, uint8_t* scales, brq_layout layout,
                                     void* stream) {
    brq_status st = check_rows(x, xdt, M, K, ldx);
    if (st != BRQ_OK) return st;
    if (!layout_ok(layout)) return BRQ_ERR_LAYOUT;
    if (!aligned16(signs)) return BRQ_ERR_ALIGN;
    st = check_out(codes, scales, M);
    if (st != BRQ_OK) return st;
    int l2 = block_log2(B, K);
    if (l2 < 0) return BRQ_ERR_BLOCK;
    if (M == 0) return BRQ_OK;
    return launched(brq::launch_rowwise(2, l2, xdt == BRQ_BF16, false, x, M, K, ldx, nullptr, 0, codes, scales,
                                        layout == BRQ_LAYOUT_TILED, signs, nullptr, static_cast<hipStream_t>(stream)));
}

brq_status brq_swiglu(const void* gate, const void* up, brq_dtype xdt, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                      void* h, brq_dtype hdt, int64_t ldh, void* stream) {
    brq_status st = check_rows(gate, xdt, M, K, ldg);
    if (st != BRQ_OK) return st;
    st = check_rows(up, xdt, M, K, ldu);
    if (st != BRQ_OK) return st;
    st = check_rows(h, hdt, M, K, ldh);
    if (st != BRQ_OK) return st;
    if (M == 0) return BRQ_OK;
    const brq::Producer prod{up, ldu, false};
    return launched(brq::launch_rowwise(0, 0, xdt == BRQ_BF16, hdt == BRQ_BF16, gate, M, K, ldg, h, ldh, nullptr, nullptr,
                                        false, nullptr, &prod, static_cast<hipStream_t>(stream)));
}

brq_status brq_swiglu_rotate_quantize_fused(const void* gate, const void* up, brq_dtype xdt, int64_t M, int64_t K,
                                            int64_t ldg, int64_t ldu, brq_dtype hdt, int64_t B, const int8_t* signs,
                                            uint8_t* codes, uint8_t* scales, brq_layout layout, void* stream) {
    brq_status st = check_rows(gate, xdt, M, K, ldg);
    if (st != BRQ_OK) return st;
    st = check_rows(up, xdt, M, K, ldu);
    if (st != BRQ_OK) return st;
    if (dtype_size(hdt) == 0) return BRQ_ERR_DTYPE;
    if (!layout_ok(layout)) return BRQ_ERR_LAYOUT;
    if (!aligned16(signs)) return BRQ_ERR_ALIGN;
    st = check_out(codes, scales, M);
    if (st != BRQ_OK) return st;
    const int l2 = (B == 1) ? 0 : block_log2(B, K);   // B = 1: H_1 = [1], the quantizer alone
    if (l2 < 0 || (B == 1 && signs)) return BRQ_ERR_BLOCK;
    if (M == 0) return BRQ_OK;
    const brq::Producer prod{up, ldu, hdt == BRQ_BF16};
    return launched(brq::launch_rowwise(B == 1 ? 1 : 2, l2, xdt == BRQ_BF16, false, gate, M, K, ldg, nullptr, 0, codes,
                                        scales, layout == BRQ_LAYOUT_TILED, signs, &prod,
                                        static_cast<hipStream_t>(stream)));
}

brq_status brq_block_stats(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx, int64_t B,
                           const int8_t* signs, const float* thresholds, int64_t nt, float* amax,
                           uint64_t* count_gt, float* sqerr, float* sqerr_bfp4, void* stream) {
    brq_status st = check_rows(x, xdt, M, K, ldx);
    if (st != BRQ_OK) return st;
    if (nt < 0 || nt > 8) return BRQ_ERR_SHAPE;
    if (nt > 0 && count_gt && !thresholds) return BRQ_ERR_NULL;
    if (!aligned16(signs) || !aligned16(amax) || !aligned16(sqerr) || !aligned16(sqerr_bfp4) || (reinterpret_cast<uintptr_t>(count_gt) & 7u))
        return BRQ_ERR_ALIGN;
    const int l2 = (B == 1) ? 0 : block_log2(B, K);
    if (l2 < 0 || (B == 1 && signs)) return BRQ_ERR_BLOCK;
    if (M == 0) return BRQ_OK;
    const brq::StatsOut so{amax, sqerr, sqerr_bfp4, reinterpret_cast<unsigned long long*>(count_gt), count_gt ? (int)nt : 0, thresholds};
    return launched(brq::launch_rowwise(3, l2, xdt == BRQ_BF16, false, x, M, K, ldx, nullptr, 0, nullptr, nullptr, false,
                                        signs, nullptr, static_cast<hipStream_t>(stream), &so));
}

brq_status brq_block_stats_summary(const float* amax, const float* sqerr, const float* amax_ref, int64_t nblocks,
                                   float outlier_threshold, const float* edges, int64_t nedges, uint64_t* hist,
                                   uint64_t* counts, double* sums, void* stream) {
    if (nblocks < 0 || nedges < 0 || nedges > 32) return BRQ_ERR_SHAPE;
    if (nblocks > 0 && !amax) return BRQ_ERR_NULL;
    if (nedges > 0 && hist && !edges) return BRQ_ERR_NULL;
    if (hist)
        for (int64_t e = 1; e < nedges; ++e)
            if (!(edges[e - 1] <= edges[e])) return BRQ_ERR_SHAPE;      // edges ascend (and are not NaN)
    const uintptr_t a4 = reinterpret_cast<uintptr_t>(amax) | reinterpret_cast<uintptr_t>(sqerr) | reinterpret_cast<uintptr_t>(amax_ref);
    const uintptr_t a8 = reinterpret_cast<uintptr_t>(hist) | reinterpret_cast<uintptr_t>(counts) | reinterpret_cast<uintptr_t>(sums);
    if ((a4 & 3u) || (a8 & 7u)) return BRQ_ERR_ALIGN;
    if (nblocks == 0 || (!hist && !counts && !sums)) return BRQ_OK;
    return launched(brq::launch_block_summary(amax, sqerr, amax_ref, nblocks, outlier_threshold, edges, (int)nedges,
                                              reinterpret_cast<unsigned long long*>(hist),
                                              reinterpret_cast<unsigned long long*>(counts), sums,
                                              static_cast<hipStream_t>(stream)));
}

static brq_status check_blocks(const float* R, int64_t nR, int64_t K, int64_t ld_bytes) {
    if (K % 128 != 0 || ld_bytes * 32 >= (int64_t(1) << 32)) return BRQ_ERR_SHAPE;   // 32 rows of pitch: 32-bit offsets
    if (nR != 1 && nR != K / 32) return BRQ_ERR_BLOCK;
    if (!R) return BRQ_ERR_NULL;
    if (!aligned16(R)) return BRQ_ERR_ALIGN;
    return BRQ_OK;
}

brq_status brq_matrix_rotate(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx, const float* R, int64_t nR,
                             void* y, brq_dtype ydt, int64_t ldy, void* stream) {
    brq_status st = check_rows(x, xdt, M, K, ldx);
    if (st != BRQ_OK) return st;
    st = check_rows(y, ydt, M, K, ldy);
    if (st != BRQ_OK) return st;
    st = check_blocks(R, nR, K, ldx * dtype_size(xdt));
    if (st != BRQ_OK) return st;
    if (M == 0) return BRQ_OK;
    return launched(brq::launch_matrix_rotate(0, xdt == BRQ_BF16, ydt == BRQ_BF16, x, M, K, ldx, R, nR, y, ldy, nullptr,
                                              nullptr, false, static_cast<hipStream_t>(stream)));
}

brq_status brq_matrix_rotate_quantize_fused(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx,
                                            const float* R, int64_t nR, uint8_t* codes, uint8_t* scales,
                                            brq_layout layout, void* stream) {
    brq_status st = check_rows(x, xdt, M, K, ldx);
    if (st != BRQ_OK) return st;
    if (!layout_ok(layout)) return BRQ_ERR_LAYOUT;
    st = check_out(codes, scales, M);
    if (st != BRQ_OK) return st;
    st = check_blocks(R, nR, K, ldx * dtype_size(xdt));
    if (st != BRQ_OK) return st;
    if (M == 0) return BRQ_OK;
    return launched(brq::launch_matrix_rotate(2, xdt == BRQ_BF16, false, x, M, K, ldx, R, nR, nullptr, 0, codes, scales,
                                              layout == BRQ_LAYOUT_TILED, static_cast<hipStream_t>(stream)));
}

static brq_status check_gemm(const uint8_t* aq, const uint8_t* as, brq_layout a_layout, const uint8_t* wq,
                             const uint8_t* ws, brq_layout w_layout, int64_t M, int64_t N, int64_t K, const void* y,
                             brq_dtype ydt, int64_t ldy) {
    int es = dtype_size(ydt);
    if (es == 0) return BRQ_ERR_DTYPE;
    if (!layout_ok(a_layout) || !layout_ok(w_layout)) return BRQ_ERR_LAYOUT;
    if (M < 0 || N < 0 || K <= 0 || K % 32 != 0 || ldy < N) return BRQ_ERR_SHAPE;
    if (M >= (int64_t(1) << 31) || N >= (int64_t(1) << 31) || K >= (int64_t(1) << 31)) return BRQ_ERR_SHAPE;
    if (M > 0 && N > 0 && (!aq || !as || !wq || !ws || !y)) return BRQ_ERR_NULL;
    if (!aligned16(aq) || !aligned16(as) || !aligned16(wq) || !aligned16(ws) || !aligned16(y))
        return BRQ_ERR_ALIGN;
    return BRQ_OK;
}

brq_status brq_diag_mxfp4_gemm_clock(const uint8_t* aq, const uint8_t* as, brq_layout a_layout, const uint8_t* wq,
                                     const uint8_t* ws, brq_layout w_layout, int64_t M, int64_t N, int64_t K, void* y,
                                     brq_dtype ydt, int64_t ldy, uint64_t* clock, void* stream) {
    brq_status st = check_gemm(aq, as, a_layout, wq, ws, w_layout, M, N, K, y, ydt, ldy);
    if (st != BRQ_OK) return st;
    if (!clock) return BRQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(clock) & 7u) return BRQ_ERR_ALIGN;
    const bool both = a_layout == BRQ_LAYOUT_TILED && w_layout == BRQ_LAYOUT_TILED;
    if (M <= 128 || !brq::tiled_gemm_supported(M, N, K, ydt == BRQ_BF16, ldy, both)) return BRQ_ERR_SHAPE;
    const brq::Operand a{aq, as, a_layout == BRQ_LAYOUT_TILED}, w{wq, ws, w_layout == BRQ_LAYOUT_TILED};
    return launched(brq::launch_gemm_tiled(a, w, M, N, K, y, ydt == BRQ_BF16, ldy, static_cast<hipStream_t>(stream),
                                           reinterpret_cast<unsigned long long*>(clock)));
}

brq_status brq_diag_mxfp4_gemm_no_loads(const uint8_t* aq, const uint8_t* as, brq_layout a_layout, const uint8_t* wq,
                                        const uint8_t* ws, brq_layout w_layout, int64_t M, int64_t N, int64_t K, void* y,
                                        brq_dtype ydt, int64_t ldy, uint64_t* clock, void* stream) {
    brq_status st = check_gemm(aq, as, a_layout, wq, ws, w_layout, M, N, K, y, ydt, ldy);
    if (st != BRQ_OK) return st;
    if (!clock) return BRQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(clock) & 7u) return BRQ_ERR_ALIGN;
    const bool both = a_layout == BRQ_LAYOUT_TILED && w_layout == BRQ_LAYOUT_TILED;
    // bf16 output and at least 256 tiles of 256 x 256 (whatever the device: the launcher then takes that tile)
    if (ydt != BRQ_BF16 || M <= 128 || !brq::tiled_gemm_supported(M, N, K, true, ldy, both) ||
        ((M + 255) / 256) * ((N + 255) / 256) < 1024) return BRQ_ERR_SHAPE;
    const brq::Operand a{aq, as, a_layout == BRQ_LAYOUT_TILED}, w{wq, ws, w_layout == BRQ_LAYOUT_TILED};
    return launched(brq::launch_gemm_tiled(a, w, M, N, K, y, true, ldy, static_cast<hipStream_t>(stream),
                                           reinterpret_cast<unsigned long long*>(clock), true));
}

brq_status brq_mxfp4_gemm(const uint8_t* aq, const uint8_t* as, brq_layout a_layout, const uint8_t* wq,
                          const uint8_t* ws, brq_layout w_layout, int64_t M, int64_t N, int64_t K, void* y,
                          brq_dtype ydt, int64_t ldy, void* stream) {
    brq_status st = check_gemm(aq, as, a_layout, wq, ws, w_layout, M, N, K, y, ydt, ldy);
    if (st != BRQ_OK) return st;
    if (M == 0 || N == 0) return BRQ_OK;
    const brq::Operand a{aq, as, a_layout == BRQ_LAYOUT_TILED}, w{wq, ws, w_layout == BRQ_LAYOUT_TILED};
    return launched(brq::launch_mxfp4_gemm(a, w, M, N, K, y, ydt == BRQ_BF16, ldy, static_cast<hipStream_t>(stream)));
}

brq_status brq_rotate_quantize_gemm_fused(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx, int64_t B,
                                          const int8_t* signs, const uint8_t* wq, const uint8_t* ws, brq_layout w_layout,
                                          int64_t N, void* y, brq_dtype ydt, int64_t ldy, void* stream) {
    brq_status st = check_rows(x, xdt, M, K, ldx);
    if (st != BRQ_OK) return st;
    if (dtype_size(ydt) == 0) return BRQ_ERR_DTYPE;
    if (!layout_ok(w_layout)) return BRQ_ERR_LAYOUT;
    if (M > 16 || N < 0 || N >= (int64_t(1) << 31) || K % 512 != 0 || K > brq::DECODE_FUSED_MAX_K || ldy < N) return BRQ_ERR_SHAPE;
    if (B != 32) return BRQ_ERR_BLOCK;
    if (M > 0 && N > 0 && (!wq || !ws || !y)) return BRQ_ERR_NULL;
    if (!aligned16(signs) || !aligned16(wq) || !aligned16(ws) || !aligned16(y)) return BRQ_ERR_ALIGN;
    if (M == 0 || N == 0) return BRQ_OK;
    const brq::Operand w{wq, ws, w_layout == BRQ_LAYOUT_TILED};
    return launched(brq::launch_gemm_decode_fused(x, xdt == BRQ_BF16, M, K, ldx, signs, w, N, y, ydt == BRQ_BF16, ldy,
                                                  static_cast<hipStream_t>(stream)));
}

brq_status brq_to_rowmajor(const uint8_t* codes_tiled, const uint8_t* scales_tiled, int64_t rows, int64_t K,
                           uint8_t* codes_out, uint8_t* scales_out, void* stream) {
    if (rows < 0 || K <= 0 || K % 32 != 0) return BRQ_ERR_SHAPE;
    if (rows >= (int64_t(1) << 31) || K >= (int64_t(1) << 31)) return BRQ_ERR_SHAPE;
    if (rows > 0 && (!codes_tiled || !scales_tiled || !codes_out || !scales_out)) return BRQ_ERR_NULL;
    if (!aligned16(codes_tiled) || !aligned16(scales_tiled) || !aligned16(codes_out) || !aligned16(scales_out))
        return BRQ_ERR_ALIGN;
    if (rows == 0) return BRQ_OK;
    return launched(brq::launch_to_rowmajor(codes_tiled, scales_tiled, rows, K, codes_out, scales_out,
                                            static_cast<hipStream_t>(stream)));
}

brq_status brq_diag_mfma_ceiling(const uint8_t* operands, int64_t iters, int64_t workgroups, float* sink,
                                 void* stream) {
    if (iters < 0 || iters >= (int64_t(1) << 31) || workgroups < 0 || workgroups > 65536) return BRQ_ERR_SHAPE;
    if (!operands || !sink) return BRQ_ERR_NULL;
    if (!aligned16(operands) || !aligned16(sink)) return BRQ_ERR_ALIGN;
    if (workgroups == 0) return BRQ_OK;
    return launched(brq::launch_mfma_ceiling(operands, (int)iters, (int)workgroups, sink,
                                             static_cast<hipStream_t>(stream)));
}

const char* brq_strerror(brq_status s) {
    switch (s) {
        case BRQ_OK: return "ok";
        case BRQ_ERR_NULL: return "a required pointer is NULL";
        case BRQ_ERR_SHAPE: return "bad shape: negative size, K not a multiple of 32, pitch below row length, or too large";
        case BRQ_ERR_BLOCK: return "bad rotation block: need a power of two, 8 <= B <= 16384, B dividing K (matrix blocks: 1 or K/32 of them)";
        case BRQ_ERR_ALIGN: return "pointer or row pitch not 16-byte aligned";
        case BRQ_ERR_DTYPE: return "unknown dtype";
        case BRQ_ERR_LAUNCH: return "kernel launch failed";
        case BRQ_ERR_LAYOUT: return "unknown operand layout";
        case BRQ_ERR_DEVICE: return "no usable HIP device, or its one-time set-up failed";
        case BRQ_STATUS_INT_RANGE_: break;
    }
    return "unknown status";
}

int brq_version(void) { return 400; }

}  // extern "C"
