// Reduction of the per-block statistics to what the paper's analysis reports (Sec. 4.1, 4.2 and the
// Appendix "Rotation Comparison"): the distribution of the block-wise scales, and the quantization loss and
// the growth of the scales split into regular and outlier blocks.  Input: the per-block arrays that
// brq_block_stats writes (one fp32 per block of 32).  HBM bound and small: 8 to 12 bytes per block.
#include "brq_device.h"
#include "brq_launch.h"

namespace brq {

struct SummaryArgs {
    const float* amax;              // [n] block-wise scales after the transformation under study
    const float* sqerr;             // [n] or null: per-block MXFP4 loss after it
    const float* ref;               // [n] or null: block-wise scales of the reference (untransformed) activations
    unsigned long long n;
    float outlier;                  // a block is an outlier block when its reference scale exceeds this
    int nedges;                     // 0..32
    float edges[32];
    unsigned long long* hist;       // [nedges + 1] or null, added to
    unsigned long long* counts;     // [4] or null, added to
    double* sums;                   // [4] or null, added to
};

// One block per lane and pass, four passes' loads in flight (a lane's loads are 4 bytes; every load is
// unconditional - an absent array is replaced by the scales themselves - because a load behind a branch makes
// the compiler wait for all earlier ones).  Histogram: the edges ascend, so a scale that exceeds edge e exceeds
// every edge below it; per edge the wavefront counts its lanes above it with one comparison and the scalar
// unit's bit count, and bin j follows as (count above edge j - 1) - (count above edge j).  Class counts the same
// way.  The fp64 sums are added across a wavefront's lanes in a fixed butterfly, across the workgroup's
// wavefronts in index order, and across workgroups by the hardware's fp64 atomic add (the generic atomicAdd on a
// double is a compare-and-swap loop): the result depends on the order in which workgroups finish, to a few units
// of 2^-53 times their number.
__global__ void __launch_bounds__(1024) k_block_summary(SummaryArgs a) {
    __shared__ unsigned int s_gt[33];        // [e]: blocks above edge e; [32]: all blocks of the workgroup
    __shared__ unsigned int s_cnt[4];
    __shared__ double s_wsum[16][4];
    if (threadIdx.x < 33) s_gt[threadIdx.x] = 0;
    if (threadIdx.x < 4) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const float* const refp = a.ref ? a.ref : a.amax;
    const float* const sqp = a.sqerr ? a.sqerr : a.amax;
    const bool has_sq = a.sqerr != nullptr, has_ref = a.ref != nullptr, lane0 = (threadIdx.x & 63u) == 0;
    unsigned int cnt[4] = {0, 0, 0, 0}, nlive = 0, gt[32];     // wavefront-uniform, held by the scalar unit
#pragma unroll
    for (int e = 0; e < 32; ++e) gt[e] = 0;
    double sum[4] = {0.0, 0.0, 0.0, 0.0};
    constexpr int U = 4;
    const unsigned long long step = (unsigned long long)gridDim.x * 1024 * U;
    for (unsigned long long i0 = (unsigned long long)blockIdx.x * 1024 * U; i0 < a.n; i0 += step) {
        float am[U], rf[U], sq[U];
        bool live[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned long long i = i0 + (unsigned long long)u * 1024 + threadIdx.x;
            live[u] = i < a.n;
            const unsigned long long ic = live[u] ? i : a.n - 1;       // past the end: the last block again, masked below
            am[u] = a.amax[ic];
            rf[u] = refp[ic];
            sq[u] = sqp[ic];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned long long lm = __builtin_amdgcn_ballot_w64(live[u]);
            const unsigned long long mo = __builtin_amdgcn_ballot_w64(rf[u] > a.outlier) & lm;
            const unsigned long long mr = lm & ~mo;
            const unsigned long long mg = has_ref ? __builtin_amdgcn_ballot_w64(am[u] > rf[u]) : 0ull;
            cnt[0] += (unsigned int)__builtin_popcountll(mr);
            cnt[1] += (unsigned int)__builtin_popcountll(mo);
            cnt[2] += (unsigned int)__builtin_popcountll(mr & mg);
            cnt[3] += (unsigned int)__builtin_popcountll(mo & mg);
            const bool isr = (mr >> (threadIdx.x & 63u)) & 1ull, iso = (mo >> (threadIdx.x & 63u)) & 1ull;
            sum[0] += (double)((isr && has_sq) ? sq[u] : 0.0f);
            sum[1] += (double)((iso && has_sq) ? sq[u] : 0.0f);
            sum[2] += (double)(isr ? am[u] : 0.0f);
            sum[3] += (double)(iso ? am[u] : 0.0f);
            if (a.hist) {   // uniform; the edges beyond nedges are +inf, eight at a time behind a uniform test
                nlive += (unsigned int)__builtin_popcountll(lm);
#pragma unroll
                for (int e0 = 0; e0 < 32; e0 += 8)
                    if (e0 < a.nedges) {
#pragma unroll
                        for (int e = e0; e < e0 + 8; ++e)
                            gt[e] += (unsigned int)__builtin_popcountll(__builtin_amdgcn_ballot_w64(am[u] > a.edges[e]) & lm);
                    }
            }
        }
    }
    const unsigned int wave = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        double v = sum[k];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
        if (lane0) {
            s_wsum[wave][k] = v;
            if (cnt[k]) atomicAdd(&s_cnt[k], cnt[k]);
        }
    }
    if (lane0 && a.hist) {
        atomicAdd(&s_gt[32], nlive);
#pragma unroll
        for (int e = 0; e < 32; ++e)
            if (gt[e]) atomicAdd(&s_gt[e], gt[e]);
    }
    __syncthreads();
    if (a.hist && threadIdx.x <= (unsigned)a.nedges) {
        const unsigned int above_prev = threadIdx.x == 0 ? s_gt[32] : s_gt[threadIdx.x - 1];
        const unsigned int above_this = threadIdx.x == (unsigned)a.nedges ? 0u : s_gt[threadIdx.x];
        if (above_prev != above_this) atomicAdd(&a.hist[threadIdx.x], (unsigned long long)(above_prev - above_this));
    }
    if (threadIdx.x < 4) {
        if (a.counts && s_cnt[threadIdx.x]) atomicAdd(&a.counts[threadIdx.x], (unsigned long long)s_cnt[threadIdx.x]);
        double t = 0.0;
        for (unsigned int w = 0; w < blockDim.x / 64u; ++w) t += s_wsum[w][threadIdx.x];
        if (a.sums && t != 0.0) __builtin_amdgcn_global_atomic_fadd_f64(&a.sums[threadIdx.x], t);
    }
}

hipError_t launch_block_summary(const float* amax, const float* sqerr, const float* ref, int64_t n, float outlier,
                                const float* edges, int nedges, unsigned long long* hist, unsigned long long* counts,
                                double* sums, hipStream_t s) {
    int cus = 0;
    if (hipError_t e = device_cus(&cus); e != hipSuccess) return e;
    SummaryArgs a;
    a.amax = amax; a.sqerr = sqerr; a.ref = ref; a.n = (unsigned long long)n; a.outlier = outlier; a.nedges = nedges;
    for (int e = 0; e < 32; ++e) a.edges[e] = e < nedges ? edges[e] : __builtin_inff();   // beyond nedges: exceeded by nothing
    a.hist = hist; a.counts = counts; a.sums = sums;
    // One workgroup of 16 wavefronts per compute unit at most: every workgroup ends with an atomic per output
    // word, and atomics on the same few words from thousands of workgroups would take longer than the pass
    // over the data.
    const int64_t want = (n + 4095) / 4096;
    const int64_t cap = (int64_t)cus;
    hipLaunchKernelGGL(k_block_summary, dim3((uint32_t)(want < cap ? (want < 1 ? 1 : want) : cap)), dim3(1024), 0, s, a);
    return hipGetLastError();
}

}  // namespace brq
