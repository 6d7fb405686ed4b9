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

// One block per lane and pass.  Histogram: a lane's bin is the number of edges its scale exceeds; for every
// bin the wavefront counts its lanes in that bin with one comparison and the scalar unit's bit count (an LDS
// atomic per block would have every lane of the chip queueing for the same few words).  Every lane keeps its
// own class counts and fp64 sums; one LDS atomic per wavefront and one global atomic per workgroup and output
// word (a workgroup has 16 wavefronts, and a launch at most one workgroup per compute unit).  The fp64 sums are added in an order that depends
// on the schedule: they agree with a sequential sum to a few units of 2^-53 times the number of workgroups.
__global__ void __launch_bounds__(1024) k_block_summary(SummaryArgs a) {
    __shared__ unsigned int s_hist[33];
    __shared__ unsigned int s_cnt[4];
    __shared__ double s_sum[4];
    if (threadIdx.x < 33) s_hist[threadIdx.x] = 0;
    if (threadIdx.x < 4) { s_cnt[threadIdx.x] = 0; s_sum[threadIdx.x] = 0.0; }
    __syncthreads();
    unsigned int cnt[4] = {0, 0, 0, 0};
    double sum[4] = {0.0, 0.0, 0.0, 0.0};
    unsigned int hcnt[33];          // wavefront-uniform: blocks of this wavefront in bin j
#pragma unroll
    for (int j = 0; j < 33; ++j) hcnt[j] = 0;
    // Four passes' worth of loads are issued before any of them is used (a lane's loads are 4 bytes: without
    // this the kernel waits for memory most of the time).  Uniform trip count: lanes past the end carry a
    // scale that falls into no bin and into no class.
    constexpr int U = 4;
    const unsigned long long step = (unsigned long long)gridDim.x * 1024 * U;
    for (unsigned long long i0 = (unsigned long long)blockIdx.x * 1024 * U; i0 < a.n; i0 += step) {
        float am[U], rf[U], sq[U];
        bool live[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned long long i = i0 + (unsigned long long)u * 1024 + threadIdx.x;
            live[u] = i < a.n;
            const unsigned long long ic = live[u] ? i : a.n - 1;
            am[u] = a.amax[ic];
            rf[u] = a.ref ? a.ref[ic] : am[u];
            sq[u] = a.sqerr ? a.sqerr[ic] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool outl = rf[u] > a.outlier, grew = a.ref && am[u] > rf[u];
            const bool l = live[u];
            cnt[0] += (l && !outl) ? 1u : 0u;
            cnt[1] += (l && outl) ? 1u : 0u;
            cnt[2] += (l && !outl && grew) ? 1u : 0u;
            cnt[3] += (l && outl && grew) ? 1u : 0u;
            sum[0] += (l && !outl) ? (double)sq[u] : 0.0;
            sum[1] += (l && outl) ? (double)sq[u] : 0.0;
            sum[2] += (l && !outl) ? (double)am[u] : 0.0;
            sum[3] += (l && outl) ? (double)am[u] : 0.0;
            if (a.hist) {   // uniform
                int bin = l ? 0 : -1;
                for (int e = 0; e < a.nedges; ++e) bin += (l && am[u] > a.edges[e]) ? 1 : 0;
#pragma unroll
                for (int j = 0; j < 33; ++j)
                    if (j <= a.nedges) hcnt[j] += (unsigned int)__builtin_popcountll(__builtin_amdgcn_ballot_w64(bin == j));
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (cnt[k]) atomicAdd(&s_cnt[k], cnt[k]);
        if (sum[k] != 0.0) atomicAdd(&s_sum[k], sum[k]);
    }
    if ((threadIdx.x & 63u) == 0) {
#pragma unroll
        for (int j = 0; j < 33; ++j)
            if (j <= a.nedges && hcnt[j]) atomicAdd(&s_hist[j], hcnt[j]);
    }
    __syncthreads();
    if (a.hist && threadIdx.x <= (unsigned)a.nedges && s_hist[threadIdx.x]) atomicAdd(&a.hist[threadIdx.x], (unsigned long long)s_hist[threadIdx.x]);
    if (threadIdx.x < 4) {
        if (a.counts && s_cnt[threadIdx.x]) atomicAdd(&a.counts[threadIdx.x], (unsigned long long)s_cnt[threadIdx.x]);
        if (a.sums && s_sum[threadIdx.x] != 0.0) atomicAdd(&a.sums[threadIdx.x], s_sum[threadIdx.x]);
    }
}

hipError_t launch_block_summary(const float* amax, const float* sqerr, const float* ref, int64_t n, float outlier,
                                const float* edges, int nedges, unsigned long long* hist, unsigned long long* counts,
                                double* sums, hipStream_t s) {
    int cus = 0;
    if (hipError_t e = device_cus(&cus); e != hipSuccess) return e;
    SummaryArgs a;
    a.amax = amax; a.sqerr = sqerr; a.ref = ref; a.n = (unsigned long long)n; a.outlier = outlier; a.nedges = nedges;
    for (int e = 0; e < 32; ++e) a.edges[e] = e < nedges ? edges[e] : 0.0f;
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
