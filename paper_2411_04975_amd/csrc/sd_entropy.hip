// Empirical entropy of the global index (Appendix, "Predicting SuffixDecoding Effectiveness":
// the entropy of every node's distribution over its children, averaged over the nodes with
// weights; low values announce predictable continuations).
//
// Reading taken: a node's distribution is COUNT(child) / S with S the sum of its children's
// COUNTs, the entropy is in bits, every node with a child (the root included) weighs S.
// With H = log2 S - (1/S) sum_c n_c log2 n_c, the weighted sum over all nodes is
//     sum_v S_v log2 S_v  -  sum_{u != root} COUNT(u) log2 COUNT(u),
// and the total weight is sum_v S_v = sum over positions of min(D, tokens left in the document).
//
// On the suffix array a tree node of depth d is a maximal run of neighbouring suffixes that
// share d tokens.  lcp[i] = number of tokens suffix i shares with suffix i-1 (at most D, end
// markers excluded), len[i] = min(D, tokens before its end marker).  Entry i opens a run of two
// or more suffixes at exactly the depths d in (lcp[i], lcp[i+1]]; runs of one suffix add
// nothing to either sum.  For falling d the run's end only moves right, so one forward walk
// per entry finds all its runs.  S of a run is its width minus the suffixes that stop at depth
// d, which sit first in it.
#include "sd_internal.h"

namespace {

constexpr int TB = 256;

__global__ __launch_bounds__(TB) void k_lcp_len(const int32_t *__restrict__ text,
                                                const int32_t *__restrict__ sa, int64_t N, int32_t D,
                                                uint8_t *__restrict__ lcp, uint8_t *__restrict__ len) {
    int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x;
    if (i >= N) return;
    const int32_t *w = text + sa[i];
    int k = 0;
    if (i > 0) {
        const int32_t *v = text + sa[i - 1];
        while (k < D && w[k] >= 0 && w[k] == v[k]) k++;
    }
    lcp[i] = (uint8_t)k;
    while (k < D && w[k] >= 0) k++;
    len[i] = (uint8_t)k;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// acc[0] += sum of S log2 S, acc[1] += sum of COUNT log2 COUNT (runs of two or more),
// wsum += sum of len
__global__ __launch_bounds__(TB) void k_entropy(const int32_t *__restrict__ text,
                                                const int32_t *__restrict__ sa,
                                                const int32_t *__restrict__ bucket,
                                                const uint8_t *__restrict__ lcp,
                                                const uint8_t *__restrict__ len, int64_t N, int32_t D,
                                                double *acc, unsigned long long *wsum) {
    int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x;
    double sS = 0.0, sC = 0.0;
    unsigned long long w = 0;
    if (i < N) {
        w = len[i];
        const int lo = lcp[i], hi = i + 1 < N ? lcp[i + 1] : 0;
        int64_t j = i + 1;
        for (int d = hi; d > lo; d--) {
            // a run of depth 1 is the whole bucket of its first token: no walk needed
            if (d == 1) j = bucket[text[sa[i]] + 2];
            while (j < N && lcp[j] >= d) j++;
            const int64_t c = j - i;
            sC += (double)c * log2((double)c);
            if (d < D) {
                int64_t e = 0;  // suffixes of the run that stop at depth d
                while (i + e < j && len[i + e] == d) e++;
                const int64_t S = c - e;
                if (S >= 2) sS += (double)S * log2((double)S);
            }
        }
    }
    sS = wave_sum(sS);
    sC = wave_sum(sC);
    double wd = wave_sum((double)w);  // at most 64 * 255: exact
    if ((threadIdx.x & 63) == 0) {
        if (sS != 0.0) atomicAdd(&acc[0], sS);
        if (sC != 0.0) atomicAdd(&acc[1], sC);
        if (wd != 0.0) atomicAdd(wsum, (unsigned long long)wd);
    }
}

inline unsigned nblk(int64_t n) { return (unsigned)((n + TB - 1) / TB); }

}  // namespace

sd_status sd_entropy_impl(sd_ctx *c, double *h_mean_bits, double *h_weight, hipStream_t st) {
    const int64_t N = c->g_N;
    double acc[2] = {0.0, 0.0};
    unsigned long long wsum = 0;
    if (N > 0) {
        uint8_t *lcp = reinterpret_cast<uint8_t *>(c->b_flags), *len = lcp + N;  // 2N <= 4 cap bytes
        sd_fill_i32(reinterpret_cast<int32_t *>(c->d_entropy), 6, 0, st);
        hipLaunchKernelGGL(k_lcp_len, dim3(nblk(N)), dim3(TB), 0, st, c->g_text, c->g_sa, N, c->cfg.D,
                           lcp, len);
        hipLaunchKernelGGL(k_entropy, dim3(nblk(N)), dim3(TB), 0, st, c->g_text, c->g_sa, c->g_bucket,
                           lcp, len, N, c->cfg.D, c->d_entropy,
                           reinterpret_cast<unsigned long long *>(c->d_entropy + 2));
        if (hipGetLastError() != hipSuccess) return SD_ERR_HIP;
        double host[3];
        if (hipMemcpyAsync(host, c->d_entropy, sizeof(host), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)
            return SD_ERR_HIP;
        acc[0] = host[0];
        acc[1] = host[1];
        memcpy(&wsum, &host[2], sizeof(wsum));
    }
    // the root: every token of the corpus is one observation of "what comes first"
    const double n = (double)c->g_tokens;
    const double root = n >= 2.0 ? n * log2(n) : 0.0;
    const double weight = (double)wsum;
    *h_weight = weight;
    *h_mean_bits = weight > 0.0 ? (acc[0] + root - acc[1]) / weight : 0.0;
    return SD_OK;
}
