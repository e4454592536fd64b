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
// d, which sit first in it.  A run keeps its width over every depth above the lcp of the entry
// behind it, so the walk handles such a chain of unary nodes as one term times its length.
#include "sd_internal.h"

namespace {

constexpr int TB = 256;

// lenpos[p] = min(D, tokens from text position p up to its end marker).  A wave takes 64
// neighbouring positions and reads the text behind them 64 tokens at a time: one ballot per
// chunk marks the end markers, and every lane looks up the first one at or behind its own
// position.  The text carries SD_TEXT_PAD >= 64 + D end markers behind position N - 1, so the
// chunks a wave may touch (up to position base + 63 + D) exist.
__global__ __launch_bounds__(TB) void k_len_pos(const int32_t *__restrict__ text, int64_t N, int32_t D,
                                                uint8_t *__restrict__ lenpos) {
    const int lane = threadIdx.x & 63;
    const int64_t base = (int64_t)blockIdx.x * TB + (threadIdx.x - lane);
    if (base >= N) return;  // the whole wave
    int k = -1;             // distance to the first end marker, once known
    for (int c = 0; c * 64 < 64 + D; c++) {
        const unsigned long long m = __ballot(text[base + c * 64 + lane] < 0);
        if (k < 0) {
            // markers of chunk c at or behind this lane's position
            const unsigned long long mm = c == 0 ? (m >> lane) << lane : m;
            if (mm) k = c * 64 + __builtin_ctzll(mm) - lane;
        }
        if (__all(k >= 0)) break;
    }
    if (k < 0 || k > D) k = D;
    if (base + lane < N) lenpos[base + lane] = (uint8_t)k;
}

typedef int32_t tok4 __attribute__((ext_vector_type(4), aligned(4)));

__global__ __launch_bounds__(TB) void k_lcp_len(const int32_t *__restrict__ text,
                                                const int32_t *__restrict__ sa,
                                                const uint8_t *__restrict__ lenpos, int64_t N,
                                                uint8_t *__restrict__ lcp, uint8_t *__restrict__ len) {
    int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x;
    if (i >= N) return;
    const int32_t p = sa[i];
    const int L = lenpos[p];
    int k = 0;
    if (i > 0) {
        // the neighbour's end marker differs from every token of w: no bound of its own needed
        // (four tokens of either suffix per step, loaded as one 16-byte word at 4-byte
        // alignment; what lies behind a suffix's end is text or padding and is not looked at)
        const int32_t *w = text + p, *v = text + sa[i - 1];
        while (k < L) {
            const tok4 a = *reinterpret_cast<const tok4 *>(w + k), b = *reinterpret_cast<const tok4 *>(v + k);
            const int left = L - k;
            int same = 0;
            if (a.x == b.x) {
                same = 1;
                if (left > 1 && a.y == b.y) {
                    same = 2;
                    if (left > 2 && a.z == b.z) {
                        same = 3;
                        if (left > 3 && a.w == b.w) same = 4;
                    }
                }
            }
            k += same;
            if (same < 4) break;
        }
    }
    lcp[i] = (uint8_t)k;
    len[i] = (uint8_t)L;
}

// first index j' in [j, lim] with j' == lim or lcp[j'] < d; lcp is 16-byte aligned and the walk
// takes 16 entries per load once j is
__device__ __forceinline__ int64_t run_end(const uint8_t *__restrict__ lcp, int64_t j, int64_t lim,
                                           int d) {
    while (j < lim && (j & 15)) {
        if (lcp[j] < d) return j;
        j++;
    }
    while (j + 16 <= lim) {
        const uint4 x = *reinterpret_cast<const uint4 *>(lcp + j);
        const uint32_t wds[4] = {x.x, x.y, x.z, x.w};
        uint32_t m = 0;
#pragma unroll
        for (int q = 0; q < 16; q++)
            m |= (uint32_t)((int)((wds[q >> 2] >> (8 * (q & 3))) & 255u) < d) << q;
        if (m) return j + __builtin_ctz(m);
        j += 16;
    }
    while (j < lim) {
        if (lcp[j] < d) return j;
        j++;
    }
    return lim;
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
                                                const int32_t *__restrict__ tok1,
                                                const int32_t *__restrict__ bucket,
                                                const uint8_t *__restrict__ lcp,
                                                const uint8_t *__restrict__ len, int64_t N, int32_t D,
                                                double *acc, unsigned long long *wsum) {
    double sS = 0.0, sC = 0.0;
    unsigned long long w = 0;
    // a fixed number of workgroups strides over the entries: the three totals are single
    // addresses, and one atomic per wave of a grid as long as the array would queue up on them
    for (int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x; i < N; i += (int64_t)gridDim.x * TB) {
        w += len[i];
        const int lo = lcp[i], hi = i + 1 < N ? lcp[i + 1] : 0;
        if (hi > lo) {
            // every run entry i opens lies inside the bucket of its first token
            const int64_t bend = bucket[text[sa[i]] + 2];
            const int Li = len[i];
            int64_t j = i + 1;
            int d = hi;
            while (d > lo) {
                if (d == 1) {
                    j = bend;  // a run of depth 1 is the whole bucket
                } else if (d == 2) {
                    // second tokens rise along the bucket: the run ends where they pass tok1[i]
                    const int32_t t1 = tok1[i];
                    int64_t a = j, b = bend;
                    while (a < b) {
                        const int64_t m = (a + b) >> 1;
                        if (tok1[m] <= t1) a = m + 1; else b = m;
                    }
                    j = a;
                } else {
                    j = run_end(lcp, j, bend, d);
                }
                // the run [i, j) is the same node chain for every depth above lcp[j]
                const int below = j < N ? (int)lcp[j] : 0;
                const int dn = below > lo ? below : lo;
                const int span = d - dn;
                const int64_t c = j - i;
                const double tc = (double)c * log2((double)c);
                sC += (double)span * tc;
                // S = c at every depth below D, except where suffixes of the run stop: they
                // sit first in it, so only at depth len[i], which can only be the top one
                int plain = span - (d == D ? 1 : 0);
                if (d == hi && Li == d && d < D) {
                    plain--;
                    int64_t good = 0, step = 1;  // len[i + good] == d
                    while (good + step < c && len[i + good + step] == d) {
                        good += step;
                        step <<= 1;
                    }
                    int64_t bad = good + step < c ? good + step : c;  // c, or len[i + bad] != d
                    while (bad - good > 1) {
                        const int64_t m = (good + bad) >> 1;
                        if (len[i + m] == d) good = m; else bad = m;
                    }
                    const int64_t S = c - bad;
                    if (S >= 2) sS += (double)S * log2((double)S);
                }
                sS += (double)plain * tc;
                d = dn;
            }
        }
    }
    sS = wave_sum(sS);
    sC = wave_sum(sC);
    double wd = wave_sum((double)w);  // far below 2^53: exact
    __shared__ double part[3][TB / 64];
    if ((threadIdx.x & 63) == 0) {
        part[0][threadIdx.x >> 6] = sS;
        part[1][threadIdx.x >> 6] = sC;
        part[2][threadIdx.x >> 6] = wd;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        sS = sC = wd = 0.0;
        for (int q = 0; q < TB / 64; q++) {
            sS += part[0][q];
            sC += part[1][q];
            wd += part[2][q];
        }
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
        // N <= g_cap bytes each, in two build buffers of 4 g_cap bytes: lcp (16-byte aligned) in
        // one, lenpos and len in the halves of the other
        uint8_t *lcp = reinterpret_cast<uint8_t *>(c->b_flags);
        uint8_t *lenpos = reinterpret_cast<uint8_t *>(c->b_gid2), *len = lenpos + 2 * c->g_cap;
        sd_fill_i32(reinterpret_cast<int32_t *>(c->d_entropy), 6, 0, st);
        hipLaunchKernelGGL(k_len_pos, dim3(nblk(N)), dim3(TB), 0, st, c->g_text, N, c->cfg.D, lenpos);
        hipLaunchKernelGGL(k_lcp_len, dim3(nblk(N)), dim3(TB), 0, st, c->g_text, c->g_sa, lenpos, N,
                           lcp, len);
        hipLaunchKernelGGL(k_entropy, dim3(nblk(N) < 4096u ? nblk(N) : 4096u), dim3(TB), 0, st, c->g_text, c->g_sa, c->g_tok1,
                           c->g_bucket, lcp, len, N, c->cfg.D, c->d_entropy,
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
