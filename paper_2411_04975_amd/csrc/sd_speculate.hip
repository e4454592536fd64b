// Batched draft generation: MatchPattern, ExpandSpeculationTree and the best-tree choice of
// GenerateCandidateTree (Algorithm 1), for every request of a batch, both indexes and every
// pattern length p = 1..P.
//
// A node of either suffix structure is a range [lo, hi) of a sorted suffix list: the suffixes
// that start with the node's path.  COUNT = hi - lo.  The children of a node at depth d are
// the runs of equal token at offset d inside the range (an end marker, which sorts first,
// means the suffix stops there and is no child).
//
//  k_req_occurrences  one workgroup per request: scan the context for earlier occurrences of
//                     its last token, measure how far each extends to the left (up to P), and
//                     sort the occurrences by what follows them.  The occurrences with
//                     left-extension >= p, in that order, are the sorted suffix list of the
//                     per-request structure below the pattern of length p.
//  k_expand           one wavefront per (request, index, p) unit: find the node N_p, then
//                     grow the tree greedily; the frontier lives in LDS, the arg-max is a
//                     wave reduction.
//  k_select           one wavefront per request: strictly-greater scan over the 2P unit
//                     scores, coalesced copy of the winner.
#include <math.h>

#include "sd_internal.h"

namespace {

struct SpecParams {
    const int32_t *g_text, *g_sa, *g_bucket;
    int32_t g_N;
    const int32_t *r_text, *r_len;
    int64_t r_stride;
    int32_t max_slots, max_ctx;
    int32_t D, P, max_nodes;
    double alpha, min_score;
    int2 *occ;
    int32_t *occ_n, *cntL, *unit_sa, *unit_n;
    double *unit_score;
    int32_t *unit_tok, *unit_par;
    double *unit_sc;
    int32_t *err;
    unsigned long long *algo_bytes;
};

// In the counting variants (STATS) every lane adds up the bytes it asks memory for: 4 per
// suffix-array word or token, 8 per occurrence record.  Loads that all lanes share are counted
// once.  The timed variants compile the counters away.
#define SD_CNT(n) do { if (STATS) nb += (unsigned)(n); } while (0)

template <bool STATS>
__device__ __forceinline__ void flush_count(unsigned nb, unsigned long long *dst) {
    if (!STATS) return;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) nb += __shfl_xor(nb, o);
    if ((threadIdx.x & 63) == 0) atomicAdd(dst, (unsigned long long)nb);
}

__device__ __forceinline__ uint64_t lanemask_lt() { return (1ull << (threadIdx.x & 63)) - 1ull; }

// ------------------------------------------------------------------------------------------
// per-request occurrence lists
// ------------------------------------------------------------------------------------------
constexpr int OCC_THREADS = 256;
constexpr int OCC_LDS_SORT = 2048;

// order of two occurrences by the tokens that follow them (end marker lowest), then by position
template <bool STATS>
__device__ __forceinline__ bool occ_less(const int32_t *__restrict__ x, int2 a, int2 b, int depth,
                                         unsigned &nb) {
    const int32_t *pa = x + a.x + 1, *pb = x + b.x + 1;
    for (int k = 0; k < depth; k++) {
        int32_t ta = pa[k], tb = pb[k];
        SD_CNT(8);
        if (ta != tb) return ta < tb;
        if (ta == SD_END_TOKEN) break;
    }
    return a.x < b.x;
}

// bitonic network in its all-ascending form (mirror step, then half-cleaners); positions at or
// beyond m act as +infinity and are never touched, so m need not be a power of two
template <bool STATS>
__device__ void occ_sort(int2 *arr, int m, const int32_t *__restrict__ x, int depth, unsigned &nb) {
    int n2 = 1;
    while (n2 < m) n2 <<= 1;
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < m; i += OCC_THREADS) {
                int l = (j == (k >> 1)) ? (i ^ (k - 1)) : (i ^ j);
                if (l > i && l < m) {
                    int2 a = arr[i], b = arr[l];
                    if (occ_less<STATS>(x, b, a, depth, nb)) {
                        arr[i] = b;
                        arr[l] = a;
                    }
                }
            }
            __syncthreads();
        }
    }
}

template <bool STATS>
__global__ __launch_bounds__(OCC_THREADS) void k_req_occurrences(SpecParams p,
                                                                 const int32_t *__restrict__ slot_ids) {
    __shared__ int s_m;
    __shared__ int s_cnt[72];
    __shared__ int2 s_sort[OCC_LDS_SORT];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const int32_t slot = slot_ids[b];
    const bool slot_ok = slot >= 0 && slot < p.max_slots;
    if (!slot_ok && tid == 0) atomicOr(&p.err[SD_DEVERR_SLOT], 1);
    const int t = slot_ok ? p.r_len[slot] : 0;
    const int32_t *x = p.r_text + (int64_t)(slot_ok ? slot : 0) * p.r_stride;
    int2 *occ = p.occ + (int64_t)b * p.max_ctx;
    unsigned nb = 0;
    if (tid == 0) s_m = 0;
    if (tid < 72) s_cnt[tid] = 0;
    __syncthreads();
    if (t > 0) {
        const int32_t last = x[t - 1];
        const uint64_t lt = lanemask_lt();
        for (int base = 0; base < t; base += OCC_THREADS) {
            int e = base + tid;
            bool hit = e < t && x[e] == last;
            if (e < t) SD_CNT(4);
            uint64_t mask = __ballot(hit);
            if (mask) {
                int leader = __ffsll((unsigned long long)mask) - 1;
                int off = 0;
                if (lane == leader) off = atomicAdd(&s_m, __popcll(mask));
                off = __shfl(off, leader);
                if (hit) occ[off + __popcll(mask & lt)].x = e;
            }
        }
    }
    __syncthreads();
    const int m = s_m;
    // how far each occurrence extends to the left together with the context's own tail
    for (int i = tid; i < m; i += OCC_THREADS) {
        int e = occ[i].x;
        int lim = e + 1 < p.P ? e + 1 : p.P;
        int l = 1;
        while (l < lim && x[e - l] == x[t - 1 - l]) l++;
        SD_CNT(8 * l + 8);
        occ[i].y = l;
        atomicAdd(&s_cnt[l], 1);
    }
    __syncthreads();
    if (tid == 0) {
        int acc = 0;
        int32_t *cl = p.cntL + (int64_t)b * (p.P + 1);
        for (int l = p.P; l >= 1; l--) {
            acc += s_cnt[l];
            cl[l] = acc;
        }
        cl[0] = m;
        p.occ_n[b] = m;
    }
    if (m > 1) {
        const int depth = p.D - 1;
        if (m <= OCC_LDS_SORT) {
            for (int i = tid; i < m; i += OCC_THREADS) s_sort[i] = occ[i];
            __syncthreads();
            occ_sort<STATS>(s_sort, m, x, depth, nb);
            for (int i = tid; i < m; i += OCC_THREADS) occ[i] = s_sort[i];
        } else {
            occ_sort<STATS>(occ, m, x, depth, nb);
        }
    }
    flush_count<STATS>(nb, p.algo_bytes + SD_K_OCCURRENCES);
}

// ------------------------------------------------------------------------------------------
// expansion
// ------------------------------------------------------------------------------------------
struct Key {
    double s;
    int32_t tok, par, idx;  // idx < 0: no entry
};

// selection order of the greedy arg-max: score high, token low, parent low
__device__ __forceinline__ bool key_better(const Key &a, const Key &b) {
    if (a.s != b.s) return a.s > b.s;
    if (a.tok != b.tok) return a.tok < b.tok;
    return a.par < b.par;
}

__device__ __forceinline__ Key key_shfl_xor(const Key &k, int o) {
    Key r;
    r.s = __shfl_xor(k.s, o);
    r.tok = __shfl_xor(k.tok, o);
    r.par = __shfl_xor(k.par, o);
    r.idx = __shfl_xor(k.idx, o);
    return r;
}

// wave-wide best (want_best) or worst entry; every lane returns the same key
__device__ __forceinline__ Key wave_pick(Key mine, bool want_best) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        Key other = key_shfl_xor(mine, o);
        bool take;
        if (other.idx < 0) take = false;
        else if (mine.idx < 0) take = true;
        else take = want_best ? key_better(other, mine) : key_better(mine, other);
        if (take) mine = other;
    }
    return mine;
}

struct Frontier {
    double *score;
    int32_t *tok, *par, *lo, *hi, *dep;
    int n, cap;
};

__device__ __forceinline__ Key frontier_pick(const Frontier &f, bool want_best) {
    const int lane = threadIdx.x & 63;
    Key mine;
    mine.idx = -1; mine.s = 0.0; mine.tok = 0; mine.par = 0;
    for (int i = lane; i < f.n; i += 64) {
        Key k;
        k.s = f.score[i]; k.tok = f.tok[i]; k.par = f.par[i]; k.idx = i;
        if (mine.idx < 0 || (want_best ? key_better(k, mine) : key_better(mine, k))) mine = k;
    }
    return wave_pick(mine, want_best);
}

// Add the candidates held by the lanes with `cand` set.  The frontier keeps at most `cap`
// entries: a candidate that does not rank among the best `cap` can never be selected, because
// at most `cap` more nodes are ever taken from it.
__device__ void frontier_insert(Frontier &f, bool cand, double sc, int32_t tok, int32_t par,
                                int32_t lo, int32_t hi, int32_t dep) {
    const int lane = threadIdx.x & 63;
    uint64_t C = __ballot(cand);
    if (C == 0) return;
    int nc = __popcll(C);
    if (f.n + nc <= f.cap) {
        if (cand) {
            int s = f.n + __popcll(C & lanemask_lt());
            f.score[s] = sc; f.tok[s] = tok; f.par[s] = par; f.lo[s] = lo; f.hi[s] = hi;
            f.dep[s] = dep;
        }
        f.n += nc;
        __syncthreads();
        return;
    }
    while (C) {
        int src = __ffsll((unsigned long long)C) - 1;
        C &= C - 1;
        Key nk;
        nk.s = __shfl(sc, src); nk.tok = __shfl(tok, src); nk.par = __shfl(par, src); nk.idx = 0;
        int32_t nlo = __shfl(lo, src), nhi = __shfl(hi, src), ndep = __shfl(dep, src);
        int s = -1;
        if (f.n < f.cap) {
            s = f.n++;
        } else {
            Key worst = frontier_pick(f, false);
            if (key_better(nk, worst)) s = worst.idx;
        }
        if (s >= 0 && lane == 0) {
            f.score[s] = nk.s; f.tok[s] = nk.tok; f.par[s] = nk.par; f.lo[s] = nlo; f.hi[s] = nhi;
            f.dep[s] = ndep;
        }
        __syncthreads();
    }
}

// Children of the node [lo, hi) at depth d (its path has d tokens), as frontier candidates with
// score = ps * (COUNT(child) / COUNT(node)).
template <bool STATS>
__device__ void push_children(Frontier &f, const int32_t *__restrict__ sa,
                              const int32_t *__restrict__ text, int32_t lo, int32_t hi, int32_t d,
                              int32_t parent, double ps, double min_score, int32_t D, unsigned &nb) {
    if (d >= D) return;  // a path of D tokens has no continuation
    const int lane = threadIdx.x & 63;
    const int32_t m = hi - lo;
    const double den = (double)m;
    if (m <= 64) {
        const bool in = lane < m;
        int32_t tok = 0x7fffffff;
        if (in) tok = text[(int64_t)sa[lo + lane] + d];
        if (in) SD_CNT(8);
        int32_t prev = __shfl_up(tok, 1);
        bool start = in && (lane == 0 || tok != prev);
        uint64_t S = __ballot(start);
        uint64_t above = lane == 63 ? 0ull : (S >> (lane + 1));
        int32_t e = above ? lane + 1 + (__ffsll((unsigned long long)above) - 1) : m;
        int32_t c = e - lane;
        double sc = ps * ((double)c / den);
        bool cand = start && tok >= 0 && sc >= min_score;
        frontier_insert(f, cand, sc, tok, parent, lo + lane, lo + e, d + 1);
        return;
    }
    // Wide node: a child that can still reach min_score has at least c_min occurrences, so its
    // run contains one of the positions lo, lo + c_min, lo + 2 c_min, ...  Probe those, then
    // bracket the run of each distinct probed token by binary search.  The bound is taken a
    // little low (factor 1 - 1e-9) so that rounding can never hide an admissible child; the
    // exact binary64 test below decides.
    int64_t stride = (int64_t)floor(min_score * den / ps * (1.0 - 1e-9));
    if (stride < 1) stride = 1;
    const int64_t np = ((int64_t)m + stride - 1) / stride;
    for (int64_t k0 = 0; k0 < np; k0 += 64) {
        const int64_t k = k0 + lane;
        const bool in = k < np;
        const int32_t q = (int32_t)(lo + (in ? k : 0) * stride);
        int32_t tok = 0x7fffffff;
        if (in) tok = text[(int64_t)sa[q] + d];
        if (in) SD_CNT(8);
        int32_t prevtok = __shfl_up(tok, 1);
        if (lane == 0) prevtok = k == 0 ? (int32_t)0x80000000 : text[(int64_t)sa[q - stride] + d];
        if (lane == 0 && k != 0) SD_CNT(8);
        const bool first = in && tok >= 0 && tok != prevtok;
        int32_t lb = q, ub = hi;
        if (first) {
            if (k > 0) {  // first position in (q - stride, q] holding tok
                int32_t l = (int32_t)(q - stride + 1), h = q;
                while (l < h) {
                    int32_t mid = l + ((h - l) >> 1);
                    SD_CNT(8);
                    if (text[(int64_t)sa[mid] + d] < tok) l = mid + 1; else h = mid;
                }
                lb = l;
            }
            int32_t l = q + 1, h = hi;  // first position after q holding a larger token
            while (l < h) {
                int32_t mid = l + ((h - l) >> 1);
                SD_CNT(8);
                if (text[(int64_t)sa[mid] + d] <= tok) l = mid + 1; else h = mid;
            }
            ub = l;
        }
        double sc = ps * ((double)(ub - lb) / den);
        bool cand = first && sc >= min_score;
        frontier_insert(f, cand, sc, tok, parent, lb, ub, d + 1);
    }
}

template <bool STATS>
__global__ __launch_bounds__(64) void k_expand(SpecParams p, const int32_t *__restrict__ slot_ids) {
    extern __shared__ double smem[];
    const int lane = threadIdx.x;
    unsigned nb = 0;
    const int cap = p.max_nodes;
    // LDS carve-up: frontier (score, tok, par, lo, hi, dep) and the tree (score, tok, par)
    double *f_score = smem;
    double *t_score = f_score + cap;
    int32_t *f_tok = (int32_t *)(t_score + cap);
    int32_t *f_par = f_tok + cap, *f_lo = f_par + cap, *f_hi = f_lo + cap, *f_dep = f_hi + cap;
    int32_t *t_tok = f_dep + cap, *t_par = t_tok + cap;

    const int units = 2 * p.P;
    const int b = blockIdx.x / units, r = blockIdx.x % units;
    const int src = r / p.P, pl = r % p.P + 1;
    const int64_t uidx = (int64_t)b * units + r;
    const int32_t slot = slot_ids[b];
    const bool slot_ok = slot >= 0 && slot < p.max_slots;
    const int t = slot_ok ? p.r_len[slot] : 0;
    const int32_t *x = p.r_text + (int64_t)(slot_ok ? slot : 0) * p.r_stride;
    const int K = (int)floor(p.alpha * (double)pl);

    const int32_t *sa = nullptr, *text = nullptr;
    int32_t lo = 0, hi = 0;
    if (pl <= t && K >= 1) {
        if (src == 0) {
            if (p.g_N > 0) {
                // MatchPattern on the global suffix array: all suffixes starting with the
                // pattern's first token form one bucket; binary search inside it, comparing
                // the p pattern tokens lane-parallel (lane k holds pattern token k).
                const int32_t wk = lane < pl ? x[t - pl + lane] : 0;
                if (lane < pl) SD_CNT(4);
                if (lane == 0) SD_CNT(8);  // the two bucket bounds
                const int32_t w0 = __shfl(wk, 0);
                lo = p.g_bucket[w0 + 1];
                hi = p.g_bucket[w0 + 2];
                sa = p.g_sa;
                text = p.g_text;
                if (pl > 1 && lo < hi) {
                    int32_t l = lo, h = hi;
                    while (l < h) {  // first suffix whose leading p tokens are >= the pattern
                        int32_t mid = l + ((h - l) >> 1);
                        int64_t pos = sa[mid];
                        int32_t tk = lane < pl ? text[pos + lane] : 0;
                        SD_CNT(lane < pl ? (lane == 0 ? 8 : 4) : 0);
                        uint64_t ne = __ballot(lane < pl && tk != wk);
                        bool less = false;
                        if (ne) {
                            int fl = __ffsll((unsigned long long)ne) - 1;
                            less = __shfl(tk, fl) < __shfl(wk, fl);
                        }
                        if (less) l = mid + 1; else h = mid;
                    }
                    const int32_t lb = l;
                    h = hi;
                    while (l < h) {  // first suffix whose leading p tokens are > the pattern
                        int32_t mid = l + ((h - l) >> 1);
                        int64_t pos = sa[mid];
                        int32_t tk = lane < pl ? text[pos + lane] : 0;
                        SD_CNT(lane < pl ? (lane == 0 ? 8 : 4) : 0);
                        uint64_t ne = __ballot(lane < pl && tk != wk);
                        bool greater = false;
                        if (ne) {
                            int fl = __ffsll((unsigned long long)ne) - 1;
                            greater = __shfl(tk, fl) > __shfl(wk, fl);
                        }
                        if (!greater) l = mid + 1; else h = mid;
                    }
                    lo = lb;
                    hi = l;
                }
            }
        } else {
            // per-request structure: occurrences whose left-extension reaches p, in the
            // order k_req_occurrences left them (sorted by what follows)
            const int m1 = p.occ_n[b];
            const int m = p.cntL[(int64_t)b * (p.P + 1) + pl];
            const int2 *occ = p.occ + (int64_t)b * p.max_ctx;
            int32_t *usa = p.unit_sa + ((int64_t)b * p.P + (pl - 1)) * p.max_ctx;
            int w = 0;
            for (int base = 0; base < m1; base += 64) {
                int i = base + lane;
                int2 o = make_int2(0, 0);
                if (i < m1) o = occ[i];
                if (i < m1) SD_CNT(8);
                bool keep = i < m1 && o.y >= pl;
                uint64_t mk = __ballot(keep);
                if (keep) usa[w + __popcll(mk & lanemask_lt())] = o.x - pl + 1;
                if (keep) SD_CNT(4);
                w += __popcll(mk);
            }
            __threadfence_block();
            __syncthreads();
            lo = 0;
            hi = m;  // == w
            sa = usa;
            text = x;
        }
    }

    int n = 0;
    double total = 0.0;
    if (hi > lo) {
        Frontier f;
        f.score = f_score; f.tok = f_tok; f.par = f_par; f.lo = f_lo; f.hi = f_hi; f.dep = f_dep;
        f.n = 0;
        f.cap = K;
        push_children<STATS>(f, sa, text, lo, hi, pl, -1, 1.0, p.min_score, p.D, nb);
        while (n < K && f.n > 0) {
            Key best = frontier_pick(f, true);
            if (best.s < p.min_score) break;
            const int bi = best.idx;
            const int32_t blo = f.lo[bi], bhi = f.hi[bi], bdep = f.dep[bi];
            __syncthreads();
            if (lane == 0) {
                t_tok[n] = best.tok; t_par[n] = best.par; t_score[n] = best.s;
                const int last = f.n - 1;
                if (bi != last) {
                    f.score[bi] = f.score[last]; f.tok[bi] = f.tok[last]; f.par[bi] = f.par[last];
                    f.lo[bi] = f.lo[last]; f.hi[bi] = f.hi[last]; f.dep[bi] = f.dep[last];
                }
            }
            f.n--;
            total += best.s;
            __syncthreads();
            if (n + 1 < K)  // the last node taken cannot contribute further nodes
                push_children<STATS>(f, sa, text, blo, bhi, bdep, n, best.s, p.min_score, p.D, nb);
            n++;
        }
    }
    __syncthreads();
    for (int i = lane; i < n; i += 64) {
        p.unit_tok[uidx * cap + i] = t_tok[i];
        p.unit_par[uidx * cap + i] = t_par[i];
        p.unit_sc[uidx * cap + i] = t_score[i];
        SD_CNT(16);
    }
    if (lane == 0) {
        p.unit_n[uidx] = n;
        p.unit_score[uidx] = total;
        SD_CNT(12);
    }
    flush_count<STATS>(nb, p.algo_bytes + SD_K_EXPAND);
}

template <bool STATS>
__global__ __launch_bounds__(64) void k_select(SpecParams p, sd_trees out) {
    const int lane = threadIdx.x, b = blockIdx.x;
    unsigned nb = 0;
    const int units = 2 * p.P, cap = p.max_nodes;
    // strictly-greater scan in unit order = the earliest unit among those with the top score
    double bs = 0.0;
    int bu = -1;
    for (int u = lane; u < units; u += 64) {
        double s = p.unit_score[(int64_t)b * units + u];
        SD_CNT(8);
        if (s > bs) { bs = s; bu = u; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        double os = __shfl_xor(bs, o);
        int ou = __shfl_xor(bu, o);
        if (ou >= 0 && (bu < 0 || os > bs || (os == bs && ou < bu))) { bs = os; bu = ou; }
    }
    int n = 0;
    if (bu >= 0) n = p.unit_n[(int64_t)b * units + bu];
    const int64_t ub = ((int64_t)b * units + (bu >= 0 ? bu : 0)) * cap;
    const int64_t ob = (int64_t)b * out.max_nodes;
    for (int i = lane; i < out.max_nodes; i += 64) {
        bool live = i < n;
        out.d_tokens[ob + i] = live ? p.unit_tok[ub + i] : -1;
        out.d_parents[ob + i] = live ? p.unit_par[ub + i] : -1;
        out.d_scores[ob + i] = live ? p.unit_sc[ub + i] : 0.0;
        SD_CNT(live ? 32 : 16);
    }
    if (lane == 0) {
        out.d_n_nodes[b] = n;
        out.d_tree_score[b] = bu >= 0 ? bs : 0.0;
        out.d_match_len[b] = bu >= 0 ? bu % p.P + 1 : 0;
        out.d_source[b] = bu >= 0 ? bu / p.P : -1;
        SD_CNT(24);
    }
    flush_count<STATS>(nb, p.algo_bytes + SD_K_SELECT);
}

__global__ __launch_bounds__(64) void k_accept(const int32_t *__restrict__ n_nodes,
                                               const int32_t *__restrict__ tokens,
                                               const int32_t *__restrict__ parents, int max_nodes,
                                               const int32_t *__restrict__ target,
                                               int32_t *__restrict__ accept_len,
                                               int32_t *__restrict__ accept_path,
                                               int32_t *__restrict__ bonus) {
    const int lane = threadIdx.x, b = blockIdx.x;
    int n = n_nodes[b];
    if (n > max_nodes) n = max_nodes;
    const int32_t *tok = tokens + (int64_t)b * max_nodes, *par = parents + (int64_t)b * max_nodes;
    const int32_t *tgt = target + (int64_t)b * (max_nodes + 1);
    int32_t *path = accept_path + (int64_t)b * max_nodes;
    int v = -1, L = 0;
    while (L < n) {
        const int32_t want = tgt[v + 1];
        int found = -1;
        for (int base = 0; base < n && found < 0; base += 64) {
            int j = base + lane;
            bool hit = j < n && par[j] == v && tok[j] == want;
            uint64_t m = __ballot(hit);
            if (m) found = base + __ffsll((unsigned long long)m) - 1;
        }
        if (found < 0) break;
        if (lane == 0) path[L] = found;
        L++;
        v = found;
    }
    for (int i = L + lane; i < max_nodes; i += 64) path[i] = -1;
    if (lane == 0) {
        accept_len[b] = L;
        bonus[b] = tgt[v + 1];
    }
}

}  // namespace

sd_status sd_speculate_impl(sd_ctx *c, const int32_t *d_slot_ids, int32_t batch, sd_trees out,
                            hipStream_t st) {
    if (batch == 0) return SD_OK;
    SpecParams p;
    p.g_text = c->g_text; p.g_sa = c->g_sa; p.g_bucket = c->g_bucket; p.g_N = (int32_t)c->g_N;
    p.r_text = c->r_text; p.r_len = c->r_len; p.r_stride = c->r_stride;
    p.max_slots = c->cfg.max_batch_slots; p.max_ctx = c->cfg.max_ctx_tokens;
    p.D = c->cfg.D; p.P = c->cfg.P; p.max_nodes = c->max_nodes;
    p.alpha = c->cfg.alpha; p.min_score = c->cfg.min_score;
    p.occ = c->s_occ; p.occ_n = c->s_occ_n; p.cntL = c->s_cntL; p.unit_sa = c->s_unit_sa;
    p.unit_n = c->s_unit_n; p.unit_score = c->s_unit_score; p.unit_tok = c->s_unit_tok;
    p.unit_par = c->s_unit_par; p.unit_sc = c->s_unit_sc; p.err = c->d_err;
    p.algo_bytes = c->d_algo_bytes;
    const bool stats = c->prof_mode == 2;
    const size_t lds = (size_t)c->max_nodes * (2 * sizeof(double) + 7 * sizeof(int32_t));
    const dim3 g_units((unsigned)(batch * 2 * c->cfg.P)), g_req((unsigned)batch);
    {
        sd_span sp(c, SD_K_OCCURRENCES, st);
        if (stats) hipLaunchKernelGGL(k_req_occurrences<true>, g_req, dim3(OCC_THREADS), 0, st, p, d_slot_ids);
        else hipLaunchKernelGGL(k_req_occurrences<false>, g_req, dim3(OCC_THREADS), 0, st, p, d_slot_ids);
    }
    {
        sd_span sp(c, SD_K_EXPAND, st);
        if (stats) hipLaunchKernelGGL(k_expand<true>, g_units, dim3(64), lds, st, p, d_slot_ids);
        else hipLaunchKernelGGL(k_expand<false>, g_units, dim3(64), lds, st, p, d_slot_ids);
    }
    {
        sd_span sp(c, SD_K_SELECT, st);
        if (stats) hipLaunchKernelGGL(k_select<true>, g_req, dim3(64), 0, st, p, out);
        else hipLaunchKernelGGL(k_select<false>, g_req, dim3(64), 0, st, p, out);
    }
    return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}

sd_status sd_accept_impl(sd_ctx *c, sd_trees trees, int32_t batch, const int32_t *d_target,
                         int32_t *d_accept_len, int32_t *d_accept_path, int32_t *d_bonus,
                         hipStream_t st) {
    if (batch == 0) return SD_OK;
    sd_span sp(c, SD_K_ACCEPT, st);
    hipLaunchKernelGGL(k_accept, dim3((unsigned)batch), dim3(64), 0, st, trees.d_n_nodes,
                       trees.d_tokens, trees.d_parents, trees.max_nodes, d_target, d_accept_len,
                       d_accept_path, d_bonus);
    return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}
