// Batched draft generation: MatchPattern, ExpandSpeculationTree and the best-tree choice of
// GenerateCandidateTree (Algorithm 1), for every request of a batch, both indexes and every
// pattern length p = 1..P.
//
// A node of either suffix structure is a range [lo, hi) of a sorted suffix list: the suffixes
// that start with the node's path.  COUNT = hi - lo.  The children of a node at depth d are
// the runs of equal token at offset d inside the range (an end marker, which sorts first,
// means the suffix stops there and is no child).
//
// One kernel, k_speculate, one workgroup per request (up to 16 wavefronts):
//   1. all waves: scan the context for earlier occurrences of its last token, measure how far
//      each extends to the left (up to P) and sort the occurrences by what follows them; the
//      occurrences with left-extension >= p, in that order, are the sorted suffix list of the
//      per-request structure below the pattern of length p.  Meanwhile the waves match the P
//      patterns against the global index: the suffixes that start with the context's last two
//      tokens are located (first token -> bucket, second token -> column) and, if they are
//      few, extended to the left in the same way, which settles every pattern length at once
//      and leaves their sorted suffix lists in LDS; otherwise every pattern length is
//      searched for on its own (bucket, column, then the text).
//   2. pattern lengths with equal occurrence counts share one expansion; the waves take such
//      runs from a queue in LDS and grow the trees greedily, one wavefront per tree (frontier
//      and tree in LDS, arg-max by wave-wide maxima, shortcuts for unary runs and for tied
//      single-occurrence chains).
//   3. every wave keeps its best tree; the best of the workgroup is written out.
// The same kernel has a form that first settles the previous step (acceptance of the verified
// drafts, append of the accepted tokens), and k_accept does that alone.
#include <math.h>

#include "sd_internal.h"

namespace {

struct SpecParams {
    const int32_t *g_text, *g_sa, *g_bucket, *g_tok1, *g_tok1s;
    int32_t g_N;
    const int32_t *r_text, *r_len;
    int64_t r_stride;
    int32_t max_slots, max_ctx;
    int32_t D, P, max_nodes;
    int32_t den_mode, linear;
    int32_t occ_cap;  // occurrence records (with their keys) that fit the workgroup's LDS
    int32_t key_bits; // bits of a token code (0 .. vocab) inside an occurrence's sort key
    int32_t key_toks; // tokens after an occurrence that its sort key holds: 3 if they fit, else 2
    double alpha, min_score, tau;
    uint32_t *occ;
    int32_t *unit_sa;
    int32_t *err;
    unsigned long long *counters;  // what sd_get_stats reports (SD_CTR_*)
    unsigned long long *algo_bytes;
    uint32_t *unit_ticks;  // timing variant only: wall-clock marks of each expanded unit
    uint32_t *wg_ticks;    // timing variant only: [request][16 waves][8] phase marks
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

// Values that are the same in every lane but were read through vector memory or LDS are
// "divergent" to the compiler, which then runs all the control code around them on the vector
// ALU.  uni() moves such a value into a scalar register so that compares, selects and branches
// on it become scalar instructions.
__device__ __forceinline__ int32_t uni(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ double uni(double v) {
    union { double d; int32_t i[2]; } u;
    u.d = v;
    u.i[0] = __builtin_amdgcn_readfirstlane(u.i[0]);
    u.i[1] = __builtin_amdgcn_readfirstlane(u.i[1]);
    return u.d;
}

// All cross-lane traffic of a unit stays inside one wavefront.  The LDS operations of a wave
// are issued and completed in order, so what one lane wrote is seen by a later read of another
// lane without a hardware barrier; wsync() only stops the compiler from moving LDS accesses
// across it.
__device__ __forceinline__ void wsync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// ------------------------------------------------------------------------------------------
// per-request occurrence lists
// ------------------------------------------------------------------------------------------
constexpr int OCC_LDS_SORT = 2048;

// An occurrence record (end position e, common-suffix length L <= P <= 64) as it is kept in the
// request's row of scratch memory: one word, L in the low seven bits (sd_create bounds
// max_ctx_tokens by 2^25).  In registers and in LDS a record is an int2 (e, L).
__device__ __forceinline__ uint32_t occ_pack(int2 r) { return ((uint32_t)r.x << 7) | (uint32_t)r.y; }
__device__ __forceinline__ int2 occ_unpack(uint32_t u) { return make_int2((int)(u >> 7), (int)(u & 127u)); }

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
// beyond m act as +infinity and are never touched, so m need not be a power of two.  Run by
// the whole workgroup.  With `key` given (the two tokens after each occurrence packed into one
// word, kept beside the records) most compares are decided without touching memory; equal
// keys fall back to the token-by-token compare.
__device__ __forceinline__ int2 occ_get(const int2 *arr, int i) { return arr[i]; }
__device__ __forceinline__ int2 occ_get(const uint32_t *arr, int i) { return occ_unpack(arr[i]); }
__device__ __forceinline__ void occ_put(int2 *arr, int i, int2 r) { arr[i] = r; }
__device__ __forceinline__ void occ_put(uint32_t *arr, int i, int2 r) { arr[i] = occ_pack(r); }

template <bool STATS, class Rec>
__device__ __forceinline__ void occ_sort(Rec *arr, uint64_t *key, int m, const int32_t *__restrict__ x, int depth, unsigned &nb) {
    int n2 = 1;
    while (n2 < m) n2 <<= 1;
    // Thread t handles elements t, t + blockDim, ...: a wave owns whole aligned blocks of 64
    // elements.  A step whose partners stay inside such a block needs no workgroup barrier
    // before or after another step of that kind: wave-level ordering of the LDS (or, for the
    // global-memory case, of the wave's own accesses) is enough.
    const bool wave_local_ok = key != nullptr;  // records in LDS
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            const bool mirror = j == (k >> 1);
            for (int i = threadIdx.x; i < m; i += blockDim.x) {
                int l = mirror ? (i ^ (k - 1)) : (i ^ j);
                if (l > i && l < m) {
                    const int2 a = occ_get(arr, i), b = occ_get(arr, l);
                    bool swap;
                    if (key) {
                        const uint64_t ka = key[i], kb = key[l];
                        // equal keys with the low bit clear: two occurrences that are never asked
                        // for more than the key's two tokens (see the caller): any order will do
                        swap = ka != kb ? kb < ka : ((ka & 1) ? occ_less<STATS>(x, b, a, depth, nb) : false);
                        if (swap) { key[i] = kb; key[l] = ka; }
                    } else {
                        swap = occ_less<STATS>(x, b, a, depth, nb);
                    }
                    if (swap) {
                        occ_put(arr, i, b);
                        occ_put(arr, l, a);
                    }
                }
            }
            // the step after this one: (k, j / 2), or the mirror step of 2k
            const bool local = wave_local_ok && (mirror ? k <= 64 : j < 64);
            const bool next_local = wave_local_ok && (j > 1 ? (j >> 1) < 64 : 2 * k <= 64);
            if (local && next_local) wsync();
            else __syncthreads();
        }
    }
}

// Sort key of an occurrence record (end position, left-extension): see request_occurrences.
template <bool STATS>
__device__ __forceinline__ uint64_t occ_key(const SpecParams &p, const int32_t *__restrict__ x, int2 rec,
                                            int depth, unsigned &nb) {
    const int kt = p.key_toks < depth ? p.key_toks : depth;  // (a path of D tokens ends the compare)
    const uint64_t t1 = (uint64_t)(uint32_t)(x[rec.x + 1] + 1);
    const uint64_t t2 = kt >= 2 ? (uint64_t)(uint32_t)(x[rec.x + 2] + 1) : 0ull;
    const uint64_t t3 = kt >= 3 ? (uint64_t)(uint32_t)(x[rec.x + 3] + 1) : 0ull;
    SD_CNT(4 * kt);
    const uint64_t more = floor(p.alpha * (double)rec.y) > (double)p.key_toks ? 1ull : 0ull;
    const int kb = p.key_bits;
    return p.key_toks == 3 ? (t1 << (2 * kb + 1)) | (t2 << (kb + 1)) | (t3 << 1) | more
                           : (t1 << (kb + 1)) | (t2 << 1) | more;
}

// Sort of up to one element per thread (m is at most the workgroup's size; threads without an
// element pass the key ~0).  Every wave first orders its own 64 elements with a bitonic network
// whose partners are reached by lane permutes, and leaves the keys as a sorted run in LDS; an
// element's final place is then its place in its own run plus, for every other run, the number
// of that run's keys that go before it, found by a binary search in the run (among equal keys
// of different runs the earlier run goes first).  That is some 250 instructions and 50 LDS
// reads per element, all waves at work, where a network over the whole list takes 55 steps
// with ten of them across waves (18 us for the 550 occurrences of a frequent token), and
// counting the keys that go before an element one by one is bound by LDS bandwidth (13 us).
// Equal keys whose low bit is set must be ordered by the tokens beyond the key: such groups
// (rare: the key holds three tokens) lie side by side after the placement and are put in order
// by token-by-token compares in memory.  s_rec receives the sorted records; s_key and *s_flag
// are scratch.  Every thread of the workgroup calls this (barriers inside).
template <bool STATS>
__device__ __forceinline__ void occ_sort_runs(int2 rec, uint64_t key, int m, int2 *s_rec, uint64_t *s_key,
                                              int *s_flag, const int32_t *__restrict__ x, int depth,
                                              unsigned &nb, bool presorted = false) {
    const int i = threadIdx.x, lane = i & 63, w0 = i & ~63;  // w0: where this wave's run starts
    const bool busy = w0 < m;                                // (the same for all lanes of a wave)
    if (m <= 64) {
        // One run (the usual case where contexts hardly repeat their last token): the first
        // wave's network is the whole sort, equal keys are settled inside it, and nobody waits
        // at a barrier.
        if (busy) {
            int n2 = 1;  // the network's size: elements beyond the list carry the key ~0
            while (n2 < m) n2 <<= 1;
            for (int k = 2; k <= n2; k <<= 1) {
                for (int j = k >> 1; j > 0; j >>= 1) {
                    const int src = lane ^ (j == (k >> 1) ? k - 1 : j);
                    int2 orec;
                    orec.x = __shfl(rec.x, src);
                    orec.y = __shfl(rec.y, src);
                    const uint32_t klo = (uint32_t)__shfl((int)(uint32_t)key, src);
                    const uint32_t khi = (uint32_t)__shfl((int)(uint32_t)(key >> 32), src);
                    const uint64_t okey = ((uint64_t)khi << 32) | klo;
                    const bool lower = src > lane;  // a: the lower place's element
                    const int2 a = lower ? rec : orec, b = lower ? orec : rec;
                    const uint64_t ka = lower ? key : okey, kb = lower ? okey : key;
                    bool swap;
                    if (ka != kb) swap = kb < ka;
                    else swap = ((ka & 1) && ka != ~0ull) ? occ_less<STATS>(x, b, a, depth, nb) : false;
                    if (swap) { rec = orec; key = okey; }
                }
            }
            if (lane < m) s_rec[lane] = rec;
        }
        return;
    }
    if (busy && !presorted) {
        for (int k = 2; k <= 64; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                const int src = lane ^ (j == (k >> 1) ? k - 1 : j);
                int2 orec;
                orec.x = __shfl(rec.x, src);
                orec.y = __shfl(rec.y, src);
                const uint32_t klo = (uint32_t)__shfl((int)(uint32_t)key, src);
                const uint32_t khi = (uint32_t)__shfl((int)(uint32_t)(key >> 32), src);
                const uint64_t okey = ((uint64_t)khi << 32) | klo;
                // both partners look at the same ordered pair: the lower place keeps the lower key
                const bool take = src > lane ? okey < key : key < okey;
                if (take) { rec = orec; key = okey; }
            }
        }
        s_key[i] = key;
    }
    if (i == 0) *s_flag = 0;
    __syncthreads();
    int place = lane;
    if (busy) {
        const int nruns = (m + 63) >> 6;
#pragma unroll 2
        for (int r = 0; r < nruns; r++) {
            if (r * 64 == w0) continue;
            const uint64_t *run = s_key + r * 64;
            const bool first = r * 64 < w0;  // an earlier run: its equal keys go before mine
            int pos = 0;
#pragma unroll
            for (int step = 32; step > 0; step >>= 1) {
                const uint64_t kq = run[pos + step - 1];
                pos += (first ? kq <= key : kq < key) ? step : 0;
            }
            const uint64_t kq = run[pos];
            place += pos + ((first ? kq <= key : kq < key) ? 1 : 0);
        }
    }
    __syncthreads();  // all keys have been read
    const bool mine = busy && key != ~0ull;
    if (mine) { s_rec[place] = rec; s_key[place] = key; }
    __syncthreads();
    bool tie = false;
    if (mine && (key & 1))
        tie = (place > 0 && s_key[place - 1] == key) || (place + 1 < m && s_key[place + 1] == key);
    if (tie) *s_flag = 1;
    __syncthreads();
    if (*s_flag) {
        int np = place;
        if (tie) {
            int g0 = place, g1 = place + 1;
            while (g0 > 0 && s_key[g0 - 1] == key) g0--;
            while (g1 < m && s_key[g1] == key) g1++;
            np = g0;
            for (int q = g0; q < g1; q++)
                if (q != place) np += occ_less<STATS>(x, s_rec[q], rec, depth, nb) ? 1 : 0;
        }
        __syncthreads();
        if (tie) s_rec[np] = rec;
        __syncthreads();
    }
}

// Wave-wide maximum in every lane.  Inside a row of 16 lanes the values meet through four
// data-parallel moves (lane ^ 1, lane ^ 2, 7 - lane within 8, 15 - lane within 16); the four
// row results are then read out as scalars.
template <int CTRL>
__device__ __forceinline__ int32_t dpp_move(int32_t v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}
constexpr int PICK_SCAN_MAX = 3;  // frontiers up to this size are scanned by every lane
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    uint32_t o;
    o = (uint32_t)dpp_move<DPP_XOR1>((int32_t)v); v = o > v ? o : v;
    o = (uint32_t)dpp_move<DPP_XOR2>((int32_t)v); v = o > v ? o : v;
    o = (uint32_t)dpp_move<DPP_HALF_MIRROR>((int32_t)v); v = o > v ? o : v;
    o = (uint32_t)dpp_move<DPP_MIRROR>((int32_t)v); v = o > v ? o : v;
    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int32_t)v, 0),
                   b = (uint32_t)__builtin_amdgcn_readlane((int32_t)v, 16),
                   c = (uint32_t)__builtin_amdgcn_readlane((int32_t)v, 32),
                   d = (uint32_t)__builtin_amdgcn_readlane((int32_t)v, 48);
    const uint32_t ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}

template <int CTRL>
__device__ __forceinline__ double dpp_move_f64(double v) {
    const int32_t lo = dpp_move<CTRL>(__double2loint(v)), hi = dpp_move<CTRL>(__double2hiint(v));
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double wave_max_f64(double v) {  // no NaNs among the inputs
    double o;
    o = dpp_move_f64<DPP_XOR1>(v); v = o > v ? o : v;
    o = dpp_move_f64<DPP_XOR2>(v); v = o > v ? o : v;
    o = dpp_move_f64<DPP_HALF_MIRROR>(v); v = o > v ? o : v;
    o = dpp_move_f64<DPP_MIRROR>(v); v = o > v ? o : v;
    double r = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 0),
                                __builtin_amdgcn_readlane(__double2loint(v), 0));
#pragma unroll
    for (int l = 16; l < 64; l += 16) {
        const double x = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), l),
                                          __builtin_amdgcn_readlane(__double2loint(v), l));
        r = x > r ? x : r;
    }
    return r;
}

// Inclusive prefix sum over the lanes: four shifted adds inside each row of 16 lanes (a lane
// without a source adds zero), then the totals of the rows below.
__device__ __forceinline__ int32_t wave_inclusive_sum(int32_t v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);  // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);  // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);  // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);  // row_shr:8
    const int32_t t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31),
                  t2 = __builtin_amdgcn_readlane(v, 47);
    const int row = (threadIdx.x & 63) >> 4;
    return v + (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
}

// Workgroup-shared state of one request.
struct WgShared {
    int m;           // occurrences of the context's last token
    int next;        // head of the unit queue
    int sort_flag;   // scratch of the occurrence sort
    unsigned long long ctr[SD_CTR_ACCEPT_REQUESTS];  // the request's drafting counters, on their way through the launch
    int n_surv;      // occurrences whose left-extension the one-token check did not settle
    int scan_done;   // waves that have put down the hits of their part of the context scan
    int chunk_next;  // frequent last token: the next 64 occurrences nobody has taken yet
    int early;       // the occurrences were dealt with in such parts before the barrier
    unsigned long long top_bits;  // highest SCORE of a finished tree so far (bits of the double)
    int t_new;       // context length after the append of the fused form
    int newtok[260]; // fused form: the tokens appended in this launch
    int cnt[72];     // [l]: occurrences whose left-extension is l; afterwards: is at least l
    int g_lo[65], g_hi[65];  // [p]: suffix-array range of the pattern of length p (global index)
    // global index, list form (g_mode 1): the g_n2 <= 64 suffixes that start with the context's
    // last two tokens, in suffix-array order: where each starts and how many tokens of the
    // context's tail it matches to the left (2 .. P); gcnt[l]: how many match exactly l
    int gl_pos[64], gl_L[64], gcnt[72];
    int g_mode, g_n2;
    double best_s[16];
    int best_o[16], best_n[16];
};

// MatchPattern on the per-request structure, for all pattern lengths at once, by the whole
// workgroup: the occurrences of the last token, each with its left-extension L(e) (how many
// tokens before it agree with the context's tail, capped at P), sorted by what follows them.
// The occurrences with L >= p, in that order, are the sorted suffix list below the pattern of
// length p.
// Two steps with a workgroup barrier of the caller between them: occ_scan_issue sets the
// counters and issues the first round of scan loads over the t_old tokens the context is known
// to hold at that time; request_occurrences does the rest for the context of t >= t_old tokens,
// of which those from t_old on (appended meanwhile by the first wave) are taken from `newtok`
// in LDS.  `between` is independent work of the caller (the global matches), run after this
// wave has dealt with its part of the scan, while other waves may still be at it.
// With EARLY every wave counts itself in (scan_done) once its hits are down, and `between` may
// call occ_take_chunks, which then deals with a frequent last token's occurrences before the
// barrier and says so in `early`.
struct ScanState {
    int4 v[4];         // the first round of scan loads
    int32_t last_old;  // token t_old - 1
};

template <bool STATS>
__device__ __forceinline__ void occ_scan_issue(int t_old, const int32_t *__restrict__ x, WgShared &sh,
                                               ScanState &st, unsigned &nb) {
    const int tid = threadIdx.x, nthr = blockDim.x;
    if (tid == 0) { sh.m = 0; sh.next = 0; sh.top_bits = 0; sh.n_surv = 0; sh.scan_done = 0; sh.chunk_next = 0; sh.early = 0; }
    if (tid < 72) { sh.cnt[tid] = 0; sh.gcnt[tid] = 0; }
    // Coalesced scan, 16 bytes per load, four loads in flight per thread; rows start 256-byte
    // aligned.
    const int4 *x4 = reinterpret_cast<const int4 *>(x);
    const int nq = t_old > 0 ? (t_old + 3) >> 2 : 0;
#pragma unroll
    for (int k = 0; k < 4; k++) {
        int q = k * nthr + tid;
        st.v[k] = q < nq ? x4[q] : make_int4(-1, -1, -1, -1);
        if (q < nq) SD_CNT(16);
    }
    st.last_old = t_old > 0 ? x[t_old - 1] : 0;
}

// Left-extensions when the last token has more occurrences than one trip of the workgroup
// takes (a frequent token; records in LDS): most occurrences differ from the context's tail
// in the very next token to the left.  One load per occurrence, an occurrence per thread,
// settles those; the rest is listed (in `lst`) and compared token by token as in the caller's
// loop, PP lanes per occurrence.  Out of line: the route is rare and is kept from weighing on
// the registers and the code layout of the usual one.  Called by every thread (barrier inside).
template <bool STATS>
__device__ __attribute__((noinline)) unsigned left_extensions_many(int m, int t, int P, int32_t tail,
                                                                    const int32_t *__restrict__ x,
                                                                    int2 *s_sort, int32_t *lst,
                                                                    WgShared &sh) {
    unsigned nb = 0;
    const int tid = threadIdx.x, lane = tid & 63, nthr = blockDim.x;
    const int wave = uni((int32_t)(tid >> 6)), nw = nthr >> 6;
    const int32_t tl1 = __builtin_amdgcn_readlane(tail, 1);
    for (int i = tid; i < ((m + 63) & ~63); i += nthr) {
        const bool on = i < m;
        const int e = on ? s_sort[i].x : -1;
        const int lim = e + 1 < P ? e + 1 : P;
        const bool rd = on && e != t - 1 && lim > 1;
        const int32_t vv = rd ? x[e - 1] : tl1;
        if (rd) SD_CNT(8);
        const bool one = on && (lim <= 1 || (rd && vv != tl1));  // left-extension 1
        const bool surv = on && !one;
        if (one) s_sort[i].y = 1;
        const uint64_t om = __ballot(one), sm = __ballot(surv);
        if (lane == 0 && om) atomicAdd(&sh.cnt[1], (int)__popcll(om));
        if (sm) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&sh.n_surv, (int)__popcll(sm));
            base = uni(base);
            if (surv) lst[base + __popcll(sm & lanemask_lt())] = i;
        }
    }
    __syncthreads();
    const int n_items = sh.n_surv;
    int pplog = 0;
    while ((1 << pplog) < P) pplog++;
    const int PP = 1 << pplog, G = 64 >> pplog, g = lane >> pplog, k = lane & (PP - 1);
    const uint64_t gmask = PP >= 64 ? ~0ull : ((1ull << PP) - 1ull);
    const int32_t tl = __shfl(tail, k);
    for (int j0 = wave * G; j0 < n_items; j0 += nw * G) {
        const int j = j0 + g;
        const int i = j < n_items ? lst[j] : -1;
        const int e = i >= 0 ? s_sort[i].x : -1;
        const int lim = e + 1 < P ? e + 1 : P;  // (0 for an empty place)
        const bool rd = e >= 0 && e != t - 1 && k < lim;
        const int32_t v = rd ? x[e - k] : tl;
        if (rd) SD_CNT(8);
        const uint64_t mis = __ballot(k >= 1 && k < lim && v != tl);
        const uint64_t gm = (mis >> (g << pplog)) & gmask;
        const int l = gm ? __ffsll((unsigned long long)gm) - 1 : lim;
        if (k == 0 && e >= 0) {
            s_sort[i].y = l;
            atomicAdd(&sh.cnt[l], 1);
            SD_CNT(8);
        }
    }
    return nb;
}

// Frequent last token, occurrences [64 c, 64 c + 64) of the list in LDS on one wave: their
// left-extensions (most differ from the context's tail in the very next token to the left,
// which one load per occurrence settles; the rest is compared token by token, PP lanes per
// occurrence), their sort keys, and the wave's 64-element network, which leaves records and
// keys as a sorted run in place.  No barrier: a wave takes such a part whenever it is free,
// while others are still searching the global index.
template <bool STATS>
__device__ __forceinline__ unsigned occ_chunk(int c, int m, int t, int P, int depth,
                                                         int key_toks, int key_bits, double alpha,
                                                         int32_t tail, const int32_t *__restrict__ x,
                                                         int2 *s_sort, uint64_t *s_key, WgShared &sh) {
    unsigned nb = 0;
    const int lane = threadIdx.x & 63;
    const int i = c * 64 + lane;
    const bool on = i < m;
    const int e = on ? s_sort[i].x : -1;
    const int lim = e + 1 < P ? e + 1 : P;
    const int32_t tl1 = __builtin_amdgcn_readlane(tail, 1);
    const bool rd = on && e != t - 1 && lim > 1;
    const int32_t vv = rd ? x[e - 1] : tl1;
    if (rd) SD_CNT(8);
    // the tokens behind the occurrence, for its key (rows are padded with end markers)
    const int kt = key_toks < depth ? key_toks : depth;
    const uint64_t t1 = on ? (uint64_t)(uint32_t)(x[e + 1] + 1) : 0ull;
    const uint64_t t2 = on && kt >= 2 ? (uint64_t)(uint32_t)(x[e + 2] + 1) : 0ull;
    const uint64_t t3 = on && kt >= 3 ? (uint64_t)(uint32_t)(x[e + 3] + 1) : 0ull;
    if (on) SD_CNT(4 * kt);
    const bool one = on && (lim <= 1 || (rd && vv != tl1));  // left-extension 1
    uint64_t sm = __ballot(on && !one);
    int pplog = 0;
    while ((1 << pplog) < P) pplog++;
    const int PP = 1 << pplog, G = 64 >> pplog, g = lane >> pplog, k = lane & (PP - 1);
    const uint64_t gmask = PP >= 64 ? ~0ull : ((1ull << PP) - 1ull);
    const int32_t tl = __shfl(tail, k);
    while (sm) {  // G of the others per trip, PP lanes each
        int src = -1;
        for (int q = 0; q < G && sm; q++) {
            const int l = __ffsll((unsigned long long)sm) - 1;
            sm &= sm - 1;
            if (g == q) src = l;
        }
        const int es = __shfl(e, src >= 0 ? src : lane);
        const int ee = src >= 0 ? es : -1;
        const int lims = ee + 1 < P ? ee + 1 : P;  // (0 for an empty place)
        const bool rdk = ee >= 0 && ee != t - 1 && k < lims;
        const int32_t v = rdk ? x[ee - k] : tl;
        if (rdk) SD_CNT(8);
        const uint64_t mis = __ballot(k >= 1 && k < lims && v != tl);
        const uint64_t gm = (mis >> (g << pplog)) & gmask;
        const int l = gm ? __ffsll((unsigned long long)gm) - 1 : lims;
        if (k == 0 && ee >= 0) {
            s_sort[c * 64 + src].y = l;
            SD_CNT(8);
        }
    }
    wsync();
    const int L = one ? 1 : (on ? s_sort[i].y : 0);
    if (on) atomicAdd(&sh.cnt[L], 1);
    int2 rec = make_int2(e, L);
    uint64_t key = ~0ull;
    if (on) {
        const uint64_t more = floor(alpha * (double)L) > (double)key_toks ? 1ull : 0ull;
        key = key_toks == 3 ? (t1 << (2 * key_bits + 1)) | (t2 << (key_bits + 1)) | (t3 << 1) | more
                            : (t1 << (key_bits + 1)) | (t2 << 1) | more;
    }
    for (int kk = 2; kk <= 64; kk <<= 1) {
        for (int j = kk >> 1; j > 0; j >>= 1) {
            const int src = lane ^ (j == (kk >> 1) ? kk - 1 : j);
            int2 orec;
            orec.x = __shfl(rec.x, src);
            orec.y = __shfl(rec.y, src);
            const uint32_t klo = (uint32_t)__shfl((int)(uint32_t)key, src);
            const uint32_t khi = (uint32_t)__shfl((int)(uint32_t)(key >> 32), src);
            const uint64_t okey = ((uint64_t)khi << 32) | klo;
            // both partners look at the same ordered pair: the lower place keeps the lower key
            const bool take = src > lane ? okey < key : key < okey;
            if (take) { rec = orec; key = okey; }
        }
    }
    wsync();
    s_sort[i] = rec;  // (within the room of the list's 64-entry parts: the LDS holds whole parts)
    s_key[i] = key;
    return nb;
}

// What a wave does with a frequent last token once its own search in the global index is over
// (per-pattern route only, where the waves' searches take unequal times): it waits until every
// wave's hits are down (each wave has counted itself in before it waits for anything, so the
// wait ends; it is over long before a wave gets here), and if the list is of the kind that
// request_occurrences sorts with one element per thread, it takes parts of 64 occurrences
// until none is left: left-extensions, keys and the per-wave part of the sort then do not wait
// behind the workgroup's barrier for the slowest search.  Out of line: the route is rare and is
// kept from weighing on the registers and the code layout of the usual one.
template <bool STATS>
__device__ __attribute__((noinline)) unsigned occ_take_chunks(int nw, int t, int P, int depth, int occ_cap,
                                                               int key_toks, int key_bits, double alpha,
                                                               int32_t tail, const int32_t *__restrict__ x,
                                                               int2 *s_sort, WgShared &sh) {
    unsigned nb = 0;
    const int lane = threadIdx.x & 63;
    while (__hip_atomic_load(&sh.scan_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < nw)
        __builtin_amdgcn_s_sleep(1);
    wsync();
    const int m_all = __hip_atomic_load(&sh.m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    int pplog = 0;
    while ((1 << pplog) < P) pplog++;
    if (!(m_all > nw * (64 >> pplog) * 4 && m_all <= occ_cap && m_all <= nw * 64)) return 0;
    uint64_t *s_key = reinterpret_cast<uint64_t *>(s_sort + occ_cap);
    if (lane == 0) sh.early = 1;  // (every wave that gets here writes the same)
    for (;;) {
        int c = 0;
        if (lane == 0) c = atomicAdd(&sh.chunk_next, 1);
        c = uni(c);
        if (c * 64 >= m_all) break;
        nb += occ_chunk<STATS>(c, m_all, t, P, depth, key_toks, key_bits, alpha, tail, x, s_sort, s_key, sh);
    }
    return nb;
}

template <bool STATS, bool EARLY, class Between>
__device__ __forceinline__ void request_occurrences(const SpecParams &p, int b, int t, int t_old,
                                    const int32_t *newtok, const int32_t *__restrict__ x,
                                    int2 *s_sort, WgShared &sh, ScanState &st, int32_t tail,
                                    unsigned &nb, Between between) {
    const int tid = threadIdx.x, lane = tid & 63, nthr = blockDim.x;
    uint32_t *occ = p.occ + (int64_t)b * p.max_ctx;
    const int4 *x4 = reinterpret_cast<const int4 *>(x);
    const int nq = t_old > 0 ? (t_old + 3) >> 2 : 0;
    int4(&v)[4] = st.v;
    const int n_new = t - t_old;
    const int occ_cap = p.occ_cap;  // records the workgroup's LDS can sort
    const int32_t last = n_new > 0 ? newtok[n_new - 1] : st.last_old;
    if (t > 0) {
        // the first t_old tokens, from memory (what sits behind them in a loaded word is not
        // looked at: end markers, or appended tokens that the load may have missed)
        for (int q0 = 0; q0 < nq; q0 += 4 * nthr) {
            if (q0 > 0) {
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    int q = q0 + k * nthr + tid;
                    v[k] = q < nq ? x4[q] : make_int4(-1, -1, -1, -1);
                    if (q < nq) SD_CNT(16);
                }
            }
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const int e0 = 4 * (q0 + k * nthr + tid);
                const int h0 = v[k].x == last && e0 < t_old, h1 = v[k].y == last && e0 + 1 < t_old,
                          h2 = v[k].z == last && e0 + 2 < t_old, h3 = v[k].w == last && e0 + 3 < t_old;
                const int nh = h0 + h1 + h2 + h3;
                if (__ballot(nh > 0)) {
                    // hits in the lanes below this one: nh <= 4, one ballot per bit of it
                    const uint64_t b0 = __ballot(nh & 1), b1 = __ballot(nh & 2), b2 = __ballot(nh & 4);
                    const uint64_t lt = lanemask_lt();
                    const int below = __popcll(b0 & lt) + 2 * __popcll(b1 & lt) + 4 * __popcll(b2 & lt);
                    const int all = __popcll(b0) + 2 * __popcll(b1) + 4 * __popcll(b2);
                    int off = 0;
                    if (lane == 0) off = atomicAdd(&sh.m, all);
                    off = uni(off) + below;
                    // the first occ_cap hits are also kept in LDS, where they are sorted
                    const int es[4] = {e0, e0 + 1, e0 + 2, e0 + 3};
                    const int hs[4] = {h0, h1, h2, h3};
#pragma unroll
                    for (int c = 0; c < 4; c++)
                        if (hs[c]) {
                            occ[off] = occ_pack(make_int2(es[c], 0));
                            if (off < occ_cap) s_sort[off].x = es[c];
                            off++;
                        }
                }
            }
        }
        // the appended tokens, from LDS
        if (tid < 64) {
            for (int i0 = 0; i0 < n_new; i0 += 64) {
                const int i = i0 + lane;
                const uint64_t hm = __ballot(i < n_new && newtok[i] == last);
                if (hm) {
                    int off = 0;
                    if (lane == 0) off = atomicAdd(&sh.m, (int)__popcll(hm));
                    off = uni(off) + __popcll(hm & lanemask_lt());
                    if ((hm >> lane) & 1) {
                        occ[off] = occ_pack(make_int2(t_old + i, 0));
                        if (off < occ_cap) s_sort[off].x = t_old + i;
                    }
                }
            }
        }
    }
    // (this wave's hits are down: the count below says when every wave's are.  The hits and
    // the count are LDS operations of one wave, which the LDS takes in the order they were
    // issued: the compiler must keep that order, nothing has to be waited for.)
    if (EARLY) {
        wsync();
        if (lane == 0) atomicAdd(&sh.scan_done, 1);
    }
    between();
    __syncthreads();
    const int m = sh.m;
    // (a frequent last token's occurrences may have been dealt with already, in parts of 64 by
    // the waves that came out of the caller's work early: see occ_take_chunks)
    const bool early = EARLY && uni(sh.early) != 0;
    // A single occurrence is the context's own last token: nothing follows it, so no pattern
    // has a continuation in this index, and the counts stay at zero, which says just that.
    if (__builtin_expect(m <= 1, 1)) return;
    const bool in_lds = m <= occ_cap;
    // How far each occurrence extends to the left together with the context's own tail.  An
    // occurrence takes PP lanes (P rounded up to a power of two): lane k of them compares the
    // k-th token before both ends.  A wave handles 64 / PP occurrences side by side and four
    // such batches per trip, all loads of a trip in flight together.
    {
        const int wave = uni((int32_t)(tid >> 6)), nw = nthr >> 6;
        int pplog = 0;
        while ((1 << pplog) < p.P) pplog++;
        const int PP = 1 << pplog, G = 64 >> pplog, g = lane >> pplog, k = lane & (PP - 1);
        const uint64_t gmask = PP >= 64 ? ~0ull : ((1ull << PP) - 1ull);
        const int32_t tl = __shfl(tail, k);  // the k-th token from the context's end (0 beyond it)
        constexpr int U = 4;
        if (early) {
            // (done already, see above)
        } else if (__builtin_expect(in_lds && m > nw * G * U, 0)) {
            // (the room of the sort keys, free until the sort, takes the list)
            const unsigned cnt_many = left_extensions_many<STATS>(
                m, t, p.P, tail, x, s_sort, reinterpret_cast<int32_t *>(s_sort + occ_cap), sh);
            SD_CNT(cnt_many);
        } else
        for (int i0 = wave * G * U; i0 < m; i0 += nw * G * U) {
            int e[U];
            int32_t v[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int i = i0 + u * G + g;
                e[u] = i < m ? (in_lds ? s_sort[i].x : occ_unpack(occ[i]).x) : -1;
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int lim = e[u] + 1 < p.P ? e[u] + 1 : p.P;  // (0 for an empty place)
                // the context's own tail agrees with itself all the way: nothing to read
                const bool rd = e[u] >= 0 && e[u] != t - 1 && k < lim;
                v[u] = rd ? x[e[u] - k] : tl;
                if (rd) SD_CNT(8);
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int lim = e[u] + 1 < p.P ? e[u] + 1 : p.P;
                const uint64_t mis = __ballot(k >= 1 && k < lim && v[u] != tl);
                const uint64_t gm = (mis >> (g << pplog)) & gmask;
                const int l = gm ? __ffsll((unsigned long long)gm) - 1 : lim;
                if (k == 0 && e[u] >= 0) {
                    const int i = i0 + u * G + g;
                    if (in_lds) s_sort[i].y = l;
                    else occ[i] = occ_pack(make_int2(e[u], l));
                    atomicAdd(&sh.cnt[l], 1);
                    SD_CNT(8);
                }
            }
        }
    }
    __syncthreads();
    if (tid < 64) {  // cnt[l] becomes the sum over l' >= l (lane k holds cnt[P - k], so that a
                     // prefix sum over the lanes does it); nothing below reads cnt before the
                     // closing barrier
        const bool mine = lane < p.P;
        const int c = wave_inclusive_sum(mine ? sh.cnt[p.P - lane] : 0);
        if (mine) sh.cnt[p.P - lane] = c;
        if (lane == 0) sh.cnt[0] = m;
    }
    if (m > 0) {
        const int depth = p.D - 1;
        if (in_lds) {
            if (m > 1) {
                // Sort key: the three tokens after the occurrence (two if three codes do not fit
                // 63 bits), end marker lowest (rows are padded with end markers, and only a
                // pattern's own tail is followed by one), then one bit that says whether the
                // occurrence can ever be asked for more.  An occurrence with left-extension L
                // belongs to the lists of the patterns p <= L, whose trees have at most
                // floor(alpha p) <= floor(alpha L) nodes and therefore look at no token further
                // than that many places behind it.  Where that is no more than the key holds,
                // the key is the whole order; such occurrences come before the others of the
                // same key, which are ordered among themselves by the tokens beyond.  (With two
                // tokens per key the sort of 550 occurrences of a frequent token took 18 us on
                // the low-repetition workload: every step of the network in which some pair of
                // a wave has equal keys waits for that pair's token-by-token compare in memory.)
                uint64_t *key = reinterpret_cast<uint64_t *>(s_sort + occ_cap);
                if (m <= nthr) {  // one element per thread
                    int2 rec = make_int2(0, 0);
                    uint64_t kk = ~0ull;
                    if (early) {  // the runs of 64 are sorted already, keys beside them
                        if ((tid & ~63) < m) { rec = s_sort[tid]; kk = key[tid]; }
                    } else if (tid < m) {
                        rec = s_sort[tid];
                        kk = occ_key<STATS>(p, x, rec, depth, nb);
                    }
                    occ_sort_runs<STATS>(rec, kk, m, s_sort, key, &sh.sort_flag, x, depth, nb, early);
                } else {
                    for (int i = tid; i < m; i += nthr) key[i] = occ_key<STATS>(p, x, s_sort[i], depth, nb);
                    __syncthreads();
                    occ_sort<STATS>(s_sort, key, m, x, depth, nb);
                }
            }
            for (int i = tid; i < m; i += nthr) occ[i] = occ_pack(s_sort[i]);
        } else {
            occ_sort<STATS>(occ, nullptr, m, x, depth, nb);
        }
    }
    __threadfence_block();
    __syncthreads();
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

struct Frontier {
    double *score;
    int32_t *tok, *par, *lo, *hi, *dep;
    int n, cap;
};

// Best (want_best) or worst entry of the frontier; every lane returns
// the same key (idx < 0: there is none).  Lane l looks at the entries l, l + 64, ...; across
// the lanes the extreme score is found first, and only if several lanes hold it the extreme
// token among those, then the extreme parent.
__device__ __forceinline__ Key frontier_pick(const Frontier &f, bool want_best) {
    const int lane = threadIdx.x & 63;
    Key mine;
    mine.idx = -1; mine.s = 0.0; mine.tok = 0; mine.par = 0;
    if (f.n <= PICK_SCAN_MAX) {  // a handful of entries: every lane scans them all (broadcast reads)
        for (int i = 0; i < f.n; i++) {
            Key k;
            k.s = f.score[i]; k.tok = f.tok[i]; k.par = f.par[i]; k.idx = i;
            if (mine.idx < 0 || (want_best ? key_better(k, mine) : key_better(mine, k))) mine = k;
        }
        mine.s = uni(mine.s); mine.tok = uni(mine.tok); mine.par = uni(mine.par);
        mine.idx = uni(mine.idx);
        return mine;
    }
    for (int i = lane; i < f.n; i += 64) {
        Key k;
        k.s = f.score[i]; k.tok = f.tok[i]; k.par = f.par[i]; k.idx = i;
        if (mine.idx < 0 || (want_best ? key_better(k, mine) : key_better(mine, k))) mine = k;
    }
    const bool valid = mine.idx >= 0;
    // scores are positive and finite; tokens are >= 0 and parents >= -1 in the frontier.  The
    // worst entry has the lowest score, then the highest token, then the highest parent.
    const double sv = valid ? (want_best ? mine.s : -mine.s) : -__longlong_as_double(0x7ff0000000000000ll);
    const double sx = wave_max_f64(sv);
    uint64_t T = __ballot(valid && sv == sx);
    if (T & (T - 1)) {
        const uint32_t tv = (uint32_t)mine.tok, tk = want_best ? ~tv : tv;
        const bool in1 = (T >> lane) & 1;
        const uint32_t tx = wave_max_u32(in1 ? tk : 0u);
        T = __ballot(in1 && tk == tx);
        if (T & (T - 1)) {
            const uint32_t pv = (uint32_t)(mine.par + 1), pk = want_best ? ~pv : pv;
            const bool in2 = (T >> lane) & 1;
            const uint32_t px = wave_max_u32(in2 ? pk : 0u);
            T = __ballot(in2 && pk == px);
        }
    }
    Key r;
    r.idx = -1; r.s = 0.0; r.tok = 0; r.par = 0;
    if (T) {
        const int w = __ffsll((unsigned long long)T) - 1;
        r.s = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(mine.s), w),
                               __builtin_amdgcn_readlane(__double2loint(mine.s), w));
        r.tok = __builtin_amdgcn_readlane(mine.tok, w);
        r.par = __builtin_amdgcn_readlane(mine.par, w);
        r.idx = __builtin_amdgcn_readlane(mine.idx, w);
    }
    return r;
}

// The best entry together with its suffix range and depth, and how many entries hold its
// score (several may be tied chains; a single one is strictly above everything else): what
// the expansion loop needs of the frontier per step, from one round of LDS reads.
struct Taken {
    Key k;
    int32_t lo, hi, dep;
    int ntop;
};
__device__ __forceinline__ Taken frontier_take(const Frontier &f) {
    const int lane = threadIdx.x & 63;
    Taken r;
    if (__builtin_expect(f.n > 64, 0)) {  // more entries than lanes: the parts one by one
        r.k = frontier_pick(f, true);
        r.lo = uni(f.lo[r.k.idx]); r.hi = uni(f.hi[r.k.idx]); r.dep = uni(f.dep[r.k.idx]);
        r.ntop = 0;
        for (int i0 = 0; i0 < f.n; i0 += 64) {
            const int i = i0 + lane;
            r.ntop += __popcll(__ballot(i < f.n && f.score[i] == r.k.s));
        }
        return r;
    }
    // lane l holds entry l
    const bool valid = lane < f.n;
    const int li = valid ? lane : 0;
    const double ms = f.score[li];
    const int32_t mtok = f.tok[li], mpar = f.par[li], mlo = f.lo[li], mhi = f.hi[li], mdep = f.dep[li];
    const double ninf = -__longlong_as_double(0x7ff0000000000000ll);
    const double sx = wave_max_f64(valid ? ms : ninf);
    uint64_t T = __ballot(valid && ms == sx);
    r.ntop = __popcll(T);
    if (T & (T - 1)) {  // lowest token among those, then lowest parent
        const uint32_t tk = ~(uint32_t)mtok;
        const bool in1 = (T >> lane) & 1;
        const uint32_t tx = wave_max_u32(in1 ? tk : 0u);
        T = __ballot(in1 && tk == tx);
        if (T & (T - 1)) {
            const uint32_t pk = ~(uint32_t)(mpar + 1);
            const bool in2 = (T >> lane) & 1;
            const uint32_t px = wave_max_u32(in2 ? pk : 0u);
            T = __ballot(in2 && pk == px);
        }
    }
    const int w = __ffsll((unsigned long long)T) - 1;  // f.n > 0: there is one
    r.k.s = sx;
    r.k.tok = __builtin_amdgcn_readlane(mtok, w);
    r.k.par = __builtin_amdgcn_readlane(mpar, w);
    r.k.idx = w;
    r.lo = __builtin_amdgcn_readlane(mlo, w);
    r.hi = __builtin_amdgcn_readlane(mhi, w);
    r.dep = __builtin_amdgcn_readlane(mdep, w);
    return r;
}

// close the slot freed by the node just taken: the last entry moves into it
__device__ __forceinline__ void frontier_close(Frontier &f, int hole) {
    if (hole < 0) return;
    const int last = f.n - 1;
    if (hole != last && (threadIdx.x & 63) == 0) {
        f.score[hole] = f.score[last]; f.tok[hole] = f.tok[last]; f.par[hole] = f.par[last];
        f.lo[hole] = f.lo[last]; f.hi[hole] = f.hi[last]; f.dep[hole] = f.dep[last];
    }
    f.n = last;
    wsync();
}

// Add the candidates held by the lanes with `cand` set; `hole` (>= 0) is the slot of the node
// just taken, which the first candidate reuses.  The frontier keeps at most `cap` entries: a
// candidate that does not rank among the best `cap` can never be selected, because at most
// `cap` more nodes are ever taken from it.
__device__ __forceinline__ void frontier_put(Frontier &f, int hole, bool cand, double sc, int32_t tok, int32_t par,
                             int32_t lo, int32_t hi, int32_t dep) {
    const int lane = threadIdx.x & 63;
    uint64_t C = __ballot(cand);
    if (C == 0) {
        frontier_close(f, hole);
        return;
    }
    const int nc = __popcll(C);
    const int stay = f.n - (hole >= 0 ? 1 : 0);
    if (__builtin_expect(stay + nc <= f.cap, 1)) {
        if (cand) {
            int j = __popcll(C & lanemask_lt());
            int s = hole >= 0 ? (j == 0 ? hole : f.n + j - 1) : f.n + j;
            f.score[s] = sc; f.tok[s] = tok; f.par[s] = par; f.lo[s] = lo; f.hi[s] = hi;
            f.dep[s] = dep;
        }
        f.n = stay + nc;
        wsync();
        return;
    }
    frontier_close(f, hole);
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
        wsync();
    }
}

// LDS staging of one narrow part of a suffix list: the positions of up to 64 consecutive
// suffixes and, per suffix, a window of W consecutive tokens starting at depth cb[slot].
// Sibling branches of the speculation tree are disjoint suffix ranges and a suffix is only
// ever asked for deeper tokens, so each slot's window moves forward only.  With W tokens per
// slot one coalesced fill serves W levels of the tree: expansion then runs out of LDS.
constexpr int TC_TOKENS = 512;
constexpr int FILL_U = TC_TOKENS / 64;  // loads per lane that fill all the windows of a wave
constexpr int CB_NONE = -(1 << 30);
constexpr int CHAIN_MAX_M = 8;  // widest node the unary-run shortcut looks at
constexpr int MED_MAX = 256;  // widest node whose suffixes are all read (a multiple of 64)

struct Stage {
    int32_t *pos, *cb, *tc;  // LDS: [64], [64], [TC_TOKENS]
    int32_t *tmp;            // LDS: [128] scratch of the chain merge
    int lo, m, wlog;         // staged range [lo, lo + m) of the suffix list, window = 1 << wlog
};

__device__ __forceinline__ void stage_set_width(Stage &s, int m) {
    int p2 = 1;
    while (p2 < m) p2 <<= 1;
    int w = TC_TOKENS / p2;
    if (w > 64) w = 64;
    s.wlog = 31 - __clz(w);
}

// Stage the node [lo, lo + m) (m <= 64) and make every one of its windows cover depth d.
// Returns the window base of this lane's suffix (lanes < m).
__device__ __forceinline__ int stage_node(Stage &sg, const int32_t *__restrict__ sa,
                                          const int32_t *__restrict__ text, int32_t lo, int32_t m,
                                          int32_t d) {
    const int lane = threadIdx.x & 63;
    const bool in = lane < m;
    if (!(lo >= sg.lo && lo + m <= sg.lo + sg.m)) {
        sg.lo = lo;
        sg.m = m;
        stage_set_width(sg, m);
        if (in) {
            sg.pos[lane] = sa[lo + lane];
            sg.cb[lane] = CB_NONE;
        }
        wsync();
    }
    const int slot0 = lo - sg.lo, slot = slot0 + lane;
    const int W = 1 << sg.wlog;
    int mycb = in ? sg.cb[slot] : d;
    const bool miss = in && !(mycb <= d && d < mycb + W);
    if (__ballot(miss)) {  // move the windows of this node's suffixes to depth d
        wsync();
        if (in) sg.cb[slot] = d;
        // (at most TC_TOKENS tokens, FILL_U loads per lane, all of them in flight together: a
        // loop of load, wait, store took a memory round trip per 64 tokens)
        const int total = m << sg.wlog;
        int32_t v[FILL_U];
#pragma unroll
        for (int u = 0; u < FILL_U; u++) {
            const int idx = u * 64 + lane;
            v[u] = 0;
            if (u * 64 < total && idx < total)
                v[u] = text[(int64_t)sg.pos[slot0 + (idx >> sg.wlog)] + d + (idx & (W - 1))];
        }
#pragma unroll
        for (int u = 0; u < FILL_U; u++) {
            const int idx = u * 64 + lane;
            if (u * 64 < total && idx < total) sg.tc[(slot0 << sg.wlog) + idx] = v[u];
        }
        wsync();
        mycb = d;
    }
    return mycb;
}

// Lane l: the token that all m staged suffixes from slot0 on hold at depth d + l, or -2 if they
// differ there or a window does not reach that far (m <= M).  The window bases come from the
// lanes' registers and all tokens are read in one round of LDS reads (the slots past m repeat
// the last suffix).
template <int M>
__device__ __forceinline__ int32_t common_token(const Stage &sg, int slot0, int m, int d, int W,
                                                int32_t mycb) {
    const int lane = threadIdx.x & 63;
    int32_t off[M], v[M];
    // window base of suffix i: lane i's value of `mycb` (what stage_node returned)
#pragma unroll
    for (int i = 0; i < M; i++) {
        const int ii = i < m ? i : m - 1;
        off[i] = d + lane - __builtin_amdgcn_readlane(mycb, ii);
    }
#pragma unroll
    for (int i = 0; i < M; i++) {
        const int ii = i < m ? i : m - 1;
        const int o = off[i] < W ? off[i] : W - 1;
        v[i] = sg.tc[((slot0 + ii) << sg.wlog) + o];
    }
    int32_t tk = off[0] < W ? v[0] : -2;
#pragma unroll
    for (int i = 1; i < M; i++) tk = (off[i] < W && v[i] == tk) ? tk : -2;
    return tk;
}

// Children of the node [lo, hi) at depth d (its path has d tokens), as frontier candidates with
// score = ps * (COUNT(child) / COUNT(node)).  `hole` is the frontier slot the node came from.
template <bool STATS>
__device__ __forceinline__ void push_children(Frontier &f, int hole, Stage &sg, const int32_t *__restrict__ sa,
                              const int32_t *__restrict__ text, int32_t lo, int32_t hi, int32_t d,
                              int32_t parent, double ps, double min_score, int32_t D, int den_mode,
                              unsigned &nb) {
    if (d >= D) {  // a path of D tokens has no continuation
        frontier_close(f, hole);
        return;
    }
    const int lane = threadIdx.x & 63;
    const int32_t m = hi - lo;
    if (__builtin_expect(m <= 64, 1)) {
        const bool in = lane < m;
        const int mycb = stage_node(sg, sa, text, lo, m, d);
        int32_t tok = 0x7fffffff;
        if (in) tok = sg.tc[((lo - sg.lo + lane) << sg.wlog) + (d - mycb)];
        if (in) SD_CNT(8);
        // denominator of C(N): all occurrences of the node, or (den_mode 1) only those that
        // go on, i.e. the sum over the children
        const int32_t dn = den_mode ? m - __popcll(__ballot(in && tok < 0)) : m;
        const double den = (double)dn;
        int32_t prev = __shfl_up(tok, 1);
        bool start = in && (lane == 0 || tok != prev);
        uint64_t S = __ballot(start);
        uint64_t above = lane == 63 ? 0ull : (S >> (lane + 1));
        int32_t e = above ? lane + 1 + (__ffsll((unsigned long long)above) - 1) : m;
        int32_t c = e - lane;
        double sc = c == dn ? ps : ps * ((double)c / den);  // x / x == 1 and ps * 1 == ps exactly
        bool cand = start && tok >= 0 && sc >= min_score;
        frontier_put(f, hole, cand, sc, tok, parent, lo + lane, lo + e, d + 1);
        return;
    }
    if (m <= MED_MAX) {
        // Medium node: read the next token of every suffix (all loads in flight together) and
        // take the children from the run boundaries, 64 suffixes at a time.  A run that is
        // still open at the end of a group of 64 is carried into the next group.
        frontier_close(f, hole);
        int32_t tk[MED_MAX / 64];
        int64_t ps_[MED_MAX / 64];
#pragma unroll
        for (int c = 0; c < MED_MAX / 64; c++) {
            const int32_t i = lo + c * 64 + lane;
            ps_[c] = i < hi ? sa[i] : 0;
        }
        int32_t ended = 0;
#pragma unroll
        for (int c = 0; c < MED_MAX / 64; c++) {
            const bool in = lo + c * 64 + lane < hi;
            tk[c] = in ? text[ps_[c] + d] : 0x7fffffff;
            if (in) SD_CNT(8);
            ended += __popcll(__ballot(in && tk[c] < 0));
        }
        const int32_t dn = den_mode ? m - ended : m;
        if (dn == 0) return;
        const double den = (double)dn;
        bool open = false;  // the carried run: token and first position
        int32_t otok = 0, olb = 0;
#pragma unroll
        for (int c = 0; c < MED_MAX / 64; c++) {
            const int32_t base = lo + c * 64;
            if (base >= hi) break;
            const bool in = base + lane < hi, lastgrp = base + 64 >= hi;
            const int32_t tok = tk[c];
            int32_t prev = __shfl_up(tok, 1);
            if (lane == 0) prev = c == 0 ? (int32_t)0x80000000 : __builtin_amdgcn_readlane(tk[c > 0 ? c - 1 : 0], 63);
            const bool start = in && tok != prev;
            const uint64_t S = __ballot(start);
            if (open && (S || lastgrp)) {  // the carried run ends at the first start of this group
                const int32_t ub = S ? base + __ffsll((unsigned long long)S) - 1 : hi;
                const int32_t cnt = ub - olb;
                const double sc = cnt == dn ? ps : ps * ((double)cnt / den);
                frontier_put(f, -1, lane == 0 && otok >= 0 && sc >= min_score, sc, otok, parent, olb, ub,
                             d + 1);
                open = false;
            }
            if (S) {
                const uint64_t above = lane == 63 ? 0ull : (S >> (lane + 1));
                const bool closed = above != 0 || lastgrp;
                const int32_t e = above ? base + lane + 1 + (__ffsll((unsigned long long)above) - 1) : hi;
                const int32_t cnt = e - (base + lane);
                const double sc = cnt == dn ? ps : ps * ((double)cnt / den);
                const bool cand = start && closed && tok >= 0 && sc >= min_score;
                frontier_put(f, -1, cand, sc, tok, parent, base + lane, e, d + 1);
                if (!lastgrp) {  // the last run of the group stays open
                    const int ll = 63 - __clzll((unsigned long long)S);
                    open = true;
                    otok = __builtin_amdgcn_readlane(tok, ll);
                    olb = base + ll;
                }
            }
        }
        return;
    }
    // Wide node: a child that can still reach min_score has at least c_min occurrences, so its
    // run contains one of the positions lo, lo + c_min, lo + 2 c_min, ...  Probe those, then
    // bracket the run of each distinct probed token by a multi-way search.  The bound is taken a
    // little low (factor 1 - 1e-9) so that rounding can never hide an admissible child; the
    // exact binary64 test below decides.
    frontier_close(f, hole);
    int32_t dn = m;
    if (den_mode) {  // leave out the suffixes that stop here: they sit first in the range
        int32_t l = lo, h = hi;
        while (l < h) {
            int32_t mid = l + ((h - l) >> 1);
            if (lane == 0) SD_CNT(8);
            if (text[(int64_t)sa[mid] + d] < 0) l = mid + 1; else h = mid;
        }
        dn = hi - l;
        if (dn == 0) return;
    }
    const double den = (double)dn;
    int64_t stride = (int64_t)floor(min_score * den / ps * (1.0 - 1e-9));
    if (stride < 1) stride = 1;
    int64_t np = ((int64_t)m + stride - 1) / stride;
    // Where the probes a stride apart would leave most of the wave idle, the whole wave probes
    // at a finer step instead: an admissible run (at least `stride` long) then holds at least
    // floor(stride / step) probes in a row, which rules out most of the probed tokens at once
    // (on independent tokens nearly every probe a stride apart shows another token, and the
    // searches below share the wave: 10 candidates leave 3 probes per search and round, one
    // candidate 32), and the ends of a run are bracketed that much more narrowly.
    int need = 1;
    {
        const int64_t fine = ((int64_t)m + 63) / 64;
        if (fine < stride) {
            need = (int)(stride / fine);
            stride = fine;
            np = ((int64_t)m + stride - 1) / stride;  // <= 64: one group of probes
        }
    }
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
        const bool change = in && tok != prevtok;
        // The run of a probed token starts in (q - stride, q] and ends behind the last probe
        // that holds the token: before the next probe if there is one (in this group of 64),
        // else before hi, which is at most a stride away unless further groups follow.
        const uint64_t Cm = __ballot(change);
        const uint64_t above = lane == 63 ? 0ull : (Cm >> (lane + 1));
        const int n_in = np - k0 < 64 ? (int)(np - k0) : 64;  // probes in this group
        int nxt = above ? lane + 1 + (__ffsll((unsigned long long)above) - 1) : 64;
        if (nxt > n_in) nxt = n_in;  // the next probe with another token, or the end of the group
        // (need > 1 only with a single group, where the probes that hold a token are all in sight)
        const bool first = change && tok >= 0 && nxt - lane >= need;
        const int32_t q_ls = (int32_t)(q + (int64_t)(nxt - 1 - lane) * stride);
        int32_t lb_lo = q, lb_hi = q, ub_lo = q_ls + 1, ub_hi = hi;  // (hi: the run may go on into the next group)
        if (k > 0) lb_lo = (int32_t)(q - stride + 1);
        if (nxt < n_in) ub_hi = (int32_t)(q_ls + stride);
        int32_t lb = q, ub = hi;
        const uint64_t Fm = __ballot(first);
        const int nf = __popcll(Fm);
        if (nf > 0 && nf <= 32) {
            // All 2 nf searches (lower and upper end of every run) side by side: search j gets
            // G lanes, which probe G points of its interval per round ((G + 1)-ary search).
            const int G = 64 / (2 * nf);
            wsync();
            if (first) sg.tmp[__popcll(Fm & lanemask_lt())] = lane;
            wsync();
            const int srch = lane / G, sub = lane - srch * G;
            const bool act = srch < 2 * nf;
            const int srcl = act ? sg.tmp[srch >> 1] : 0;
            const bool upper = srch & 1;
            const int32_t ctok = __shfl(tok, srcl);
            // (the shuffles run with all lanes on; the choice between the two ends is the
            // reading lane's)
            const int32_t l0 = __shfl(lb_lo, srcl), h0 = __shfl(lb_hi, srcl);
            const int32_t l1 = __shfl(ub_lo, srcl), h1 = __shfl(ub_hi, srcl);
            int32_t l = upper ? l1 : l0, h = upper ? h1 : h0;
            if (!act) { l = 0; h = 0; }
            const uint64_t gmask = G >= 64 ? ~0ull : ((1ull << G) - 1ull);
            while (__ballot(l < h)) {
                const bool go = l < h;
                const int64_t n = (int64_t)h - l;
                const int32_t pt = (int32_t)(l + n * (sub + 1) / (G + 1));
                int32_t v = 0;
                if (go) v = text[(int64_t)sa[pt] + d];
                if (go) SD_CNT(8);
                // the answer is the first position whose token is >= (lower end) or > (upper
                // end) the run's token: the probes that say "not yet" form a prefix
                const bool notyet = go && (upper ? v <= ctok : v < ctok);
                const uint64_t nm = __ballot(notyet);
                const int cf = __popcll((nm >> (srch * G)) & gmask);
                const int32_t nl = cf > 0 ? (int32_t)(l + n * cf / (G + 1)) + 1 : l;
                const int32_t nh = cf < G ? (int32_t)(l + n * (cf + 1) / (G + 1)) : h;
                if (go) { l = nl; h = nh; }
            }
            const int r = __popcll(Fm & lanemask_lt());
            const int32_t lbv = __shfl(l, (2 * r) * G & 63), ubv = __shfl(l, (2 * r + 1) * G & 63);
            if (first) { lb = lbv; ub = ubv; }
        } else if (first) {
            int32_t l = lb_lo, h = lb_hi;
            while (l < h) {
                int32_t mid = l + ((h - l) >> 1);
                SD_CNT(8);
                if (text[(int64_t)sa[mid] + d] < tok) l = mid + 1; else h = mid;
            }
            lb = l;
            l = ub_lo; h = ub_hi;
            while (l < h) {
                int32_t mid = l + ((h - l) >> 1);
                SD_CNT(8);
                if (text[(int64_t)sa[mid] + d] <= tok) l = mid + 1; else h = mid;
            }
            ub = l;
        }
        double sc = ps * ((double)(ub - lb) / den);
        bool cand = first && sc >= min_score;
        frontier_put(f, -1, cand, sc, tok, parent, lb, ub, d + 1);
    }
}

// Tied single-occurrence chains.  When every frontier entry that shares the top score is a
// node with one occurrence (at most TIE_MAX of them, all staged), each of them heads a chain
// whose nodes all keep that score (count ratio 1/1), while everything else in the frontier
// scores strictly lower.  The greedy rule therefore keeps taking the head with the lowest
// (token, parent) among these chains until they end or K is reached: a merge that needs no
// frontier traffic.  Returns false (and changes nothing) if the frontier does not have that form.
//
// Few chains are merged as whole sequences, one after the other (taking the best head among k
// chains equals merging them pairwise, because (token, parent) keys are distinct).  Merging a
// chain X into the sequence Y merged so far under "take the head with the lower (token,
// parent)": element x_t leaves after exactly r(t) elements of Y, where r(t) is the first
// j >= r(t-1) at which y_j does not beat x_t.  y_j beats x_t if its token is lower, or equal
// with the lower parent index; parents are the predecessors within a chain, x_t's is x_(t-1),
// which left after r(t-1) elements of Y, so on equal tokens y_j wins iff its predecessor's
// place in Y is below r(t-1) (the given parents of chain heads are older than every new node
// and decide among themselves).  Three ballots per x_t give {j : y_j < x_t}, {j : y_j == x_t}
// and the predecessors below r(t-1) as lane masks, and r(t) follows with a few scalar bit
// operations.  The loop runs over the elements of the chain that is added, never over the
// sequence merged so far (which is as long as all chains before together: with the roles the
// other way round the third chain of a merge cost as much as the rest of the expansion).
// x_t lands at t + r(t); the elements of Y fill the positions left over, in order.  At most 63
// nodes are taken per call (one 64-token window per chain: its head plus 63 tokens), the caller
// comes back for more.  Per-chain state lives in the lanes of vector registers (lane q: chain q).
constexpr int TIE_MAX = 64;
// From this many chains on the merge goes step by step over all chains at once (below); fewer
// chains are merged as whole sequences.  4 measured best on the synthetic workloads (2, 3, 8, 16 tried).
constexpr int KWAY_MIN = 4;

// total + s + s + ... (n times), added one by one in that order like the sequential sum of node
// scores it stands for
__device__ __forceinline__ double add_times(double total, double s, int n) {
    int i = 0;
    for (; i + 8 <= n; i += 8) {
        total += s; total += s; total += s; total += s;
        total += s; total += s; total += s; total += s;
    }
    for (; i < n; i++) total += s;
    return total;
}

__device__ __forceinline__ uint64_t ballot64(bool pred) { return __builtin_amdgcn_ballot_w64(pred); }
// v with lane `idx` replaced by the uniform value `val`
__device__ __forceinline__ int32_t set_lane(int32_t val, int idx, int32_t v) {
    return (int)(threadIdx.x & 63) == idx ? val : v;
}

template <bool STATS>
__device__ __forceinline__ bool tied_chains(Frontier &f, Stage &sg, const int32_t *__restrict__ text, double s,
                            int K, int D, int &n, double &total, int32_t *t_tok, int32_t *t_par,
                            double *t_score, bool &deepest, unsigned &nb) {
    const int lane = threadIdx.x & 63;
    if (f.n > 64) return false;
    const bool have = lane < f.n;
    const bool tie = have && f.score[lane] == s;
    const int32_t mylo = have ? f.lo[lane] : 0, myhi = have ? f.hi[lane] : 0;
    const bool fit = myhi - mylo == 1 && mylo >= sg.lo && mylo < sg.lo + sg.m;
    const uint64_t T = ballot64(tie);
    const int j = __popcll(T);
    // a single top entry is not a tie: the unary-run shortcut takes its whole chain at once
    if (j < 2 || j > TIE_MAX || ballot64(tie && !fit)) return false;
    int32_t *TT = sg.tmp, *MM = sg.tmp + 64;
    // chain q = the q-th tied entry in frontier order; its head moves into lane q
    const int32_t etok = have ? f.tok[lane] : 0, epar = have ? f.par[lane] : 0,
                  edep = have ? f.dep[lane] : 0;
    const double eks = have ? f.score[lane] : 0.0;
    if (tie) TT[__popcll(T & lanemask_lt())] = lane;
    wsync();
    const int srcl = lane < j ? TT[lane] : 0;
    const int32_t ctokv = __shfl(etok, srcl), cparv = __shfl(epar, srcl), cdepv = __shfl(edep, srcl),
                  cslotv = __shfl(mylo, srcl) - sg.lo;
    const int32_t cposv = lane < j ? sg.pos[cslotv] : 0;
    // Where the staged windows of all these suffixes reach from their heads down to depth D,
    // every token the merge can ask for is in LDS already and nothing is loaded.
    const int32_t ccbv = lane < j ? sg.cb[cslotv] : 0;
    const bool covered = !ballot64(lane < j && !(ccbv <= cdepv && ccbv + (1 << sg.wlog) >= D));
    // take the tied entries out of the frontier (the others keep their relative order)
    {
        const bool keep = have && !tie;
        const int dst = __popcll(ballot64(keep) & lanemask_lt());
        wsync();
        if (keep) {
            f.score[dst] = eks; f.tok[dst] = etok; f.par[dst] = epar; f.lo[dst] = mylo; f.hi[dst] = myhi;
            f.dep[dst] = edep;
        }
        f.n -= j;
        wsync();
    }
    const int n0 = uni(n), KK = uni(K);
    if (j >= KWAY_MIN) {
        // Many chains: one pass that takes the lowest head each step.  The heads sit
        // in the lanes with their rank among the heads (0 = lowest key); a step takes the
        // head of rank 0, moves every other rank up, and ranks the chain's next element among
        // the others with one ballot.  That element's parent is the node just taken, the
        // highest index so far, so on equal tokens every older head goes first: the ballot
        // needs tokens only.  The chains' upcoming tokens sit in LDS (the staging windows'
        // space, handed back afterwards), W per chain.
        int jp2 = 1;
        while (jp2 < j) jp2 <<= 1;
        const int wlog = 31 - __clz(TC_TOKENS / jp2), W = 1 << wlog;
        // Per chain (lane q < j): the head's token, parent and depth, its rank, and the tokens
        // of the next two elements.  Tokens compare as unsigned numbers, which puts the end
        // marker (-1) above every real token: a chain whose next element does not exist (end
        // of the text, or the depth bound) gets the marker as its head, which is how it dies;
        // lanes >= j start dead.  Dead heads rank behind all live ones.
        const uint32_t DEAD = 0xffffffffu;
        const bool chain = lane < j;
        uint32_t htok = chain ? (uint32_t)ctokv : DEAD;
        int32_t hpar = cparv, hdep = chain ? cdepv : 0;
        const int32_t pos0 = cposv + cdepv;  // text index of the token of the chain's element 1
        // (covered: the chain's staged window, whose token i stands at child index ccb + i)
        const int base = covered ? (chain ? (cslotv << sg.wlog) - ccbv : 0) : (chain ? lane : 0) << wlog;
        int32_t abase = 0;
        uint32_t nexttok = DEAD, n2 = DEAD, cand = DEAD;
        // token windows: W tokens per chain from the element after its head on
        // (`need` <= W tokens per chain are fetched, rounded up to a power of two; all loads in
        // flight together)
        auto fill = [&](int need) {
            if (covered) {  // tokens hdep, hdep + 1, ... of the staged window
                abase = base + 1;
                nexttok = chain ? (uint32_t)sg.tc[base + hdep] : DEAD;
                n2 = (uint32_t)sg.tc[abase + hdep];
                cand = hdep < D ? nexttok : DEAD;
                return;
            }
            wsync();
            int flog = 3;
            while ((1 << flog) < need) flog++;
            const int total = j << flog;  // <= TC_TOKENS
            const int32_t adv = hdep - cdepv;  // elements of the chain taken so far
            int32_t v[FILL_U];
#pragma unroll
            for (int u = 0; u < FILL_U; u++) {
                const int idx = u * 64 + lane, q = (idx >> flog) & 63;
                v[u] = 0;
                if (u * 64 < total) {
                    const int32_t pq = __shfl(pos0, q), aq = __shfl(adv, q);  // all lanes take part
                    if (idx < total) {
                        v[u] = text[(int64_t)pq + aq + (idx & ((1 << flog) - 1))];
                        SD_CNT(4);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < FILL_U; u++) {
                const int idx = u * 64 + lane;
                if (u * 64 < total && idx < total)
                    sg.tc[((idx >> flog) << wlog) + (idx & ((1 << flog) - 1))] = v[u];
            }
            wsync();
            abase = base + 1 - hdep;
            nexttok = chain ? (uint32_t)sg.tc[base] : DEAD;
            n2 = (uint32_t)sg.tc[base + 1];
            cand = hdep < D ? nexttok : DEAD;
        };
        int32_t rank = 1 << 20;
        if (chain) {
            rank = 0;
            for (int q = 0; q < j; q++) {
                const uint32_t kt = (uint32_t)__builtin_amdgcn_readlane(ctokv, q);
                const int32_t kp = __builtin_amdgcn_readlane(cparv, q);
                rank += (kt < htok || (kt == htok && kp < hpar)) ? 1 : 0;
            }
        }
        int nn = n0;
        double tot = total;
        bool done = false;
        // a chain moves by at most one element per step and looks two elements ahead
        const int burst = covered ? 64 : W - 2 < 64 ? W - 2 : 64;
        while (nn < KK && !done) {
            const int lim = KK - nn < burst ? KK - nn : burst;
            fill(lim + 2);
            int32_t otok = 0, opar = 0;  // lane k: the node taken in step k of this burst
            int k = 0;
            for (; k < lim; k++) {
                const uint64_t first = ballot64(rank == 0);
                if (!first) { done = true; break; }
                const int w = __ffsll((unsigned long long)first) - 1;
                const uint32_t wtok = (uint32_t)__builtin_amdgcn_readlane((int32_t)htok, w);
                if (wtok == DEAD) { done = true; break; }  // no chain left
                const int32_t wpar = __builtin_amdgcn_readlane(hpar, w);
                const uint32_t nt = (uint32_t)__builtin_amdgcn_readlane((int32_t)cand, w);
                otok = set_lane((int32_t)wtok, k, otok);
                opar = set_lane(wpar, k, opar);
                tot += s;
                // The new head's parent is the node just taken, the highest index so far: among
                // equal tokens every other head goes first.
                const bool me = lane == w;
                const bool older = !me && htok <= nt;
                const int nr = __popcll(ballot64(older));
                rank = me ? nr : rank - (older ? 1 : 0);
                htok = me ? nt : htok;
                hpar = me ? nn + k : hpar;
                hdep += me ? 1 : 0;
                nexttok = me ? n2 : nexttok;
                n2 = (uint32_t)sg.tc[abase + hdep];
                cand = hdep < D ? nexttok : DEAD;
            }
            if (lane < k) {
                t_tok[nn + lane] = otok; t_par[nn + lane] = opar; t_score[nn + lane] = s;
                SD_CNT(8);
            }
            nn += k;
        }
        // a head of depth D that was taken left its chain at depth D + 1
        if (ballot64(chain && hdep > D)) deepest = true;
        wsync();
        if (!covered) sg.cb[lane] = CB_NONE;  // the staged token windows were overwritten
        wsync();
        n = nn;
        total = tot;
        return true;
    }
    const int room = KK - n0 < 63 ? KK - n0 : 63;
    // chain q as a sequence: element 0 is the frontier entry, element k its k-th descendant
    // (the token at child index cdep + k - 1); `alen` = how many elements exist
    int32_t alenv = 0;
    int32_t zt, zm = lane, zprev = lane - 1, zinit;
    int lz;
    // lane l >= 1: the token of chain q's element l (child index cdep + l - 1), from the staged
    // window or from memory (the load for the next chain is issued before this one is used)
    int32_t wnext = 0;
    if (!covered)
        wnext = text[(int64_t)__builtin_amdgcn_readlane(cposv, 0) + __builtin_amdgcn_readlane(cdepv, 0) + lane];
    auto chain_tokens = [&](int q) -> int32_t {
        if (covered) {
            const int at = (__builtin_amdgcn_readlane(cslotv, q) << sg.wlog) +
                           __builtin_amdgcn_readlane(cdepv, q) - __builtin_amdgcn_readlane(ccbv, q);
            return sg.tc[at + (lane >= 1 ? lane - 1 : 0)];
        }
        const int32_t w = wnext;
        if (q + 1 < j)
            wnext = text[(int64_t)__builtin_amdgcn_readlane(cposv, q + 1) +
                         __builtin_amdgcn_readlane(cdepv, q + 1) + lane];
        return __shfl_up(w, 1);
    };
    {
        const int cd = __builtin_amdgcn_readlane(cdepv, 0);
        const int32_t up = chain_tokens(0);
        zt = lane == 0 ? __builtin_amdgcn_readlane(ctokv, 0) : up;
        const uint64_t bad = ballot64(lane >= 1 && (up < 0 || cd + lane - 1 >= D));
        const int a = bad ? __ffsll((unsigned long long)bad) - 1 : 64;
        alenv = set_lane(a, 0, alenv);
        lz = a < room ? a : room;
        zinit = __builtin_amdgcn_readlane(cparv, 0);
    }
    for (int q = 1; q < j; q++) {
        const int cd = __builtin_amdgcn_readlane(cdepv, q);
        const int32_t up = chain_tokens(q);
        const int32_t yt = lane == 0 ? __builtin_amdgcn_readlane(ctokv, q) : up;
        const uint64_t bad = ballot64(lane >= 1 && (up < 0 || cd + lane - 1 >= D));
        const int a = bad ? __ffsll((unsigned long long)bad) - 1 : 64;
        alenv = set_lane(a, q, alenv);
        const int ly = a < room ? a : room;
        const int32_t yinit = __builtin_amdgcn_readlane(cparv, q);
        // The loop goes over the new chain X (plain: x_t's predecessor is x_(t-1)), the
        // sequence merged so far is Y.  x_t lands at t + r(t) and r never decreases: once that
        // reaches `room` neither x_t nor anything after it is kept, and every y_j still
        // unplaced lands at j + t >= room as well.  Lanes the loop never reached keep myr = 64
        // (dropped).  Equal tokens: y_j wins iff its predecessor left before x_(t-1), which
        // left after r(t-1) elements of Y, i.e. iff that predecessor's place in Y is below
        // r(t-1) (a head's given parent is older than every new node); for x_0 the given
        // parents decide, and only heads of Y can win.
        const uint64_t zmask = lz >= 64 ? ~0ull : ((1ull << lz) - 1ull);
        const uint64_t tie0 = ballot64(zprev < 0 && zinit < yinit);
        int r = 0;
        int32_t myr = 64;
        for (int t = 0; t < ly && t + r < room; t++) {  // r < 63 inside the loop
            const int32_t xt = __builtin_amdgcn_readlane(yt, t);
            const uint64_t lt = ballot64(zt < xt), eq = ballot64(zt == xt);
            const uint64_t tie = t ? ballot64(zprev < r) : tie0;
            const uint64_t wins = (lt | (eq & tie)) & zmask;
            const uint64_t rest = ~(wins >> r);  // (never empty: wins has no bit from 63 on)
            r += __ffsll((unsigned long long)rest) - 1;
            myr = set_lane(r, t, myr);
        }
        wsync();
        MM[lane] = -1;
        wsync();
        if (lane < ly && lane + myr < 64) { TT[lane + myr] = yt; MM[lane + myr] = (q << 8) | lane; }
        wsync();
        const int32_t mt = TT[lane], mm = MM[lane];
        const bool hole = mm == -1;  // not taken by X: the holes take Y's elements in order
        const int h = __popcll(ballot64(hole) & lanemask_lt());
        const int32_t zv = __shfl(zt, h), zmv = __shfl(zm, h);
        zt = hole ? zv : mt;
        zm = hole ? zmv : mm;
        lz = lz + ly < room ? lz + ly : room;
        // predecessor links and given parents of the new sequence
        zprev = -1;
        for (int c = 0; c <= q; c++) {
            const bool mine = lane < lz && (zm >> 8) == c;
            const uint64_t mc = ballot64(mine);
            if (mine) {
                const uint64_t prev = mc & lanemask_lt();
                zprev = prev ? 63 - __clzll((unsigned long long)prev) : -1;
            }
        }
        zinit = __shfl(cparv, (zm >> 8) & 63);
        wsync();
    }
    const bool live = lane < lz;
    const int myc = zm >> 8;
    if (live) {
        t_tok[n0 + lane] = zt; t_par[n0 + lane] = zprev < 0 ? zinit : n0 + zprev; t_score[n0 + lane] = s;
        SD_CNT(8);
    }
    total = add_times(total, s, lz);
    const int nn = n0 + lz;
    // per chain: how many elements were taken and where the last of them went
    int32_t usedv = 0, lastv = 0;
    for (int q = 0; q < j; q++) {
        const uint64_t mq = ballot64(live && myc == q);
        usedv = set_lane((int)__popcll(mq), q, usedv);
        lastv = set_lane(mq ? 63 - (int)__clzll((unsigned long long)mq) : 0, q, lastv);
    }
    if (ballot64(lane < j && usedv > 0 && cdepv + usedv - 1 >= D)) deepest = true;
    n = nn;
    if (nn < KK) {  // chains that go on put their next element back into the frontier
        const bool goes_on = lane < j && usedv < alenv;
        int32_t ntok = ctokv;
        if (goes_on && usedv > 0) {
            ntok = text[(int64_t)cposv + cdepv + usedv - 1];
            SD_CNT(4);
        }
        const uint64_t A = ballot64(goes_on);
        if (goes_on) {
            const int d = f.n + __popcll(A & lanemask_lt());
            f.score[d] = s; f.tok[d] = ntok; f.par[d] = usedv > 0 ? n0 + lastv : cparv;
            f.lo[d] = sg.lo + cslotv; f.hi[d] = sg.lo + cslotv + 1; f.dep[d] = cdepv + usedv;
        }
        f.n += __popcll(A);
    }
    wsync();
    return true;
}

// MatchPattern on the global index, one pattern length at a time (the route taken when the
// context's last two tokens start too many suffixes for the list form).  The pattern's first
// token selects a bucket of the suffix array; the second token is located in the bucket's
// second-token column (sorted, read with coalesced loads: buckets up to SCAN_MAX entries are
// simply scanned, up to SAMPLED_MAX a sample of the column is read first); the few suffixes left
// are compared with the whole pattern lane-parallel, and a dependent chain of bucket -> column
// -> suffix array -> text is all there is, whatever p is.  More suffixes than that (frequent
// tokens, text repeated many times over) are narrowed by a multi-way search that compares
// several tokens per probe; so is a bucket too wide for the column's short routes, from the
// pattern's second token on.
constexpr int SCAN_MAX = 256;
constexpr int DIRECT_MAX = 8;  // up to this many suffixes are compared with the whole pattern at once
constexpr int LEVEL_TLOG = 2;  // tokens per level of the search over a long range: 2^LEVEL_TLOG

// [lo, hi): the suffixes (a range of the sorted suffix array) that agree with the pattern on its
// first `depth` tokens (lane k of wk: pattern token k, pl of them).  Narrows the range to the
// suffixes that also agree on the next T = 2^tlog <= 32 tokens, as far as the pattern goes.  Lower
// and upper end are searched side by side, one half of the wave per end: a round probes
// F = 32 / T suffixes per end, evenly spaced over the interval the end is known to lie in, T
// lanes per probe comparing one token each, and keeps the gap between two probes (an (F + 1)-ary
// search whose compares span T tokens).  The dependent chain is two loads per round (suffix
// array, text) and log_(F+1)(hi - lo) rounds, where narrowing token by token costs as many
// rounds again for every further token that a wide range needs.
template <bool STATS>
__device__ __forceinline__ void range_fan_tokens(const int32_t *__restrict__ sa,
                                                 const int32_t *__restrict__ text, int32_t wk, int pl,
                                                 int depth, int tlog, int32_t &lo, int32_t &hi,
                                                 unsigned &nb) {
    const int lane = threadIdx.x & 63, half = lane >> 5, k = lane & 31;
    const int T = 1 << tlog, F = 32 >> tlog, j = k >> tlog, tt = k & (T - 1);
    const uint32_t tmask = T >= 32 ? ~0u : (1u << T) - 1u;
    const int32_t w = __shfl(wk, (depth + tt) & 63);
    const bool tok_on = depth + tt < pl;
    // probe j of an interval of n places sits at floor(n * frac / 2^32) with frac about
    // 2^32 (j + 1) / (F + 1): increasing in j and below n, which is all the search needs (one
    // multiply, no 64-bit division: F + 1 is one of 2, 3, 5, 9, 17, 33)
    const uint32_t recip = tlog >= 5 ? 2147483648u : tlog == 4 ? 1431655765u : tlog == 3 ? 858993459u
                           : tlog == 2 ? 477218588u : tlog == 1 ? 252645135u : 130150524u;
    const uint32_t frac = recip * (uint32_t)(j + 1);
    int32_t l = lo, h = hi;  // the interval this lane's end lies in: [l, h]
    while (__ballot(l < h)) {
        const bool go = l < h;
        const uint32_t n = (uint32_t)(h - l);
        const int32_t pt = l + (int32_t)__umulhi(n, frac);
        int32_t v = w;
        if (go && tok_on) {
            v = text[(int64_t)sa[pt] + depth + tt];
            SD_CNT(tt == 0 ? 8 : 4);
        }
        // probe against pattern over the T tokens: the first token that differs decides
        const uint64_t ne = __ballot(v != w), lt = __ballot(v < w);
        const int sh = k & ~(T - 1);
        const uint32_t gne = ((uint32_t)(ne >> (half * 32)) >> sh) & tmask;
        const uint32_t glt = ((uint32_t)(lt >> (half * 32)) >> sh) & tmask;
        const int cmp = gne == 0 ? 0 : ((glt & (gne & (0u - gne))) ? -1 : 1);
        // the end is the first suffix that is not below (lower end) / above (upper end) the
        // pattern: the probes that say "further on" form a prefix
        const bool further = go && (half ? cmp <= 0 : cmp < 0);
        const uint64_t fm = __ballot(further && tt == 0);
        const int cfa = __popc((uint32_t)fm), cfb = __popc((uint32_t)(fm >> 32));
        const int cf = half ? cfb : cfa;
        // the end lies behind the last probe that says "further on" and at or before the next
        // one: their places are read from the lanes that made them (scalar lane indices)
        const int32_t la_ = __builtin_amdgcn_readlane(pt, (cfa > 0 ? cfa - 1 : 0) << tlog);
        const int32_t na_ = __builtin_amdgcn_readlane(pt, (cfa < F ? cfa : 0) << tlog);
        const int32_t lb_ = __builtin_amdgcn_readlane(pt, 32 + ((cfb > 0 ? cfb - 1 : 0) << tlog));
        const int32_t nb_ = __builtin_amdgcn_readlane(pt, 32 + ((cfb < F ? cfb : 0) << tlog));
        const int32_t nl = cf > 0 ? (half ? lb_ : la_) + 1 : l;
        const int32_t nh = cf < F ? (half ? nb_ : na_) : h;
        if (go) { l = nl; h = nh; }
    }
    lo = __builtin_amdgcn_readlane(l, 0);
    hi = __builtin_amdgcn_readlane(l, 32);
}

// Result of an out-of-line second-stage lookup for two patterns.
struct WideOut {
    int32_t loA, hiA, loB, hiB;
    unsigned nb;  // bytes asked for (counting variant)
};

// Second stage for buckets of up to SAMPLED_MAX entries through the sampled column (every 16th
// entry of the column): the bucket's samples are read and counted, which confines each end of
// the range to the fifteen entries between two samples (or between an end of the bucket and
// the nearest sample); those two blocks are read next, a quarter of the wave per block (lower
// and upper end of A, lower and upper end of B).  Two memory rounds and a few lines per pattern;
// reading such a bucket whole in one round moved eight times the bytes and was slower on the
// 100M-token corpus, whose buckets are of this size (the step is traffic-bound there).
// (Not inlined: the route is taken by workloads with buckets of that size only, and kept out
// of line it costs the others neither registers nor instruction-cache room.)
constexpr int SAMP_C = 4;                     // sample loads per lane and pattern
constexpr int SAMPLED_MAX = 64 * SAMP_C * 16;  // widest bucket whose samples one such round covers
template <bool STATS>
__device__ __attribute__((noinline)) WideOut col_sampled(const int32_t *__restrict__ col,
                                                          const int32_t *__restrict__ samples,
                                                          bool doA, int32_t w1A, int32_t loA,
                                                          int32_t hiA, bool doB, int32_t w1B,
                                                          int32_t loB, int32_t hiB) {
    unsigned nb = 0;
    const int lane = threadIdx.x & 63;
    // samples inside a bucket [lo, hi): indices (lo + 15) / 16 .. (hi - 1) / 16
    const int32_t j0A = (loA + 15) >> 4, j1A = (hiA - 1) >> 4;
    const int32_t j0B = (loB + 15) >> 4, j1B = (hiB - 1) >> 4;
    int32_t vA[SAMP_C], vB[SAMP_C];
#pragma unroll
    for (int c = 0; c < SAMP_C; c++) {
        const int32_t jA = j0A + c * 64 + lane, jB = j0B + c * 64 + lane;
        vA[c] = doA && jA <= j1A ? samples[jA] : 0x7fffffff;
        vB[c] = doB && jB <= j1B ? samples[jB] : 0x7fffffff;
        if (doA && jA <= j1A) SD_CNT(4);
        if (doB && jB <= j1B) SD_CNT(4);
    }
    int32_t cA = 0, cB = 0;  // samples below the token (low half) and not above it (high half)
#pragma unroll
    for (int c = 0; c < SAMP_C; c++) {
        cA += (vA[c] < w1A ? 1 : 0) + (vA[c] <= w1A ? 0x10000 : 0);
        cB += (vB[c] < w1B ? 1 : 0) + (vB[c] <= w1B ? 0x10000 : 0);
    }
    const int32_t sA = __builtin_amdgcn_readlane(wave_inclusive_sum(cA), 63);
    const int32_t sB = __builtin_amdgcn_readlane(wave_inclusive_sum(cB), 63);
    // With c samples below (not above) the token, the lower (upper) end of the range lies
    // behind sample c - 1 and at or before sample c: in the block of entries between them, or
    // between the bucket's start and its first sample, or its last sample and its end.
    const int quarter = lane >> 4, k = lane & 15;
    const bool isB = quarter >= 2, upper = quarter & 1;
    const int32_t lo_ = isB ? loB : loA, hi_ = isB ? hiB : hiA, j0 = isB ? j0B : j0A;
    const int32_t w1 = isB ? w1B : w1A, sc = isB ? sB : sA;
    const int32_t cnt = upper ? sc >> 16 : sc & 0xffff;
    const int32_t base = cnt == 0 ? lo_ : ((j0 + cnt - 1) << 4) + 1;
    int32_t end = (j0 + cnt) << 4;
    if (end > hi_) end = hi_;
    const bool act = (isB ? doB : doA) && base + k < end;
    const int32_t v = act ? col[base + k] : 0x7fffffff;
    if (act) SD_CNT(4);
    const uint64_t bm = __ballot(act && (upper ? v <= w1 : v < w1));
    const int32_t found = base + __popc((uint32_t)(bm >> (quarter * 16)) & 0xffffu);
    const int32_t nlA = __builtin_amdgcn_readlane(found, 0), nhA = __builtin_amdgcn_readlane(found, 16);
    const int32_t nlB = __builtin_amdgcn_readlane(found, 32), nhB = __builtin_amdgcn_readlane(found, 48);
    if (doA) { loA = nlA; hiA = nhA; }
    if (doB) { loB = nlB; hiB = nhB; }
    return WideOut{loA, hiA, loB, hiB, nb};
}

// last stage for one pattern: [lo, hi) holds the suffixes that start with its first `depth` tokens
template <bool STATS>
__device__ __forceinline__ void match_rest(const SpecParams &p, int32_t wk, int pl, int32_t &lo,
                                           int32_t &hi, int depth, unsigned &nb) {
    const int lane = threadIdx.x & 63;
    // A long range is narrowed by the pattern's next four tokens at a time, which usually
    // shrinks it by orders of magnitude.  When a level hardly shrank it (many suffixes that
    // share the whole pattern: text copied from one template), the next level takes all the
    // tokens that are left, up to 32 per probe.  Once at most DIRECT_MAX suffixes remain they
    // are compared with the whole pattern in one go.
    int tlog = LEVEL_TLOG;
    while (hi - lo > DIRECT_MAX && depth < pl) {
        const int32_t before = hi - lo;
        range_fan_tokens<STATS>(p.g_sa, p.g_text, wk, pl, depth, tlog, lo, hi, nb);
        depth += 1 << tlog;
        if ((int64_t)(hi - lo) * 4 > before)
            while (tlog < 5 && (1 << tlog) < pl - depth) tlog++;
    }
    if (lo >= hi || depth >= pl) return;
    {  // compare every remaining suffix with the whole pattern
        const int32_t cnt = hi - lo;
        const int64_t pos = lane < cnt ? p.g_sa[lo + lane] : 0;
        if (lane < cnt) SD_CNT(4);
        int32_t tk[DIRECT_MAX];
#pragma unroll
        for (int c = 0; c < DIRECT_MAX; c++) {
            const int64_t pc = __shfl(pos, c);
            tk[c] = (c < cnt && lane < pl) ? p.g_text[pc + lane] : wk;
            if (c < cnt && lane < pl) SD_CNT(4);
        }
        int nless = 0, nleq = 0;
#pragma unroll
        for (int c = 0; c < DIRECT_MAX; c++) {
            const uint64_t ne = __ballot(c < cnt && lane < pl && tk[c] != wk);
            int r = 0;
            if (ne) {
                int fl = __ffsll((unsigned long long)ne) - 1;
                r = __shfl(tk[c], fl) < __shfl(wk, fl) ? -1 : 1;
            }
            if (c < cnt) {
                nless += r < 0;
                nleq += r <= 0;
            }
        }
        hi = lo + nleq;
        lo = lo + nless;
    }
}

template <bool STATS>
__device__ __forceinline__ void col_stage(const SpecParams &p, int32_t w1, int32_t &lo, int32_t &hi,
                                          unsigned &nb);

template <bool STATS>
__device__ __forceinline__ void match_global(const SpecParams &p, int32_t wk, int pl, int32_t &lo, int32_t &hi,
                             unsigned &nb) {
    const int lane = threadIdx.x & 63;
    const int32_t w0 = __builtin_amdgcn_readlane(wk, 0);
    const int32_t bv = lane < 2 ? p.g_bucket[w0 + 1 + lane] : 0;
    if (lane < 2) SD_CNT(4);
    lo = __builtin_amdgcn_readlane(bv, 0);
    hi = __builtin_amdgcn_readlane(bv, 1);
    if (pl == 1 || lo >= hi) return;
    // (a bucket too wide for the second-token column's short routes is searched with several
    // tokens per probe from the start)
    const bool wide = hi - lo > SAMPLED_MAX;
    if (!wide) {
        const int32_t w1 = __builtin_amdgcn_readlane(wk, 1);
        col_stage<STATS>(p, w1, lo, hi, nb);
    }
    if (wide || pl > 2) match_rest<STATS>(p, wk, pl, lo, hi, wide ? 1 : 2, nb);
}

// Second stage for one pattern: narrows the first token's bucket [lo, hi) to the suffixes whose
// second token is w1, by the route that fits the bucket's size.
template <bool STATS>
__device__ __forceinline__ void col_stage(const SpecParams &p, int32_t w1, int32_t &lo, int32_t &hi,
                                          unsigned &nb) {
    const int lane = threadIdx.x & 63;
    const int32_t *col = p.g_tok1;
    int32_t l = lo, h = hi;
    if (h - l > SCAN_MAX && h - l <= SAMPLED_MAX) {
        const WideOut r = col_sampled<STATS>(col, p.g_tok1s, true, w1, l, h, false, 0, 0, 0);
        l = r.loA; h = r.hiA;
        SD_CNT(r.nb);
    } else if (h - l > SCAN_MAX) {  // (callers send such buckets elsewhere; kept for completeness)
        range_fan_tokens<STATS>(p.g_sa, p.g_text, w1, 2, 1, LEVEL_TLOG, l, h, nb);
    } else {
        int32_t v[SCAN_MAX / 64];
#pragma unroll
        for (int c = 0; c < SCAN_MAX / 64; c++) {
            int32_t i = l + c * 64 + lane;
            v[c] = i < h ? col[i] : 0x7fffffff;
            if (i < h) SD_CNT(4);
        }
        int nless = 0, nleq = 0;
#pragma unroll
        for (int c = 0; c < SCAN_MAX / 64; c++) {
            nless += __popcll(__ballot(v[c] < w1));
            nleq += __popcll(__ballot(v[c] <= w1));
        }
        h = l + nleq;
        l = l + nless;
    }
    lo = l;
    hi = h;
}

// Two patterns of one context at once (pattern lengths plA, plB <= 32; lane k of wkA / wkB holds
// pattern token k).  The stages of the two searches are issued side by side, so that the wave
// waits for memory once per stage instead of once per stage and pattern: both bucket reads in
// one load, both column scans together, and the final compare with one half of the wave per
// pattern.  A pattern that leaves the common route (wide bucket, more than DIRECT_MAX
// candidates) finishes on its own with the single-pattern stages.
template <bool STATS>
__device__ __forceinline__ void match_global_pair(const SpecParams &p, int32_t wkA, int plA, int32_t wkB,
                                                  int plB, int32_t &loA, int32_t &hiA, int32_t &loB,
                                                  int32_t &hiB, unsigned &nb) {
    const int lane = threadIdx.x & 63, half = lane >> 5, k = lane & 31;
    const int32_t w0A = __builtin_amdgcn_readlane(wkA, 0), w0B = __builtin_amdgcn_readlane(wkB, 0);
    const int32_t bv = lane < 4 ? p.g_bucket[(lane < 2 ? w0A : w0B) + 1 + (lane & 1)] : 0;
    if (lane < 4) SD_CNT(4);
    loA = __builtin_amdgcn_readlane(bv, 0); hiA = __builtin_amdgcn_readlane(bv, 1);
    loB = __builtin_amdgcn_readlane(bv, 2); hiB = __builtin_amdgcn_readlane(bv, 3);
    const bool goA = plA > 1 && loA < hiA, goB = plB > 1 && loB < hiB;  // second stage needed
    const int32_t w1A = __builtin_amdgcn_readlane(wkA, 1), w1B = __builtin_amdgcn_readlane(wkB, 1);
    const int32_t *col = p.g_tok1;
    const bool narrowA = goA && hiA - loA <= SCAN_MAX, narrowB = goB && hiB - loB <= SCAN_MAX;
    {
        int32_t vA[SCAN_MAX / 64], vB[SCAN_MAX / 64];
#pragma unroll
        for (int c = 0; c < SCAN_MAX / 64; c++) {
            const int32_t iA = loA + c * 64 + lane, iB = loB + c * 64 + lane;
            vA[c] = narrowA && iA < hiA ? col[iA] : 0x7fffffff;
            vB[c] = narrowB && iB < hiB ? col[iB] : 0x7fffffff;
            if (narrowA && iA < hiA) SD_CNT(4);
            if (narrowB && iB < hiB) SD_CNT(4);
        }
        int lsA = 0, leA = 0, lsB = 0, leB = 0;
#pragma unroll
        for (int c = 0; c < SCAN_MAX / 64; c++) {
            lsA += __popcll(__ballot(vA[c] < w1A)); leA += __popcll(__ballot(vA[c] <= w1A));
            lsB += __popcll(__ballot(vB[c] < w1B)); leB += __popcll(__ballot(vB[c] <= w1B));
        }
        if (narrowA) { hiA = loA + leA; loA = loA + lsA; }
        if (narrowB) { hiB = loB + leB; loB = loB + lsB; }
    }
    const bool smpA = goA && !narrowA && hiA - loA <= SAMPLED_MAX;
    const bool smpB = goB && !narrowB && hiB - loB <= SAMPLED_MAX;
    if (smpA || smpB) {
        const WideOut r = col_sampled<STATS>(col, p.g_tok1s, smpA, w1A, loA, hiA, smpB, w1B, loB, hiB);
        loA = r.loA; hiA = r.hiA; loB = r.loB; hiB = r.hiB;
        SD_CNT(r.nb);
    }
    // (a wider bucket goes to the search with several tokens per probe, from its second token on)
    const bool wideA = goA && !narrowA && !smpA, wideB = goB && !narrowB && !smpB;
    // last stage: compare the few suffixes left with the whole pattern, A in the lower half of
    // the wave and B in the upper half
    const bool restA = goA && (plA > 2 || wideA) && loA < hiA, restB = goB && (plB > 2 || wideB) && loB < hiB;
    const bool dirA = restA && hiA - loA <= DIRECT_MAX, dirB = restB && hiB - loB <= DIRECT_MAX;
    if (dirA || dirB) {
        const int32_t cntA = dirA ? hiA - loA : 0, cntB = dirB ? hiB - loB : 0;
        const int32_t cnt = half ? cntB : cntA, plh = half ? plB : plA;
        const int64_t pos = k < cnt ? p.g_sa[(half ? loB : loA) + k] : 0;  // lane 32 h + c: suffix c
        if (k < cnt) SD_CNT(4);
        // pattern token k of this half's pattern (the shuffle runs with all lanes on: a lane
        // that is switched off would hand out zero)
        const int32_t wkBk = __shfl(wkB, k);
        const int32_t wkh = half ? wkBk : wkA;
        int32_t tk[DIRECT_MAX];
#pragma unroll
        for (int c = 0; c < DIRECT_MAX; c++) {
            const int64_t pc = __shfl(pos, half * 32 + c);
            tk[c] = (c < cnt && k < plh) ? p.g_text[pc + k] : wkh;
            if (c < cnt && k < plh) SD_CNT(4);
        }
        int lsA = 0, leA = 0, lsB = 0, leB = 0;
#pragma unroll
        for (int c = 0; c < DIRECT_MAX; c++) {
            const uint64_t ne = __ballot(c < cnt && k < plh && tk[c] != wkh);
            const uint32_t neA = (uint32_t)ne, neB = (uint32_t)(ne >> 32);
            int rA = 0, rB = 0;
            if (neA) {
                const int fl = __ffs(neA) - 1;
                rA = __shfl(tk[c], fl) < __shfl(wkh, fl) ? -1 : 1;
            }
            if (neB) {
                const int fl = 32 + __ffs(neB) - 1;
                rB = __shfl(tk[c], fl) < __shfl(wkh, fl) ? -1 : 1;
            }
            if (c < cntA) { lsA += rA < 0; leA += rA <= 0; }
            if (c < cntB) { lsB += rB < 0; leB += rB <= 0; }
        }
        if (dirA) { hiA = loA + leA; loA = loA + lsA; }
        if (dirB) { hiB = loB + leB; loB = loB + lsB; }
    }
    if (restA && !dirA) match_rest<STATS>(p, wkA, plA, loA, hiA, wideA ? 1 : 2, nb);
    if (restB && !dirB) match_rest<STATS>(p, wkB, plB, loB, hiB, wideB ? 1 : 2, nb);
}

// One unit (request b, index src: 0 global / 1 request, pattern length pl) on one wavefront:
// ExpandSpeculationTree below the matched node into the LDS tree (t_tok, t_par, t_score).
// Returns the number of draft nodes and leaves their SCORE in `total`; `deepest` tells whether
// a node of depth D (which may have no children) was taken.
template <bool STATS, bool TICKS>
__device__ __forceinline__ int run_unit(const SpecParams &p, const WgShared &sh, int b, int t,
                        const int32_t *__restrict__ x, int src, int pl, int usa_off, Frontier &f, Stage &sg,
                        int32_t *t_tok, int32_t *t_par, double *t_score, double &total,
                        bool &deepest, unsigned &nb) {
    const int lane = threadIdx.x & 63;
    deepest = false;
    const uint64_t tick0 = TICKS ? wall_clock64() : 0;
    const int64_t uidx = (int64_t)b * (2 * p.P) + src * p.P + (pl - 1);
    const int K = (int)floor(p.alpha * (double)pl);
    uint32_t tick_setup = 0, tick_match = 0, tick_root = 0;
    sg.lo = 0; sg.m = 0; sg.wlog = 0;

    const int32_t *sa = nullptr, *text = nullptr;
    int32_t lo = 0, hi = 0;
    if (pl <= t && K >= 1) {
        if (src == 0 && pl >= 2 && uni(sh.g_mode) != 0) {
            // list form: the listed suffixes that match at least pl tokens, in their order
            // (the suffix array's, i.e. sorted by what follows the pattern), staged whole
            const int n2 = uni(sh.g_n2);
            const bool keep = lane < n2 && sh.gl_L[lane] >= pl;
            const uint64_t mk = __ballot(keep);
            const int m = __popcll(mk);
            if (keep) {
                const int dst = __popcll(mk & lanemask_lt());
                sg.pos[dst] = sh.gl_pos[lane] - (pl - 2);
                sg.cb[dst] = CB_NONE;
            }
            sg.lo = 0;
            sg.m = m;
            stage_set_width(sg, m > 0 ? m : 1);
            __threadfence_block();
            wsync();
            sa = p.g_sa;  // never read: the whole list is staged
            text = p.g_text;
            lo = 0;
            hi = m;
        } else if (src == 0) {  // matched by the whole workgroup beforehand
            sa = p.g_sa;
            text = p.g_text;
            lo = uni(sh.g_lo[pl]);
            hi = uni(sh.g_hi[pl]);
        } else {
            // per-request structure: occurrences whose left-extension reaches pl, in the
            // order request_occurrences left them (sorted by what follows)
            const int m = uni(sh.cnt[pl]);
            // m == 1 is the context's own tail alone: it stops at the end marker, so the
            // unit has no candidate at all and nothing else needs to be read
            const int m1 = m > 1 ? uni(sh.m) : 0;
            const uint32_t *occ = p.occ + (int64_t)b * p.max_ctx;
            // a list of more than 64 occurrences goes to the request's row of scratch memory,
            // at the place the caller has assigned to this run of pattern lengths
            int32_t *usa = p.unit_sa + (int64_t)b * p.max_ctx + usa_off;
            const bool narrow = m <= 64;
            int w = 0;
            for (int base = 0; base < m1; base += 64) {
                int i = base + lane;
                int2 o = make_int2(0, 0);
                if (i < m1) o = occ_unpack(occ[i]);
                if (i < m1) SD_CNT(4);
                bool keep = i < m1 && o.y >= pl;
                uint64_t mk = __ballot(keep);
                if (keep) {
                    int dst = w + __popcll(mk & lanemask_lt());
                    if (narrow) { sg.pos[dst] = o.x - pl + 1; sg.cb[dst] = CB_NONE; }
                    else usa[dst] = o.x - pl + 1;
                    SD_CNT(4);
                }
                w += __popcll(mk);
            }
            if (narrow) {  // the whole list is staged: nothing below it ever reads `usa`
                sg.lo = 0;
                sg.m = m;
                stage_set_width(sg, m > 0 ? m : 1);
            }
            __threadfence_block();
            wsync();
            lo = 0;
            hi = m > 1 ? m : 0;  // == w when the list was gathered
            sa = usa;
            text = x;
        }
    }

    int n = 0;
    total = 0.0;
    if (TICKS) tick_match = (uint32_t)(wall_clock64() - tick0) + (uint32_t)((hi - lo) & 0);
    if (hi > lo) {
        f.n = 0;
        f.cap = K;
        // Unary run below the node [blo, blo + m) of depth d, whose score is sc and whose place
        // in the tree is cur (-1: the matched node itself): while all suffixes of the node agree
        // on the next token and none has ended, the node has exactly one child, with the node's
        // own score (count ratio 1).  Where nothing else in the frontier shares that score the
        // greedy rule must take that child next, and so on down the run: the run is taken at
        // once.
        auto unary_run = [&](int32_t blo, int32_t m, int32_t &d, int &cur, double sc) {
            const int32_t mycb = stage_node(sg, sa, text, blo, m, d);
            const int slot0 = blo - sg.lo, W = 1 << sg.wlog;
            const int32_t tk = m <= CHAIN_MAX_M / 2
                                   ? common_token<CHAIN_MAX_M / 2>(sg, slot0, m, d, W, mycb)
                                   : common_token<CHAIN_MAX_M>(sg, slot0, m, d, W, mycb);
            int lim = K - n < p.D - d ? K - n : p.D - d;
            uint64_t ok = __ballot(tk >= 0 && lane < lim);
            int L = ~ok ? __ffsll((unsigned long long)~ok) - 1 : 64;
            if (L > 0) {
                if (lane < L) {
                    t_tok[n + lane] = tk; t_par[n + lane] = cur + lane;
                    t_score[n + lane] = sc;
                    SD_CNT(8 * m);
                }
                total = add_times(total, sc, L);
                cur += L;
                n += L;
                d += L;
                if (d >= p.D) deepest = true;
            }
        };
        // The matched node first: a narrow one whose suffixes all go on alike (the usual case: a
        // pattern seen once or a few times) has one child of score 1, which is taken with its
        // run without going through the frontier.
        {
            int32_t d = pl;
            int cur = -1;
            if (d < p.D && hi - lo <= CHAIN_MAX_M) unary_run(lo, hi - lo, d, cur, 1.0);
            if (n < K)
                push_children<STATS>(f, -1, sg, sa, text, lo, hi, d, cur, 1.0, p.min_score, p.D,
                                     p.den_mode, nb);
        }
        if (TICKS) tick_root = (uint32_t)(wall_clock64() - tick0) + (uint32_t)(f.n & 0);
        while (n < K && f.n > 0) {
            const Taken tk0 = frontier_take(f);
            const Key best = tk0.k;
            if (best.s < p.min_score) break;
            // Nodes are taken in non-increasing score order, so the K - n nodes still to come
            // add at most that many times the best score left: a tree that cannot reach the
            // best finished SCORE any more is given up (it could neither win nor tie; nor could
            // the shorter patterns of its run, whose trees are its first nodes).  The SCORE is a
            // sum of rounded additions, which may come out a few units in the last place above
            // this product form (and two trees of equal nodes must tie exactly): hence the
            // margin.  Checked once per step here; checks inside the merges of tied chains
            // cost more than they saved.
            {
                const double top = uni(__longlong_as_double((long long)sh.top_bits));
                if ((total + (double)(K - n) * best.s) * (1.0 + 1e-9) < top) {
                    n = 0;
                    total = 0.0;
                    break;
                }
            }
            const int ntop = tk0.ntop;
            if (ntop >= 2 && !p.linear) {
                const uint64_t m0 = TICKS ? wall_clock64() : 0;
                const bool merged = tied_chains<STATS>(f, sg, text, best.s, K, p.D, n, total, t_tok,
                                                       t_par, t_score, deepest, nb);
                if (TICKS) tick_setup += (uint32_t)(wall_clock64() - m0);  // time spent merging
                if (merged) continue;
            }
            const int bi = best.idx;
            const int32_t blo = tk0.lo, bhi = tk0.hi;
            int32_t d = tk0.dep;
            if (d >= p.D) deepest = true;
            if (lane == 0) {
                t_tok[n] = best.tok; t_par[n] = best.par; t_score[n] = best.s;
            }
            total += best.s;
            int cur = n++;
            int hole = bi;
            if (p.linear) {  // chain variant: nothing but the new node's children may follow
                f.n = 0;
                hole = -1;
            }
            // (the unary run below the node, if no other entry shares the top score)
            const int32_t m = bhi - blo;
            if (n < K && d < p.D && m <= CHAIN_MAX_M && (ntop == 1 || p.linear))
                unary_run(blo, m, d, cur, best.s);
            if (n < K)
                push_children<STATS>(f, hole, sg, sa, text, blo, bhi, d, cur, best.s, p.min_score,
                                     p.D, p.den_mode, nb);
            else
                frontier_close(f, hole);  // the last node taken cannot contribute further nodes
        }
    }
    wsync();
    if (TICKS && lane == 0) {  // time spent merging tied chains; marks: match, root children, whole unit
        p.unit_ticks[uidx * 4 + 0] = tick_setup;
        p.unit_ticks[uidx * 4 + 1] = tick_match;
        p.unit_ticks[uidx * 4 + 2] = tick_root;
        p.unit_ticks[uidx * 4 + 3] = (uint32_t)(wall_clock64() - tick0);
    }
    return n;
}

struct AppendArgs {
    const int32_t *slot_ids;
    int32_t *r_text, *r_len;
    int64_t stride;
    int32_t max_ctx, max_slots, vocab;
    int32_t *err;
};

// What sd_accept hands back besides the trees it reads.
struct AcceptArgs {
    const int32_t *target;
    int32_t *accept_len, *accept_path, *bonus;
    unsigned long long *counters;  // what sd_get_stats reports (SD_CTR_*)
};

// Acceptance for request b on one wavefront (max_nodes <= 256): node j is accepted iff its
// token equals the target token at its parent's position and its parent is accepted, which
// pointer jumping over the parent links settles in at most eight rounds (trees of up to 64
// nodes: one node per lane, links and flags in registers; larger ones in LDS).  s_tgt[257],
// s_anc[256] and s_ok[256] are LDS of the calling wave.  With APPEND the accepted tokens and the bonus
// token go behind the slot's context (and into s_new in LDS if that is given).  Returns the
// slot's context length afterwards (0 for a bad slot), which only the APPEND form looks up.
// What the acceptance reads first, for lane l: the node count, node l and target position l
// (and position 64, which a tree of 64 nodes has), and the request's two counters.  Kept apart
// from accept_wave so that a caller with other loads to wait for can issue these first.
struct AcceptIn {
    int32_t n, tok0, par0, tgt0, tgt64;
    unsigned long long c_req, c_len;
};

__device__ __forceinline__ AcceptIn accept_fetch(int b, const int32_t *__restrict__ n_nodes,
                                                 const int32_t *__restrict__ tokens,
                                                 const int32_t *__restrict__ parents, int max_nodes,
                                                 const AcceptArgs &aa) {
    const int lane = threadIdx.x & 63;
    const int32_t *tgt = aa.target + (int64_t)b * (max_nodes + 1);
    AcceptIn in;
    in.n = n_nodes[b];
    in.tok0 = lane < max_nodes ? tokens[(int64_t)b * max_nodes + lane] : -1;
    in.par0 = lane < max_nodes ? parents[(int64_t)b * max_nodes + lane] : -1;
    in.tgt0 = lane <= max_nodes ? tgt[lane] : 0;
    in.tgt64 = max_nodes >= 64 ? tgt[64] : 0;
    // this request's counters of verified requests and accepted nodes (see sd_internal.h)
    const unsigned long long *ctr = aa.counters + (int64_t)b * SD_CTR_STRIDE;
    in.c_req = 0; in.c_len = 0;
    if (lane == 0) { in.c_req = ctr[SD_CTR_ACCEPT_REQUESTS]; in.c_len = ctr[SD_CTR_ACCEPT_LEN]; }
    return in;
}

template <bool APPEND>
__device__ __forceinline__ int accept_wave(int b, const AcceptIn &in,
                                           const int32_t *__restrict__ tokens,
                                           const int32_t *__restrict__ parents, int max_nodes,
                                           const AcceptArgs &aa, const AppendArgs &ap, int32_t *s_tgt,
                                           int32_t *s_anc, int32_t *s_ok, int32_t *s_new,
                                           int32_t known_slot = -2, int32_t known_len = 0) {
    const int lane = threadIdx.x & 63;
    const int32_t *tok = tokens + (int64_t)b * max_nodes, *par = parents + (int64_t)b * max_nodes;
    const int32_t *tgt = aa.target + (int64_t)b * (max_nodes + 1);
    int32_t *path = aa.accept_path + (int64_t)b * max_nodes;
    int n = in.n;
    unsigned long long *ctr = aa.counters + (int64_t)b * SD_CTR_STRIDE;
    const unsigned long long c_req = in.c_req, c_len = in.c_len;
    const bool small = max_nodes <= 64;  // one node per lane: settled in registers, below
    int32_t mt[4], mp[4];
    mt[0] = in.tok0; mp[0] = in.par0;
#pragma unroll
    for (int r = 1; r < 4; r++) {
        int j = lane + 64 * r;
        mt[r] = j < max_nodes ? tok[j] : -1;
        mp[r] = j < max_nodes ? par[j] : -1;
    }
    if (!small) {
        s_tgt[lane] = in.tgt0;
        for (int i = 64 + lane; i <= max_nodes; i += 64) s_tgt[i] = tgt[i];
    }
    if (n > max_nodes) n = max_nodes;
    if (n < 0) n = 0;
#pragma unroll
    for (int r = 0; r < 4; r++)
        if (lane + 64 * r >= n) { mt[r] = -1; mp[r] = -1; }
    uint64_t am[4] = {0ull, 0ull, 0ull, 0ull};
    int L = 0, last = -1;
    int32_t bon;
    if (small) {
        // the same pointer jumping with the links and flags in registers, passed between
        // lanes by permutes: no LDS round trip and no wave barrier per round
        const bool wf = lane < n && mp[0] >= -1 && mp[0] < lane;
        const int32_t want = __shfl(in.tgt0, wf ? mp[0] + 1 : 0);  // (mp[0] + 1 <= lane <= 63)
        int32_t ok = wf && mt[0] == want, anc = wf ? mp[0] : -1;
        for (int round = 0; round < 6; round++) {  // 2^6 >= the deepest possible path
            const bool open = anc >= 0;
            if (!__ballot(open)) break;
            const int src = open ? anc : lane;
            const int32_t o2 = __shfl(ok, src), a2 = __shfl(anc, src);
            if (open) { ok &= o2; anc = a2; }
        }
        am[0] = __ballot(lane < n && ok);
        if (am[0]) last = 63 - __clzll((unsigned long long)am[0]);
        L = __popcll(am[0]);
        bon = last + 1 < 64 ? __builtin_amdgcn_readlane(in.tgt0, (last + 1) & 63) : in.tgt64;
    } else {
    wsync();
#pragma unroll
    for (int r = 0; r < 4; r++) {
        int j = lane + 64 * r;
        if (j < n) {
            const bool wellformed = mp[r] >= -1 && mp[r] < j;
            s_ok[j] = wellformed && mt[r] == s_tgt[mp[r] + 1];
            s_anc[j] = wellformed ? mp[r] : -1;
        }
    }
    wsync();
    for (int round = 0; round < 8; round++) {  // 2^8 >= the deepest possible path
        int32_t ok[4], an[4];
        bool open = false;
#pragma unroll
        for (int r = 0; r < 4; r++) {
            int j = lane + 64 * r;
            ok[r] = 0; an[r] = -1;
            if (j < n) {
                const int a = s_anc[j];
                ok[r] = s_ok[j];
                if (a >= 0) {
                    ok[r] &= s_ok[a];
                    an[r] = s_anc[a];
                    open = true;
                }
            }
        }
        if (!__ballot(open)) break;
        wsync();
#pragma unroll
        for (int r = 0; r < 4; r++) {
            int j = lane + 64 * r;
            if (j < n) { s_ok[j] = ok[r]; s_anc[j] = an[r]; }
        }
        wsync();
    }
#pragma unroll
    for (int r = 0; r < 4; r++) {
        int j = lane + 64 * r;
        am[r] = __ballot(j < n && s_ok[j]);
        if (am[r]) last = 64 * r + 63 - __clzll((unsigned long long)am[r]);
        L += __popcll(am[r]);
    }
    bon = s_tgt[last + 1];
    }
    int32_t *row = nullptr;
    int32_t old = 0, slot_of_b = 0;
    bool slot_ok = false;
    if (APPEND) {  // L accepted tokens and the bonus token go behind the slot's context
        // (a caller that has looked up the slot and its length already passes them in)
        const int32_t slot = known_slot != -2 ? known_slot : (ap.slot_ids ? ap.slot_ids[b] : b);
        if (slot < 0 || slot >= ap.max_slots) {
            if (lane == 0) atomicOr(&ap.err[SD_DEVERR_SLOT], 1);
        } else {
            slot_ok = true;
            slot_of_b = slot;
            old = known_slot != -2 ? known_len : ap.r_len[slot];
            if ((int64_t)old + L + 1 > ap.max_ctx) {
                if (lane == 0) atomicOr(&ap.err[SD_DEVERR_CTX], 1);
            } else {
                row = ap.r_text + (int64_t)slot * ap.stride;
            }
        }
    }
    int done = 0;
#pragma unroll
    for (int r = 0; r < 4; r++) {
        int j = lane + 64 * r;
        if ((am[r] >> lane) & 1ull) {
            const int at = done + __popcll(am[r] & lanemask_lt());
            path[at] = j;
            if (APPEND && row) {
                int32_t t = mt[r];
                if (t < 0 || t >= ap.vocab) {
                    atomicOr(&ap.err[SD_DEVERR_TOKEN], 1);
                    t = 0;
                }
                row[old + at] = t;
                if (s_new) s_new[at] = t;
            }
        }
        done += __popcll(am[r]);
    }
    for (int i = L + lane; i < max_nodes; i += 64) path[i] = -1;
    if (lane == 0) {
        aa.accept_len[b] = L;
        aa.bonus[b] = bon;
        ctr[SD_CTR_ACCEPT_REQUESTS] = c_req + 1ull;
        ctr[SD_CTR_ACCEPT_LEN] = c_len + (unsigned long long)L;
        if (APPEND && row) {
            int32_t t = bon;
            if (t < 0 || t >= ap.vocab) {
                atomicOr(&ap.err[SD_DEVERR_TOKEN], 1);
                t = 0;
            }
            row[old + L] = t;
            if (s_new) s_new[L] = t;
            ap.r_len[slot_of_b] = old + L + 1;
        }
    }
    return !slot_ok ? 0 : (row ? old + L + 1 : old);
}

template <bool APPEND>
__global__ __launch_bounds__(64) void k_accept(const int32_t *__restrict__ n_nodes,
                                               const int32_t *__restrict__ tokens,
                                               const int32_t *__restrict__ parents, int max_nodes,
                                               AcceptArgs aa, AppendArgs ap) {
    __shared__ int32_t s_tgt[257];
    __shared__ int32_t s_anc[256];
    __shared__ int32_t s_ok[256];
    const AcceptIn in = accept_fetch(blockIdx.x, n_nodes, tokens, parents, max_nodes, aa);
    accept_wave<APPEND>(blockIdx.x, in, tokens, parents, max_nodes, aa, ap, s_tgt, s_anc, s_ok,
                        nullptr);
}

// GenerateCandidateTree for one request per workgroup.  All waves first build the request's
// occurrence lists together and match the P patterns against the global index; then each wave
// takes runs of pattern lengths with equal counts from a queue in LDS, longest patterns first,
// and keeps the best tree it has seen in its own LDS (two tree buffers per wave: the tree
// being grown and the wave's best so far).  The strictly-greater
// scan of Alg. 1 over (global, p = 1..P), (request, p = 1..P) picks the earliest unit among
// those with the top SCORE, so "best" means SCORE high, then scan position low; the waves'
// candidates meet in LDS after a barrier and the winning wave writes its tree out, padded
// with -1 / 0.0.  Nothing but the final tree leaves the compute unit.
constexpr int SPEC_OCC = 6;       // waves per SIMD that one or two resident workgroups may fill
constexpr int SPEC_RESIDENT = 4;  // workgroups per compute unit the wave count is sized for

// With ACCEPT the workgroup first settles the verification of the request's previous tree (the
// one `out` still holds, against aa.target) on its first wave, appends the accepted tokens and
// the bonus token to the request's context, and then drafts the next tree from the extended
// context into `out`: the end of one decoding step and the start of the next in one launch.
template <bool STATS, bool TICKS, bool ACCEPT>
// (At least six waves per SIMD: two workgroups of twelve waves are resident together when two
// requests share a compute unit; that is a bound on the kernel's registers.)
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(6))) void k_speculate(SpecParams p, const int32_t *__restrict__ slot_ids,
                                                    sd_trees out, int lds_per_wave, AcceptArgs aa,
                                                    AppendArgs ap) {
    extern __shared__ double smem[];
    __shared__ WgShared sh;
    // the wave index is the same in all lanes: keep it (and every LDS address derived from it)
    // in scalar registers
    const int lane = threadIdx.x & 63, wave = uni((int32_t)(threadIdx.x >> 6)), nw = blockDim.x >> 6;
    const int b = blockIdx.x;
    unsigned nb = 0;
    // (no slot ids given: request b is slot b, and the chain of dependent loads that every
    // request starts with is one load shorter)
    const int32_t slot = slot_ids ? uni(slot_ids[b]) : b;
    const bool slot_ok = slot >= 0 && slot < p.max_slots;
    if (!slot_ok && threadIdx.x == 0) atomicOr(&p.err[SD_DEVERR_SLOT], 1);
    // (fused form: what the acceptance reads is asked for before anything waits for memory)
    AcceptIn ain = {};
    if (ACCEPT && wave == 0) ain = accept_fetch(b, out.d_n_nodes, out.d_tokens, out.d_parents, out.max_nodes, aa);
    // the context length before this launch appends anything
    const int t_old = slot_ok ? uni(p.r_len[slot]) : 0;
    const int32_t *x = p.r_text + (int64_t)(slot_ok ? slot : 0) * p.r_stride;

    // MatchPattern on the global index for every pattern length, spread over the waves.  The
    // pattern tokens are fetched together with the context scan's first loads, and the
    // dependent loads of the matching follow once the wave has looked at its part of the scan.
    // The fused form starts the scan's loads, settles acceptance and append on the first wave
    // meanwhile, and fetches the pattern tokens once the appended tokens are in memory.
    const int P = p.P;
    const uint64_t wg0 = TICKS ? wall_clock64() : 0;
    int2 *const s_sort = reinterpret_cast<int2 *>(smem);
    ScanState scan;
    occ_scan_issue<STATS>(t_old, x, sh, scan, nb);
    // the request's row of counters (what sd_get_stats reports): read now by the last wave,
    // behind the scan's loads, and written back by it with this launch's share at the end,
    // beside the wave that writes the tree (a single wave issues an instruction every few
    // cycles, so even fifty more of them on the winner's path held every launch up by a
    // third of a microsecond).  Plain loads and stores: a row belongs to one workgroup per
    // launch.
    unsigned long long ctr_old = 0;
    if (wave == nw - 1 && lane < SD_CTR_ACCEPT_REQUESTS)
        ctr_old = p.counters[(int64_t)b * SD_CTR_STRIDE + lane];
    int t = t_old;
    // lane k < P: the k-th token from the context's end.  Loaded now for the context as it
    // stands; the fused form puts the tokens it appends in front afterwards, from LDS, so
    // that nothing has to be read back from the row once the acceptance is settled.
    int32_t tail = 0;
    if (lane < P && lane < t_old) tail = x[t_old - 1 - lane];
    // lane k: pattern token k of the wave's first two pattern lengths (taken from the tail)
    int32_t wkA0 = 0, wkB0 = 0;
    auto pattern_tokens = [&]() {
        const int plA = 1 + wave, plB = plA + nw;
        const int32_t a = __shfl(tail, (plA - 1 - lane) & 63), bb = __shfl(tail, (plB - 1 - lane) & 63);
        if (plA <= P && plA <= t && lane < plA) wkA0 = a;
        if (plB <= P && plB <= t && lane < plB) wkB0 = bb;
    };
    if (ACCEPT) {
        if (wave == 0) {
            // LDS that the occurrence sort takes over afterwards
            int32_t *s_tgt = reinterpret_cast<int32_t *>(smem), *s_anc = s_tgt + 260, *s_ok = s_anc + 256;
            const int nl = accept_wave<true>(b, ain, out.d_tokens, out.d_parents,
                                             out.max_nodes, aa, ap, s_tgt, s_anc, s_ok, sh.newtok,
                                             slot, t_old);
            if (lane == 0) sh.t_new = nl;
        }
        // The barrier orders the first wave's stores to the row before the other waves' loads
        // at workgroup scope, which is all that is needed: the waves of a workgroup share one
        // compute unit and its cache, and only this workgroup touches the row.
        __syncthreads();
        t = slot_ok ? uni(sh.t_new) : 0;
        {   // the appended tokens come first in the tail, the old tail moves back
            const int n_new = t - t_old;  // (0 for a bad slot or an append that did not fit)
            const int32_t moved = __shfl(tail, (lane - n_new) & 63);
            if (n_new > 0) tail = lane < P && lane < t ? (lane < n_new ? sh.newtok[n_new - 1 - lane] : moved) : 0;
        }
        pattern_tokens();
    } else {
        pattern_tokens();
        __syncthreads();  // the counters of the occurrence list are set
    }
    // (the counters wait in LDS for the end of the launch: two registers less to carry through
    // matching and expansion; the load is older than the tail's, which has just been waited for)
    if (wave == nw - 1 && lane < SD_CTR_ACCEPT_REQUESTS) sh.ctr[lane] = ctr_old;
    request_occurrences<STATS, ACCEPT>(p, b, t, t_old, sh.newtok, x, s_sort, sh, scan, tail, nb, [&]() {
        // List form: the suffixes that start with the context's last two tokens are located
        // once (every wave does that for itself: same loads, no barrier).  If there are at
        // most 64 of them, every longer pattern's occurrences are among them: the waves share
        // them out and count how far each agrees with the context's tail to the left, which
        // settles all pattern lengths in two more rounds of loads (suffix array, text), and
        // the expansions get their suffix lists from LDS.  Otherwise every pattern length is
        // searched for on its own, as below.
        if (P >= 2 && t >= 2 && p.g_N > 0) {
            const int32_t w_last = __builtin_amdgcn_readlane(tail, 0), w_prev = __builtin_amdgcn_readlane(tail, 1);
            const int32_t bv = lane < 4 ? p.g_bucket[(lane < 2 ? w_prev : w_last) + 1 + (lane & 1)] : 0;
            if (lane < 4) SD_CNT(4);
            int32_t lo2 = __builtin_amdgcn_readlane(bv, 0), hi2 = __builtin_amdgcn_readlane(bv, 1);
            const int32_t lo1 = __builtin_amdgcn_readlane(bv, 2), hi1 = __builtin_amdgcn_readlane(bv, 3);
            // (a first token with a bucket beyond the sampled lookup's reach would cost a long
            // search here and most likely leave more than 64 suffixes: not tried)
            const bool reach = hi2 - lo2 <= SAMPLED_MAX;
            if (reach && lo2 < hi2) col_stage<STATS>(p, w_last, lo2, hi2, nb);
            const int n2 = hi2 > lo2 ? hi2 - lo2 : 0;
            if (__builtin_expect(reach && n2 <= 64, 1)) {
                // (stored at once: two values less to keep through the loop)
                if (threadIdx.x == 0) { sh.g_lo[1] = lo1; sh.g_hi[1] = hi1; }
                int pplog = 0;
                while ((1 << pplog) < P) pplog++;
                const int PP = 1 << pplog, G = 64 >> pplog, g = lane >> pplog, k = lane & (PP - 1);
                const uint64_t gmask = PP >= 64 ? ~0ull : ((1ull << PP) - 1ull);
                const int32_t tl = __shfl(tail, k);
                constexpr int U = 4;
                for (int i0 = wave * G * U; i0 < n2; i0 += nw * G * U) {
                    int32_t ee[U], v[U];
#pragma unroll
                    for (int u = 0; u < U; u++) {  // where the suffix's second token sits
                        const int i = i0 + u * G + g;
                        ee[u] = i < n2 ? p.g_sa[lo2 + i] + 1 : -1;
                        if (i < n2 && k == 0) SD_CNT(4);
                    }
#pragma unroll
                    for (int u = 0; u < U; u++) {
                        int lim = ee[u] + 1 < P ? ee[u] + 1 : P;  // (0 for an empty place)
                        lim = lim < t ? lim : t;
                        const bool rd = ee[u] >= 0 && k < lim;
                        v[u] = rd ? p.g_text[ee[u] - k] : tl;
                        if (rd) SD_CNT(4);
                    }
#pragma unroll
                    for (int u = 0; u < U; u++) {
                        int lim = ee[u] + 1 < P ? ee[u] + 1 : P;
                        lim = lim < t ? lim : t;
                        const uint64_t mis = __ballot(k >= 1 && k < lim && v[u] != tl);
                        const uint64_t gm = (mis >> (g << pplog)) & gmask;
                        const int l = gm ? __ffsll((unsigned long long)gm) - 1 : lim;
                        if (k == 0 && ee[u] >= 0) {
                            const int i = i0 + u * G + g;
                            sh.gl_pos[i] = ee[u] - 1;
                            sh.gl_L[i] = l;
                            atomicAdd(&sh.gcnt[l], 1);
                        }
                    }
                }
                if (threadIdx.x == 0) { sh.g_mode = 1; sh.g_n2 = n2; }
                return;
            }
        }
        if (threadIdx.x == 0) sh.g_mode = 0;
        for (int plA = 1 + wave; plA <= P; plA += 2 * nw) {
            const int plB = plA + nw;  // a wave takes its pattern lengths two at a time
            const bool okA = plA <= t && p.g_N > 0, okB = plB <= P && plB <= t && p.g_N > 0;
            int32_t loA = 0, hiA = 0, loB = 0, hiB = 0;
            const bool first = plA == 1 + wave;
            int32_t wkA = wkA0, wkB = wkB0;
            if (!first) {
                wkA = okA && lane < plA ? x[t - plA + lane] : 0;
                wkB = okB && lane < plB ? x[t - plB + lane] : 0;
            }
            if (okA && lane < plA) SD_CNT(4);
            if (okB && lane < plB) SD_CNT(4);
            if (okA && okB && plB <= 32)
                match_global_pair<STATS>(p, wkA, plA, wkB, plB, loA, hiA, loB, hiB, nb);
            else {
                if (okA) match_global<STATS>(p, wkA, plA, loA, hiA, nb);
                if (okB) match_global<STATS>(p, wkB, plB, loB, hiB, nb);
            }
            if (lane == 0) {
                sh.g_lo[plA] = loA; sh.g_hi[plA] = hiA;
                if (plB <= P) { sh.g_lo[plB] = loB; sh.g_hi[plB] = hiB; }
            }
        }
        // (a frequent last token: the waves that are done with their searches early take the
        // left-extensions and the per-wave part of the occurrence sort meanwhile)
        // (in the decode step's form of the kernel; the form without the acceptance has no
        // register left for the call)
        if (ACCEPT) {
            const unsigned cnt_chunks = occ_take_chunks<STATS>(nw, t, P, p.D - 1, p.occ_cap, p.key_toks,
                                                               p.key_bits, p.alpha, tail, x, s_sort, sh);
            SD_CNT(cnt_chunks);
        }
    });
    const uint64_t wg1 = TICKS ? wall_clock64() : 0;

    // per-wave LDS: frontier (score, tok, par, lo, hi, dep), two trees (score, tok, par), staging
    const int cap = p.max_nodes;
    Frontier f;
    f.score = smem + (size_t)wave * (lds_per_wave / 8);
    double *const tsc0 = f.score + cap, *const tsc1 = tsc0 + cap;
    f.tok = (int32_t *)(tsc1 + cap);
    f.par = f.tok + cap; f.lo = f.par + cap; f.hi = f.lo + cap; f.dep = f.hi + cap;
    int32_t *const ttk0 = f.dep + cap, *const tpr0 = ttk0 + cap;
    int32_t *const ttk1 = tpr0 + cap, *const tpr1 = ttk1 + cap;
    Stage sg;
    sg.pos = tpr1 + cap; sg.cb = sg.pos + 64; sg.tc = sg.cb + 64; sg.tmp = sg.tc + TC_TOKENS;
    f.n = 0; f.cap = 0;

    // Pattern lengths with the same number of occurrences in an index have the same
    // occurrences (the longer pattern's are among the shorter one's), hence the same subtree
    // below the matched node: their trees are prefixes of one greedy order, cut at K(p) nodes,
    // unless the depth bound D interferes.  So per run of equal counts only the longest pattern
    // is expanded; if no node of depth D was taken, every shorter pattern of the run has the
    // same tree when its K reaches that size (and a strictly lower SCORE otherwise), and the
    // strictly-greater scan of Alg. 1 would keep the shortest of those.  If the bound did
    // interfere, the next shorter pattern is expanded on its own, and so on.
    // A pattern of length q with q + K(q) >= D could reach the bound; whether it does is only
    // known after its expansion, and waiting for that would serialise the run.  Such patterns
    // are therefore taken one by one (all in parallel), and runs are formed among the shorter
    // ones, where the bound cannot interfere.
    // Runs: entry i stands for pattern length P - i; lane i looks at entry i.
    int cg = 0, cr = 0, cgp = -1, crp = -1;
    bool alone = true;  // the next longer pattern may reach the depth bound
    const bool listed = uni(sh.g_mode) != 0;
    // list form: lane i (pattern length P - i) gets the number of listed suffixes that match
    // at least that many tokens (a running sum over gcnt[P], gcnt[P - 1], ...)
    const int32_t gsum = listed ? wave_inclusive_sum(lane < P ? sh.gcnt[P - lane] : 0) : 0;
    const int32_t gsum_up = __shfl_up(gsum, 1);
    if (lane < P) {
        const int pl = P - lane;
        cg = listed && pl >= 2 ? gsum : sh.g_hi[pl] - sh.g_lo[pl];
        cr = sh.cnt[pl];
        if (lane > 0) {
            cgp = listed ? gsum_up : sh.g_hi[pl + 1] - sh.g_lo[pl + 1];
            crp = sh.cnt[pl + 1];
            alone = pl + 1 + (int)floor(p.alpha * (double)(pl + 1)) >= p.D;
        }
    }
    // a request-side list of one entry is the context's own tail: nothing follows it
    const uint64_t start_g = __ballot(lane < P && cg > 0 && (alone || cg != cgp));
    const uint64_t start_r = __ballot(lane < P && cr > 1 && (alone || cr != crp));
    const int ng = __popcll(start_g), nruns = ng + __popcll(start_r);
    // A request-side suffix list of more than 64 occurrences is written to the request's row
    // of scratch memory (max_ctx words), which the runs share: going through the runs in queue
    // order, each such run gets the words behind the previous one's, and when the row is full
    // the next run starts a new round at the row's beginning.  A round begins with a workgroup
    // barrier, so every list of the round before is done with.  One list always fits (it holds
    // at most as many occurrences as the context has tokens); on the workloads at hand all of
    // a request's lists fit together and there is one round.
    const uint64_t wide_r = start_r & __ballot(lane < P && cr > 64);
    // (round, offset into the row) of the k-th request-side run
    auto place = [&](int kth, int &round, int &off) {
        int rnd = 0, used = 0, o = 0;
        uint64_t mm = start_r;
        for (int k = 0; k <= kth; k++) {
            const int i = __ffsll((unsigned long long)mm) - 1;
            mm &= mm - 1;
            const int c = __builtin_amdgcn_readlane(cr, i);
            o = used;
            if (c > 64) {
                if (used + c > p.max_ctx) { rnd++; o = 0; }
                used = o + c;
            }
        }
        round = rnd;
        off = o;
    };
    int n_rounds = 1, my_round = 0;
    if (__builtin_expect(wide_r != 0, 0)) {
        int off_last;
        place(nruns - ng - 1, n_rounds, off_last);
        n_rounds++;
    }

    if (wave == nw - 1) {  // the routes this request takes, into the row of counters (lane k: counter k)
        const bool two = t >= 2 && P >= 2 && p.g_N > 0;
        const int add = lane == SD_CTR_GLOBAL_LIST ? (listed && two)
                        : lane == SD_CTR_GLOBAL_SEARCH ? (!listed && two)
                        : lane == SD_CTR_REQUEST_WIDE ? (wide_r != 0)
                        : lane == SD_CTR_OCC_IN_MEMORY ? (uni(sh.m) > p.occ_cap)
                        : lane == SD_CTR_LIST_ROUNDS ? n_rounds - 1 : 0;
        if (lane < SD_CTR_ACCEPT_REQUESTS) sh.ctr[lane] += (unsigned long long)add;
    }
    const uint64_t wg2 = TICKS ? wall_clock64() : 0;
    double best_s = 0.0;
    int best_o = -1, best_n = 0, cur = 0;
    for (;;) {
        int g = 0;
        if (lane == 0) g = atomicAdd(&sh.next, 1);
        g = uni(g);
        if (g >= nruns) break;
        const int src = g >= ng ? 1 : 0;
        int usa_off = 0;
        if (__builtin_expect(src && wide_r, 0)) {
            int rnd;
            place(g - ng, rnd, usa_off);
            for (; my_round < rnd; my_round++) __syncthreads();
        }
        uint64_t m = src ? start_r : start_g;
        for (int k = src ? g - ng : g; k > 0; k--) m &= m - 1;
        const int i0 = __ffsll((unsigned long long)m) - 1;
        m &= m - 1;
        const int i1 = m ? __ffsll((unsigned long long)m) - 1 : P;
        const int p_lo = P - i1 + 1;
        // No node scores above 1, so a tree of K(p) nodes cannot reach a SCORE above K(p): a run
        // whose longest pattern has fewer nodes to give than the best finished tree already
        // scores can neither win nor tie, whatever the order, and is left out.  (Which runs
        // that hits depends on timing; the result does not.)
        {
            const double top = uni(__longlong_as_double((long long)sh.top_bits));
            if (floor(p.alpha * (double)(P - i0)) < top) continue;
        }
        for (int pl = P - i0; pl >= p_lo; pl--) {
            double total = 0.0;
            bool deepest = false;
            const int n = run_unit<STATS, TICKS>(p, sh, b, t, x, src, pl, usa_off, f, sg, cur ? ttk1 : ttk0,
                                          cur ? tpr1 : tpr0, cur ? tsc1 : tsc0, total, deepest, nb);
            int pstar = pl;  // shortest pattern of the run with this very tree
            if (!deepest)
                while (pstar > p_lo && (int)floor(p.alpha * (double)(pstar - 1)) >= n) pstar--;
            const int order = src * P + (pstar - 1);
            if (n > 0 && total > 0.0 &&
                (best_o < 0 || total > best_s || (total == best_s && order < best_o))) {
                best_s = total; best_o = order; best_n = n;
                cur ^= 1;  // the tree just grown is kept; the next one grows into the other buffer
            }
            // (positive doubles order like their bit patterns)
            if (n > 0 && total > 0.0 && lane == 0)
                atomicMax(&sh.top_bits, (unsigned long long)__double_as_longlong(total));
            if (!deepest) break;
        }
    }
    for (; my_round < n_rounds - 1; my_round++) __syncthreads();  // the rounds this wave had no run in
    const uint64_t wg3 = TICKS ? wall_clock64() : 0;
    if (lane == 0) { sh.best_s[wave] = best_s; sh.best_o[wave] = best_o; sh.best_n[wave] = best_n; }
    __syncthreads();
    if (TICKS && lane == 0 && wave < 16) {
        // per wave: start (absolute, low 32 bits), then ticks since the start at: occurrences
        // and global matches done, runs set up, this wave out of runs, barrier passed;
        // number of runs; occurrences of the last token
        uint32_t *wt = p.wg_ticks + ((int64_t)b * 16 + wave) * 8;
        wt[0] = (uint32_t)wg0; wt[1] = (uint32_t)(wg1 - wg0); wt[2] = (uint32_t)(wg2 - wg0);
        wt[3] = (uint32_t)(wg3 - wg0); wt[4] = (uint32_t)(wall_clock64() - wg0);
        wt[5] = (uint32_t)nruns; wt[6] = (uint32_t)sh.m; wt[7] = (uint32_t)nw;
    }
    // (the lane number is taken afresh here: keeping it in a register from the kernel's start
    // to its end costs a register that the expansion needs)
    const int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    // the winning wave: top SCORE, then the earliest unit in scan order (lane w looks at wave w;
    // units are distinct, so the second criterion leaves one wave)
    double ws = 0.0;
    int wo = -1, ww = -1;
    {
        const double s = lane_e < nw ? sh.best_s[lane_e] : 0.0;
        const int o = lane_e < nw ? sh.best_o[lane_e] : -1;
        const bool valid = o >= 0;
        const double sx = wave_max_f64(valid ? s : -__longlong_as_double(0x7ff0000000000000ll));
        const bool top = valid && s == sx;
        const uint32_t ox = wave_max_u32(top ? ~(uint32_t)o : 0u);
        const uint64_t W = __ballot(top && ~(uint32_t)o == ox);
        if (W) {
            ww = __ffsll((unsigned long long)W) - 1;
            ws = sx;
            wo = (int)~ox;
        }
    }
    if (wave == nw - 1 && lane_e < SD_CTR_ACCEPT_REQUESTS) {  // lane k: counter k of the drafting calls
        const int n = ww < 0 ? 0 : sh.best_n[ww];
        const bool tree = n > 0;
        const int add = lane_e == SD_CTR_REQUESTS ? 1 : lane_e == SD_CTR_TREES ? tree : lane_e == SD_CTR_NODES ? n
                        : lane_e == SD_CTR_MATCH_LEN ? (tree ? wo % p.P + 1 : 0)
                        : lane_e == SD_CTR_FROM_REQUEST ? (tree && wo >= p.P) : 0;
        p.counters[(int64_t)b * SD_CTR_STRIDE + lane_e] = sh.ctr[lane_e] + (unsigned long long)add;
    }
    if (wave == (ww < 0 ? 0 : ww)) {
        const int n = ww < 0 ? 0 : best_n;
        const int kept = cur ^ 1;  // the buffer the wave's best tree was left in
        const int32_t *btk = kept ? ttk1 : ttk0, *bpr = kept ? tpr1 : tpr0;
        const double *bsc = kept ? tsc1 : tsc0;
        const int64_t ob = (int64_t)b * out.max_nodes;
        for (int i = lane_e; i < out.max_nodes; i += 64) {
            const bool live = i < n;
            out.d_tokens[ob + i] = live ? btk[i] : -1;
            out.d_parents[ob + i] = live ? bpr[i] : -1;
            out.d_scores[ob + i] = live ? bsc[i] : 0.0;
            SD_CNT(16);
        }
        if (lane_e == 0) {
            out.d_n_nodes[b] = n;
            out.d_tree_score[b] = ww >= 0 ? ws : 0.0;
            out.d_match_len[b] = ww >= 0 ? wo % p.P + 1 : 0;
            out.d_source[b] = ww >= 0 ? wo / p.P : -1;
            if (out.d_use_draft) out.d_use_draft[b] = (ww >= 0 && ws > p.tau) ? 1 : 0;
            SD_CNT(24);
        }
    }
    flush_count<STATS>(nb, p.algo_bytes + SD_K_SPECULATE);
}

// Greedy verification walk, one wavefront per request, without walking: a node is "good" if
// its token equals the target token at its parent; it is accepted iff it and all its
// ancestors are good (siblings carry distinct tokens, so the accepted nodes form one path).
// Ancestor chains are resolved by pointer jumping in LDS (log2(depth) rounds); because a
// parent always has a lower index than its child, the path in walk order is the accepted
// nodes in index order.
// With APPEND the accepted draft tokens and the bonus token are also written behind the context
// of the request's slot (what sd_index_append would do with them), in the same launch.
}  // namespace

// Scratch memory of sd_speculate_static: the occurrence records and suffix-list rows of its
// requests (8 bytes per request and context token), in place of the buffers a context
// allocates.  Every device the library runs on holds its own copy of the array at its own
// address; host code reaches it only through the address that hipGetSymbolAddress reports for
// the device that is current (kept per device in scratch_ptr, and per context).
static __device__ __align__(256) unsigned char scratch[SD_STATIC_SCRATCH_BYTES];
static void *scratch_ptr[64];  // by device ordinal; nullptr: not asked for yet

sd_status sd_speculate_setup(sd_ctx *c) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, c->cfg.device) != hipSuccess) return SD_ERR_HIP;
    {  // the calling thread has made c->cfg.device current
        const int dev = c->cfg.device;
        void *ptr = dev < 64 ? scratch_ptr[dev] : nullptr;
        if (!ptr) {
            if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SD_ERR_HIP;
            if (dev < 64) scratch_ptr[dev] = ptr;
        }
        c->static_scratch = ptr;
    }
    c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
    c->lds_cu = prop.maxSharedMemoryPerMultiProcessor > 0 ? prop.maxSharedMemoryPerMultiProcessor
                                                          : prop.sharedMemPerBlock;
    int optin = 0;
    if (hipDeviceGetAttribute(&optin, hipDeviceAttributeSharedMemPerBlockOptin, c->cfg.device) !=
            hipSuccess || optin <= 0)
        optin = (int)prop.sharedMemPerBlock;
    c->lds_optin = (size_t)optin > sizeof(WgShared) + 256 ? (size_t)optin - sizeof(WgShared) - 256 : 0;
    const void *kernels[4] = {reinterpret_cast<const void *>(&k_speculate<false, false, false>),
                              reinterpret_cast<const void *>(&k_speculate<true, false, false>),
                              reinterpret_cast<const void *>(&k_speculate<false, true, false>),
                              reinterpret_cast<const void *>(&k_speculate<false, false, true>)};
    for (const void *k : kernels)
        if (hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)c->lds_optin) != hipSuccess)
        return SD_ERR_HIP;
    return SD_OK;
}

namespace {

// Launches k_speculate; with `aa` the fused form that first accepts and appends.
sd_status launch_speculate(sd_ctx *c, const int32_t *d_slot_ids, int32_t batch, sd_trees out,
                           const AcceptArgs *aa, hipStream_t st, uint32_t *occ = nullptr,
                           int32_t *unit_sa = nullptr) {
    SpecParams p;
    p.g_text = c->g_text; p.g_sa = c->g_sa; p.g_bucket = c->g_bucket; p.g_tok1 = c->g_tok1; p.g_tok1s = c->g_tok1s;
    p.g_N = (int32_t)c->g_N;
    p.r_text = c->r_text; p.r_len = c->r_len; p.r_stride = c->r_stride;
    p.max_slots = c->cfg.max_batch_slots; p.max_ctx = c->cfg.max_ctx_tokens;
    p.D = c->cfg.D; p.P = c->cfg.P; p.max_nodes = c->max_nodes;
    p.alpha = c->cfg.alpha; p.min_score = c->cfg.min_score; p.tau = c->cfg.tau;
    p.den_mode = c->cfg.den_mode; p.linear = c->cfg.linear;
    p.occ = occ ? occ : c->s_occ; p.unit_sa = unit_sa ? unit_sa : c->s_unit_sa;
    p.key_bits = sd_bits_for((uint64_t)c->cfg.vocab);  // codes 0 .. vocab
    p.key_toks = 3 * p.key_bits + 1 <= 64 ? 3 : 2;
    p.err = c->d_err;
    p.counters = c->d_counters;
    p.algo_bytes = c->d_algo_bytes;
    p.unit_ticks = c->s_unit_ticks;
    p.wg_ticks = c->s_unit_ticks + (int64_t)c->tick_slots * 2 * c->cfg.P * 4;
    // (the timing variant indexes its marks by request: only calls that the buffers have room for)
    const bool stats = c->prof_mode == 2, ticks = c->prof_mode == 3 && batch <= c->tick_slots;
    // per wave: frontier 6 arrays, two trees of 3 arrays, staging
    size_t lds_wave = (size_t)c->max_nodes * (3 * sizeof(double) + 9 * sizeof(int32_t)) +
                      (64 + 64 + TC_TOKENS + 128) * sizeof(int32_t);
    lds_wave = (lds_wave + 7) / 8 * 8;
    // Waves per request.  One workgroup per compute unit takes the 16 waves a workgroup can
    // have; two share SPEC_OCC waves per SIMD between them (12 each if the LDS allows: the
    // registers of the kernel leave room for 7 waves per SIMD, and 14 each were not resident
    // together); three and four likewise (8 and 6 each, or what the LDS allows).  Larger batches
    // are throughput work: a compute unit's LDS holds about 20 waves' worth of frontier and
    // staging at the largest tree sizes, so up to eight workgroups per compute unit get 5 waves
    // (four resident at a time, the rest wait their turn) and more get 4 (five resident; less
    // idle time at the workgroup's barriers).  Thinner workgroups lose: every request then
    // takes longer and the end of the launch runs half empty.
    const int per_cu_all = (batch + c->n_cu - 1) / c->n_cu;
    const int per_cu = per_cu_all < SPEC_RESIDENT ? per_cu_all : SPEC_RESIDENT;
    int nw = per_cu_all <= 2 ? 4 * SPEC_OCC / per_cu_all
             : per_cu_all == 3 ? 8 : per_cu_all == 4 ? 6 : per_cu_all <= 8 ? 5 : 4;
    const size_t lds_cu = c->lds_cu > 2048 * (size_t)per_cu ? c->lds_cu - 2048 * (size_t)per_cu : 0;
    while (nw > 1 && (size_t)nw * lds_wave * per_cu > lds_cu) nw--;
    if (nw > 16) nw = 16;
    if (nw < 1) nw = 1;
    size_t lds = (size_t)nw * lds_wave;
    // the occurrence sort keeps up to OCC_LDS_SORT records and their keys in the same LDS
    // before the waves take it over: as many as fit, and room for at least half of that
    const size_t rec = sizeof(int2) + sizeof(uint64_t);
    if (lds < OCC_LDS_SORT / 2 * rec) lds = OCC_LDS_SORT / 2 * rec;
    if (lds > c->lds_optin) return SD_ERR_CAPACITY;
    p.occ_cap = lds / rec < (size_t)OCC_LDS_SORT ? (int32_t)(lds / rec) : OCC_LDS_SORT;
    const dim3 grid((unsigned)batch), block(64 * nw);
    if (aa) {
        sd_span sp(c, SD_K_ACCEPT_SPECULATE, st);
        const AppendArgs ap{d_slot_ids, c->r_text, c->r_len, c->r_stride, c->cfg.max_ctx_tokens,
                            c->cfg.max_batch_slots, c->cfg.vocab, c->d_err};
        hipLaunchKernelGGL((k_speculate<false, false, true>), grid, block, lds, st, p, d_slot_ids, out,
                           (int)lds_wave, *aa, ap);
    } else {
        sd_span sp(c, SD_K_SPECULATE, st);
        const AcceptArgs none{};
        const AppendArgs nap{};
        if (stats)
            hipLaunchKernelGGL((k_speculate<true, false, false>), grid, block, lds, st, p, d_slot_ids,
                               out, (int)lds_wave, none, nap);
        else if (ticks)
            hipLaunchKernelGGL((k_speculate<false, true, false>), grid, block, lds, st, p, d_slot_ids,
                               out, (int)lds_wave, none, nap);
        else
            hipLaunchKernelGGL((k_speculate<false, false, false>), grid, block, lds, st, p, d_slot_ids,
                               out, (int)lds_wave, none, nap);
    }
    return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}

}  // namespace

sd_status sd_speculate_impl(sd_ctx *c, const int32_t *d_slot_ids, int32_t batch, sd_trees out,
                            hipStream_t st) {
    if (batch == 0) return SD_OK;
    return launch_speculate(c, d_slot_ids, batch, out, nullptr, st);
}

sd_status sd_speculate_static_impl(sd_ctx *c, const int32_t *d_slot_ids, int32_t batch, sd_trees out,
                                   hipStream_t st) {
    if (batch == 0) return SD_OK;
    // rows of max_ctx_tokens entries per request of this call: occurrence records, then lists
    const int64_t rows = (int64_t)batch * c->cfg.max_ctx_tokens;
    if (rows * (int64_t)(sizeof(uint32_t) + sizeof(int32_t)) > (int64_t)SD_STATIC_SCRATCH_BYTES)
        return SD_ERR_CAPACITY;
    uint32_t *occ = reinterpret_cast<uint32_t *>(c->static_scratch);
    int32_t *unit_sa = reinterpret_cast<int32_t *>(occ + rows);
    return launch_speculate(c, d_slot_ids, batch, out, nullptr, st, occ, unit_sa);
}

sd_status sd_accept_append_speculate_impl(sd_ctx *c, sd_trees trees, const int32_t *d_slot_ids,
                                          int32_t batch, const int32_t *d_target,
                                          int32_t *d_accept_len, int32_t *d_accept_path,
                                          int32_t *d_bonus, hipStream_t st) {
    if (batch == 0) return SD_OK;
    if (c->prof_mode >= 2) {  // the counting and timing variants exist for the separate kernels only
        const sd_status rc = sd_accept_append_impl(c, trees, d_slot_ids, batch, d_target, d_accept_len,
                                                   d_accept_path, d_bonus, st);
        return rc != SD_OK ? rc : sd_speculate_impl(c, d_slot_ids, batch, trees, st);
    }
    const AcceptArgs aa{d_target, d_accept_len, d_accept_path, d_bonus, c->d_counters};
    return launch_speculate(c, d_slot_ids, batch, trees, &aa, st);
}

sd_status sd_accept_impl(sd_ctx *c, sd_trees trees, int32_t batch, const int32_t *d_target,
                         int32_t *d_accept_len, int32_t *d_accept_path, int32_t *d_bonus,
                         hipStream_t st) {
    if (batch == 0) return SD_OK;
    sd_span sp(c, SD_K_ACCEPT, st);
    hipLaunchKernelGGL(k_accept<false>, dim3((unsigned)batch), dim3(64), 0, st, trees.d_n_nodes,
                       trees.d_tokens, trees.d_parents, trees.max_nodes,
                       AcceptArgs{d_target, d_accept_len, d_accept_path, d_bonus, c->d_counters}, AppendArgs{});
    return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}

sd_status sd_accept_append_impl(sd_ctx *c, sd_trees trees, const int32_t *d_slot_ids, int32_t batch,
                                const int32_t *d_target, int32_t *d_accept_len,
                                int32_t *d_accept_path, int32_t *d_bonus, hipStream_t st) {
    if (batch == 0) return SD_OK;
    sd_span sp(c, SD_K_ACCEPT, st);
    AppendArgs ap{d_slot_ids, c->r_text, c->r_len, c->r_stride, c->cfg.max_ctx_tokens,
                  c->cfg.max_batch_slots, c->cfg.vocab, c->d_err};
    hipLaunchKernelGGL(k_accept<true>, dim3((unsigned)batch), dim3(64), 0, st, trees.d_n_nodes,
                       trees.d_tokens, trees.d_parents, trees.max_nodes,
                       AcceptArgs{d_target, d_accept_len, d_accept_path, d_bonus, c->d_counters}, ap);
    return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}
