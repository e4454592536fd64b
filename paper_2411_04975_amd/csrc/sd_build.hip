// Index construction (Section 3, "Suffix Tree Construction").
//
// Global index: instead of a pointer tree the library keeps a suffix array.  The documents
// are laid out in one text with an end marker after each; all positions are sorted by the
// suffix that starts there, compared on at least its first D tokens, with the end marker
// below every token.  A path w of the depth-bounded suffix tree then is the contiguous range
// of suffixes that start with w: COUNT(w) is the width of the range, its children are the
// runs of equal token at offset |w| inside it, and suffixes that stop at w sit first in it.
//
// The sort is prefix doubling: positions are first ordered by their leading two tokens (one
// radix sort), then each round orders them by the pair (rank of the first h tokens, rank of
// the next h tokens), which doubles the compared length until it reaches D.  Ranks are group
// numbers of the previous round, a group being numbered by the place where it starts.  A
// round only has to reorder entries inside the groups of the round before, which a workgroup
// does in LDS for a tile of the array as long as no group is longer than the tile's halo
// (k_round_small); only otherwise is the round a device-wide radix sort of 2*ceil(log2 N) bit
// keys, built in position order from the rank array (k_round_keys).  The random accesses
// of a round are the gather of the second ranks, for entries that still share a group, and
// the store of the ranks that changed.
//
// Per-request index: the contexts are kept as plain token rows (one per slot) followed by end
// markers; occurrences are found by scanning the row at speculation time, so building is a
// copy and appending writes the new tokens behind the old ones.
#include "sd_internal.h"

namespace {

constexpr int TB = 256;
// tokens per thread of k_layout_text
inline int layout_items(int64_t n_tokens) { return n_tokens >= (1 << 20) ? 16 : 1; }

// text[i + doc(i)] = tokens[i]: document j is shifted right by j to make room for one end
// marker after each earlier document.
__global__ __launch_bounds__(TB) void k_layout_text(const int32_t *__restrict__ tokens,
                                                    const int64_t *__restrict__ offs, int32_t n_seq,
                                                    int64_t n_tokens, int32_t *__restrict__ text,
                                                    int32_t vocab, int32_t *err, int items) {
    // The tokens of a workgroup (`items` per thread: many for a corpus, one for the few
    // documents of an insertion) lie in a few neighbouring documents: two threads find the
    // documents of its first and last token among all of them (a chain of dependent loads that
    // the whole workgroup waits for: hence long tiles for long inputs); the offsets of the
    // documents between go to LDS, where everyone else searches.
    constexpr int LDS_DOCS = 128;
    __shared__ int32_t s_doc[2];
    __shared__ int64_t s_offs[LDS_DOCS];
    const int64_t i0 = (int64_t)blockIdx.x * TB * items;
    const int64_t i1 = i0 + (int64_t)TB * items - 1 < n_tokens - 1 ? i0 + (int64_t)TB * items - 1 : n_tokens - 1;
    if (threadIdx.x < 2) {
        const int64_t q = threadIdx.x ? i1 : i0;
        int32_t lo = 0, hi = n_seq;  // largest j with offs[j] <= q, in [lo, hi)
        while (hi - lo > 1) {
            int32_t mid = (lo + hi) >> 1;
            if (offs[mid] <= q) lo = mid; else hi = mid;
        }
        s_doc[threadIdx.x] = lo;
    }
    __syncthreads();
    const int32_t d0 = s_doc[0], d1 = s_doc[1];
    const bool in_lds = d1 - d0 < LDS_DOCS;
    if (in_lds && (int)threadIdx.x <= d1 - d0) s_offs[threadIdx.x] = offs[d0 + threadIdx.x];
    __syncthreads();
    for (int k = 0; k < items; k++) {
        const int64_t i = i0 + (int64_t)k * TB + threadIdx.x;
        if (i >= n_tokens) break;
        // largest j with offs[j] <= i
        int32_t lo = d0, hi = d1 + 1;  // answer in [lo, hi)
        while (hi - lo > 1) {
            int32_t mid = (lo + hi) >> 1;
            if ((in_lds ? s_offs[mid - d0] : offs[mid]) <= i) lo = mid; else hi = mid;
        }
        int32_t t = tokens[i];
        if (t < 0 || t >= vocab) {
            atomicOr(&err[SD_DEVERR_TOKEN], 1);
            t = 0;
        }
        text[i + lo] = t;
    }
}

__global__ __launch_bounds__(TB) void k_layout_marks(const int64_t *__restrict__ offs, int32_t n_seq,
                                                     int64_t N, int32_t *__restrict__ text) {
    int64_t j = (int64_t)blockIdx.x * TB + threadIdx.x;
    if (j < n_seq) text[offs[j + 1] + j] = SD_END_TOKEN;
    if (j < SD_TEXT_PAD) text[N + j] = SD_END_TOKEN;
}

__global__ __launch_bounds__(TB) void k_init_keys(const int32_t *__restrict__ text, int64_t N,
                                                  int tok_bits, uint64_t *__restrict__ keys,
                                                  uint32_t *__restrict__ vals) {
    int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x;
    if (i >= N) return;
    uint64_t a = (uint64_t)(text[i] + 1), b = (uint64_t)(text[i + 1] + 1);
    keys[i] = (a << tok_bits) | b;
    vals[i] = (uint32_t)i;
}

// Key of position q for the next round: (group number of its first h tokens, group number of
// the h tokens after them), with the position itself as the value.  Built in position order:
// both ranks are read in order (the second h entries further on), nothing is gathered; the
// radix sort does not care in which order its input arrives.
__global__ __launch_bounds__(TB) void k_round_keys(const uint32_t *__restrict__ rank, int64_t N,
                                                   int64_t h, int rank_bits,
                                                   uint64_t *__restrict__ keys,
                                                   uint32_t *__restrict__ vals,
                                                   const int32_t *__restrict__ run_if) {
    if (run_if && *run_if == 0) return;  // (a small grid: switched off, it costs next to nothing)
    for (int64_t q = (int64_t)blockIdx.x * TB + threadIdx.x; q < N; q += (int64_t)gridDim.x * TB) {
        uint64_t r1 = rank[q];
        uint64_t r2 = (q + h < N) ? rank[q + h] : 0u;
        keys[q] = (r1 << rank_bits) | r2;
        vals[q] = (uint32_t)q;
    }
}

// Second-token column from the keys of the first sort (token codes of the two leading tokens).
// Every later step only reorders entries inside groups that share at least those two tokens,
// so the column by place stays what it is here.  Every 16th entry is also kept in the sampled
// column: a lookup in a bucket of a few hundred to a few thousand suffixes reads the bucket's
// samples (a sixteenth of its lines) and then only the two 16-entry blocks that hold the ends
// of the range.
__global__ __launch_bounds__(TB) void k_tok1_from_keys(const uint64_t *__restrict__ keys, int64_t N,
                                                       int tok_bits, int32_t *__restrict__ tok1,
                                                       int32_t *__restrict__ samples) {
    int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x;
    if (i >= N) return;
    const int32_t v = (int32_t)(keys[i] & ((1ull << tok_bits) - 1ull)) - 1;
    tok1[i] = v;
    if ((i & 15) == 0) samples[i >> 4] = v;
}

// One doubling round without a device-wide sort, for arrays whose groups are short.  The array
// is already ordered by the first h tokens (gid[i] = group of entry i: 1 + the place where the
// group starts), so a round only reorders inside groups, by the group number of the next h
// tokens.  A workgroup stages a tile of entries plus a halo of SMALL_HALO on both sides in
// LDS: (group, rank of the second half, position).  Every entry of the tile finds the ends of
// its group by walking left and right in LDS, counts the members that sort before it (rank of
// the second half, then previous order) and writes itself to that place of the output
// arrays, together with the number of its new group, which starts where the members with a
// lower second rank end: numbering groups by place needs no scan over the array.
// A group longer than SMALL_HALO raises *too_long: the caller then runs the radix sort round
// instead (whose kernels otherwise return at once).  The ranks by position are brought up to
// date by k_rank_update afterwards (not in here: other workgroups still read them).
constexpr int SMALL_TILE = 1024, SMALL_HALO = 64, SMALL_THREADS = 256;
constexpr int SMALL_LDS = SMALL_TILE + 2 * SMALL_HALO;

__global__ __launch_bounds__(SMALL_THREADS) void k_round_small(
    const uint32_t *__restrict__ vals, const uint32_t *__restrict__ gid,
    const uint32_t *__restrict__ rank, int64_t N, int64_t h,
    uint32_t *__restrict__ gid_out, uint32_t *__restrict__ vals_out, int32_t *too_long) {
    __shared__ uint32_t s_g[SMALL_LDS], s_r2[SMALL_LDS], s_pos[SMALL_LDS];
    const int64_t first = (int64_t)blockIdx.x * SMALL_TILE - SMALL_HALO;  // array index of LDS slot 0
    for (int k = threadIdx.x; k < SMALL_LDS; k += SMALL_THREADS) {
        const int64_t i = first + k;
        uint32_t g = 0, pos = 0;  // group 0 does not exist: marks slots outside the array
        if (i >= 0 && i < N) {
            g = gid[i];
            pos = vals[i];
        }
        s_g[k] = g; s_pos[k] = pos;
    }
    __syncthreads();
    // The rank of the second half is a random 4-byte read per entry: only entries that share
    // their group with another one need it (a group is numbered by its first place, so an
    // entry alone in its group is one whose number is its own place and whose right neighbour
    // has another number).
    for (int k = threadIdx.x; k < SMALL_LDS; k += SMALL_THREADS) {
        const int64_t i = first + k;
        uint32_t r2 = 0;
        if (i >= 0 && i < N) {
            const uint32_t g = s_g[k];
            const bool alone = g == (uint32_t)(i + 1) &&
                               (i + 1 == N || (k + 1 < SMALL_LDS && s_g[k + 1] != g));
            const int64_t q = (int64_t)s_pos[k] + h;
            if (!alone && q < N) r2 = rank[q];
        }
        s_r2[k] = r2;
    }
    __syncthreads();
    bool bad = false;
    for (int k = SMALL_HALO + threadIdx.x; k < SMALL_HALO + SMALL_TILE; k += SMALL_THREADS) {
        if (first + k >= N) break;
        const uint32_t g = s_g[k], r2 = s_r2[k];
        int lo = k, hi = k + 1;  // the group is [lo, hi)
        while (lo > 0 && k - lo < SMALL_HALO && s_g[lo - 1] == g) lo--;
        while (hi < SMALL_LDS && hi - k <= SMALL_HALO && s_g[hi] == g) hi++;
        // the walk was cut short although the group goes on: too long for this kernel
        if ((lo > 0 && s_g[lo - 1] == g) || (lo == 0 && first > 0 && s_g[0] == g) ||
            (hi < SMALL_LDS && s_g[hi] == g) || (hi == SMALL_LDS && first + SMALL_LDS < N)) {
            bad = true;
            continue;
        }
        int less = 0, before = 0;
        for (int j = lo; j < hi; j++) {
            less += s_r2[j] < r2 ? 1 : 0;
            before += (s_r2[j] == r2 && j < k) ? 1 : 0;
        }
        const int64_t dst = first + lo + less + before;
        gid_out[dst] = (uint32_t)(first + lo + less + 1);
        vals_out[dst] = s_pos[k];
    }
    if (bad) *too_long = 1;
}

// After an in-tile round: rank[position] = new group number, stored only where the number of
// the entry's place changed (places keep their old group through a round; most groups do not
// split, and the front part of a group that does keeps its number).
__global__ __launch_bounds__(TB) void k_rank_update(const uint32_t *__restrict__ vals,
                                                    const uint32_t *__restrict__ gid_new,
                                                    const uint32_t *__restrict__ gid_old, int64_t N,
                                                    uint32_t *__restrict__ rank,
                                                    const int32_t *__restrict__ skip_if) {
    if (*skip_if != 0) return;  // the round fell back to the device-wide sort, which does this itself
    for (int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x; i < N; i += (int64_t)gridDim.x * TB) {
        const uint32_t g = gid_new[i];
        if (g != gid_old[i]) rank[vals[i]] = g;
    }
}

// bucket[c] = first place whose key starts with a token code >= c, from the keys of the first
// sort (leading token code in the bits from tok_bits up): what k_bucket finds through suffix
// array and text, with one load per step of the search instead of two dependent ones.  No later
// step moves an entry out of its first token's bucket.
__global__ __launch_bounds__(TB) void k_bucket_keys(const uint64_t *__restrict__ keys, int64_t N,
                                                    int tok_bits, int32_t vocab,
                                                    int32_t *__restrict__ bucket) {
    int64_t c = (int64_t)blockIdx.x * TB + threadIdx.x;
    if (c > (int64_t)vocab + 1) return;
    int64_t lo = 0, hi = N;
    while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if ((int64_t)(keys[mid] >> tok_bits) < c) lo = mid + 1; else hi = mid;
    }
    bucket[c] = (int32_t)lo;
}

// bucket[c] = first index whose suffix starts with token code (token + 1) >= c
__global__ __launch_bounds__(TB) void k_bucket(const int32_t *__restrict__ text,
                                               const int32_t *__restrict__ sa, int64_t N,
                                               int32_t vocab, int32_t *__restrict__ bucket) {
    int64_t c = (int64_t)blockIdx.x * TB + threadIdx.x;
    if (c > (int64_t)vocab + 1) return;
    int64_t lo = 0, hi = N;
    while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if ((int64_t)text[sa[mid]] + 1 < c) lo = mid + 1; else hi = mid;
    }
    bucket[c] = (int32_t)lo;
}

// ---- online insertion into the global index -------------------------------------------------
// New documents are laid out behind the old text and sorted among themselves (the same prefix
// doubling, over the new part only).  Each new suffix is then ranked in the old suffix array by
// comparing up to D tokens (end marker lowest; a new suffix goes behind old ones it ties with),
// and old and new entries are merged into a second buffer in one pass: old entry i moves up
// by the number of new suffixes ranked at or before it, new entry j lands at rank_j + j.

typedef int32_t tok4 __attribute__((ext_vector_type(4), aligned(4)));

// rank[j] = number of old suffixes that sort before, or tie with, new suffix j
__global__ __launch_bounds__(TB) void k_insert_rank(const int32_t *__restrict__ text,
                                                    const int32_t *__restrict__ sa, int64_t N,
                                                    const int32_t *__restrict__ bucket,
                                                    const uint32_t *__restrict__ dsa, int64_t M,
                                                    int64_t base, int32_t D,
                                                    uint32_t *__restrict__ rank) {
    int64_t j = (int64_t)blockIdx.x * TB + threadIdx.x;
    if (j >= M) return;
    const int32_t *w = text + base + dsa[j];
    const int32_t c0 = w[0] + 1;  // token code, 0 for the end marker
    int64_t lo = bucket[c0], hi = bucket[c0 + 1];  // old suffixes with the same first token
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        const int32_t *v = text + sa[mid];
        int cmp = 0;  // sign of (old suffix - new suffix) on the first D tokens
        // (four tokens of either suffix per step, one 16-byte load at 4-byte alignment each:
        // neighbours in a templated corpus agree on dozens of tokens, and token by token
        // every load waited for the compare before it; what lies behind a suffix's end marker
        // is text or padding and is not looked at)
        for (int k = 0; k < D; k += 4) {
            const tok4 a4 = *reinterpret_cast<const tok4 *>(v + k), b4 = *reinterpret_cast<const tok4 *>(w + k);
            const int32_t as[4] = {a4.x, a4.y, a4.z, a4.w}, bs[4] = {b4.x, b4.y, b4.z, b4.w};
            bool done = false;
#pragma unroll
            for (int q = 0; q < 4; q++) {
                if (done || k + q >= D) continue;
                if (as[q] != bs[q]) { cmp = as[q] < bs[q] ? -1 : 1; done = true; }
                else if (as[q] == SD_END_TOKEN) done = true;
            }
            if (done) break;
        }
        if (cmp <= 0) lo = mid + 1; else hi = mid;
    }
    rank[j] = (uint32_t)lo;
}

__global__ __launch_bounds__(TB) void k_insert_merge_old(const int32_t *__restrict__ sa,
                                                         const int32_t *__restrict__ tok1, int64_t N,
                                                         const uint32_t *__restrict__ rank, int64_t M,
                                                         int32_t *__restrict__ sa_out,
                                                         int32_t *__restrict__ tok1_out,
                                                         int32_t *__restrict__ samples_out) {
    // how many new suffixes rank at or before an old entry: two threads find that for the
    // first and the last entry of the workgroup among all new suffixes; with few insertions
    // the two agree for most workgroups, and where they do not the others search between
    __shared__ int64_t s_cnt[2];
    const int64_t i0 = (int64_t)blockIdx.x * TB;
    const int64_t i1 = i0 + TB - 1 < N - 1 ? i0 + TB - 1 : N - 1;
    if (threadIdx.x < 2) {
        const int64_t q = threadIdx.x ? i1 : i0;
        int64_t lo = 0, hi = M;  // number of new suffixes with rank <= q
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if ((int64_t)rank[mid] <= q) lo = mid + 1; else hi = mid;
        }
        s_cnt[threadIdx.x] = lo;
    }
    __syncthreads();
    const int64_t i = i0 + threadIdx.x;
    if (i >= N) return;
    int64_t lo = s_cnt[0], hi = s_cnt[1];  // number of new suffixes with rank <= i
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)rank[mid] <= i) lo = mid + 1; else hi = mid;
    }
    const int32_t v = tok1[i];
    sa_out[i + lo] = sa[i];
    tok1_out[i + lo] = v;
    if (((i + lo) & 15) == 0) samples_out[(i + lo) >> 4] = v;
}

__global__ __launch_bounds__(TB) void k_insert_merge_new(const int32_t *__restrict__ text,
                                                         const uint32_t *__restrict__ dsa,
                                                         const uint32_t *__restrict__ rank, int64_t M,
                                                         int64_t base, int32_t *__restrict__ sa_out,
                                                         int32_t *__restrict__ tok1_out,
                                                         int32_t *__restrict__ samples_out) {
    int64_t j = (int64_t)blockIdx.x * TB + threadIdx.x;
    if (j >= M) return;
    const int64_t pos = base + dsa[j], dst = (int64_t)rank[j] + j;
    const int32_t v = text[pos + 1];
    sa_out[dst] = (int32_t)pos;
    tok1_out[dst] = v;
    if ((dst & 15) == 0) samples_out[dst >> 4] = v;
}

__global__ __launch_bounds__(TB) void k_fill_i32(int32_t *p, int64_t n, int32_t v) {
    int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x;
    if (i < n) p[i] = v;
}

// one workgroup per sequence: copy it into its slot row and close the row with end markers
__global__ __launch_bounds__(TB) void k_req_build(const int32_t *__restrict__ slot_ids,
                                                  const int32_t *__restrict__ tokens,
                                                  const int64_t *__restrict__ offs,
                                                  int32_t *__restrict__ r_text,
                                                  int32_t *__restrict__ r_len, int64_t stride,
                                                  int32_t max_ctx, int32_t max_slots, int32_t vocab,
                                                  int32_t *err) {
    const int s = blockIdx.x;
    const int32_t slot = slot_ids ? slot_ids[s] : s;  // no ids given: sequence s is slot s
    if (slot < 0 || slot >= max_slots) {
        if (threadIdx.x == 0) atomicOr(&err[SD_DEVERR_SLOT], 1);
        return;
    }
    const int64_t b = offs[s], len = offs[s + 1] - b;
    if (len < 0 || len > max_ctx) {
        if (threadIdx.x == 0) atomicOr(&err[SD_DEVERR_CTX], 1);
        return;
    }
    int32_t *row = r_text + (int64_t)slot * stride;
    for (int64_t i = threadIdx.x; i < stride; i += TB) {
        int32_t t = SD_END_TOKEN;
        if (i < len) {
            t = tokens[b + i];
            if (t < 0 || t >= vocab) {
                atomicOr(&err[SD_DEVERR_TOKEN], 1);
                t = 0;
            }
        }
        row[i] = t;
    }
    if (threadIdx.x == 0) r_len[slot] = (int32_t)len;
}

__global__ __launch_bounds__(64) void k_req_append(const int32_t *__restrict__ slot_ids,
                                                   const int32_t *__restrict__ new_tokens,
                                                   const int32_t *__restrict__ new_offs,
                                                   int32_t *__restrict__ r_text,
                                                   int32_t *__restrict__ r_len, int64_t stride,
                                                   int32_t max_ctx, int32_t max_slots, int32_t vocab,
                                                   int32_t *err) {
    const int s = blockIdx.x;
    const int32_t slot = slot_ids ? slot_ids[s] : s;
    if (slot < 0 || slot >= max_slots) {
        if (threadIdx.x == 0) atomicOr(&err[SD_DEVERR_SLOT], 1);
        return;
    }
    const int32_t b = new_offs[s], k = new_offs[s + 1] - b;
    const int32_t old = r_len[slot];
    if (k < 0 || (int64_t)old + k > max_ctx) {
        if (threadIdx.x == 0) atomicOr(&err[SD_DEVERR_CTX], 1);
        return;
    }
    int32_t *row = r_text + (int64_t)slot * stride;
    for (int32_t i = threadIdx.x; i < k; i += 64) {
        int32_t t = new_tokens[b + i];
        if (t < 0 || t >= vocab) {
            atomicOr(&err[SD_DEVERR_TOKEN], 1);
            t = 0;
        }
        row[old + i] = t;
    }
    __syncthreads();  // every lane has read `old` before it changes
    if (threadIdx.x == 0) r_len[slot] = old + k;
}

inline unsigned nblk(int64_t n) { return (unsigned)((n + TB - 1) / TB); }

}  // namespace

// A stream that is being captured into a graph cannot be waited for.
static bool stream_can_wait(hipStream_t st) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return cs == hipStreamCaptureStatusNone;
}

// Sorts the N positions of `text` (documents with an end marker after each, padding behind)
// by their suffixes, compared on at least D tokens.  Returns which of b_vals[0/1] holds the
// sorted positions (-1: a HIP call failed).
// A round's device-wide fall-back is some twenty launches that return at once when the in-tile
// kernel has done the round: about 2 us each, a tenth of the build of a 10M-token corpus.
// Groups only ever split, so once a round's in-tile kernel has coped, those of all later rounds
// will: the host waits for the stream after a round's in-tile kernel and reads its flag, until
// the first round that needs no fall-back; from there on the rounds are enqueued without
// fall-backs and without waiting (one wait for text without long repeats; text whose frequent
// tokens make the first rounds fall back pays a wait for each of those rounds and gets them
// back from the launches it no longer makes afterwards).  On a stream that cannot be waited
// for, every round is enqueued with its fall-back, switched by the flag on the device.
static int build_sorted_positions(sd_ctx *c, const int32_t *text, int64_t N, int32_t *tok1_out,
                                  hipStream_t st) {
    const bool can_wait = stream_can_wait(st);
    bool settled = false;  // no later round can need its fall-back
    const int tok_bits = sd_bits_for((uint64_t)c->cfg.vocab);  // codes 0..vocab
    SD_LAUNCH(c, SD_K_BUILD_OTHER, st, k_init_keys, dim3(nblk(N)), dim3(TB), 0, text, N, tok_bits, c->b_keys[0], c->b_vals[0]);
    int cur = sd_sort_pairs(c, N, 2 * tok_bits, 0, st);
    if (tok1_out) {  // (the global build: second-token column and bucket table come from these keys)
        SD_LAUNCH(c, SD_K_BUILD_OTHER, st, k_tok1_from_keys, dim3(nblk(N)), dim3(TB), 0, c->b_keys[cur], N, tok_bits, tok1_out, c->g_tok1s);
        SD_LAUNCH(c, SD_K_BUILD_OTHER, st, k_bucket_keys, dim3(nblk((int64_t)c->cfg.vocab + 2)), dim3(TB), 0, c->b_keys[cur], N, tok_bits, c->cfg.vocab, c->g_bucket);
    }
    const int rank_bits = sd_bits_for((uint64_t)N);  // ranks 0..N
    // So far the positions are ordered by their first h = 2 tokens.  Each round first tries the
    // in-tile reordering (enough once no group is longer than its halo, which stays true for
    // all later rounds); the device-wide sort follows, and does something only if that failed.
    // Both leave the round's result in the other buffer pair.
    sd_fill_i32(c->d_round_flag, 8, 0, st);
    const int passes = (2 * rank_bits + 7) / 8;  // of the radix sort: odd ones swap buffers
    // group numbers by place and ranks by position after the first sort
    uint32_t *gid = c->b_flags, *gid_next = c->b_gid2;
    if (2 < c->cfg.D)
        sd_group_ranks(c, c->b_keys[cur], c->b_vals[cur], N, c->b_rank, gid, nullptr, st);
    int round = 0;
    for (int64_t h = 2; h < c->cfg.D; h *= 2, round++) {
        int32_t *flag = c->d_round_flag + (round < 8 ? round : 7);
        SD_LAUNCH(c, SD_K_BUILD_OTHER, st, k_round_small,
                  dim3((unsigned)((N + SMALL_TILE - 1) / SMALL_TILE)), dim3(SMALL_THREADS), 0,
                  c->b_vals[cur], gid, c->b_rank, N, h, gid_next, c->b_vals[cur ^ 1], flag);
        if (can_wait && !settled) {
            int32_t too_long = 0;
            if (hipStreamSynchronize(st) != hipSuccess ||
                hipMemcpy(&too_long, flag, sizeof(too_long), hipMemcpyDeviceToHost) != hipSuccess)
                return -1;
            settled = too_long == 0;
        }
        // (after a round that fell back, the device-wide sort brings the ranks up to date)
        if (h * 2 < c->cfg.D && (settled || !can_wait))  // (the last round's numbers are not needed by anyone)
            SD_LAUNCH(c, SD_K_BUILD_OTHER, st, k_rank_update, dim3(nblk(N) < 8192u ? nblk(N) : 8192u),
                      dim3(TB), 0, c->b_vals[cur ^ 1], gid_next, gid, N, c->b_rank, flag);
        if (settled) {
            cur ^= 1;
            uint32_t *t = gid; gid = gid_next; gid_next = t;
            continue;
        }
        const int start = (passes & 1) ? cur : cur ^ 1;
        SD_LAUNCH(c, SD_K_BUILD_OTHER, st, k_round_keys, dim3(nblk(N) < 4096u ? nblk(N) : 4096u), dim3(TB), 0, c->b_rank, N, h, rank_bits, c->b_keys[start], c->b_vals[start], flag);
        (void)sd_sort_pairs(c, N, 2 * rank_bits, start, st, flag);
        if (h * 2 < c->cfg.D)
            sd_group_ranks(c, c->b_keys[cur ^ 1], c->b_vals[cur ^ 1], N, c->b_rank, gid_next, gid, st, flag);
        cur ^= 1;
        uint32_t *t = gid; gid = gid_next; gid_next = t;
    }
    return cur;
}

sd_status sd_build_global_impl(sd_ctx *c, const int32_t *d_tokens, const int64_t *d_offsets,
                               int32_t n_seq, int64_t n_tokens, hipStream_t st) {
    const int64_t N = n_tokens + n_seq;
    const int32_t vocab = c->cfg.vocab;
    c->g_N = N;
    c->g_tokens = n_tokens;
    c->g_docs = n_seq;
    if (n_tokens > 0)
        SD_LAUNCH(c, SD_K_BUILD_OTHER, st, k_layout_text, dim3(nblk((n_tokens + layout_items(n_tokens) - 1) / layout_items(n_tokens))), dim3(TB), 0, d_tokens, d_offsets, n_seq, n_tokens, c->g_text, vocab, c->d_err, layout_items(n_tokens));
    {
        int64_t m = n_seq > SD_TEXT_PAD ? n_seq : SD_TEXT_PAD;
        SD_LAUNCH(c, SD_K_BUILD_OTHER, st, k_layout_marks, dim3(nblk(m)), dim3(TB), 0, d_offsets, n_seq, N, c->g_text);
    }
    if (N > 0) {
        const int cur = build_sorted_positions(c, c->g_text, N, c->g_tok1, st);
        if (cur < 0) return SD_ERR_HIP;
        // The sorted positions are the suffix array: the buffer they are in becomes g_sa and the
        // old g_sa a scratch buffer (same sizes; a copy took 17 us for 10M positions).  The
        // second-token column was written after the first sort: inside the bucket of a first
        // token it is sorted, so the second pattern token is located by a coalesced scan of the
        // column instead of dependent (suffix array -> text) probes.
        int32_t *old_sa = c->g_sa;
        c->g_sa = reinterpret_cast<int32_t *>(c->b_vals[cur]);
        c->b_vals[cur] = reinterpret_cast<uint32_t *>(old_sa);
    }
    if (N == 0)  // (an empty index: every bucket is empty)
        SD_LAUNCH(c, SD_K_BUILD_OTHER, st, k_bucket, dim3(nblk((int64_t)vocab + 2)), dim3(TB), 0, c->g_text, c->g_sa, N, vocab, c->g_bucket);
    return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}

// Online insertion (Section 3: the global tree may also be kept up to date online with
// finished outputs; Appendix, "Effect of input distribution shift").  Afterwards the index holds
// exactly what a build over the old and the new documents together would hold.
sd_status sd_insert_global_impl(sd_ctx *c, const int32_t *d_tokens, const int64_t *d_offsets,
                                int32_t n_seq, int64_t n_tokens, hipStream_t st) {
    const int64_t N = c->g_N, M = n_tokens + n_seq;
    const int32_t vocab = c->cfg.vocab;
    if (M == 0) return SD_OK;
    int32_t *ntext = c->g_text + N;
    if (n_tokens > 0)
        SD_LAUNCH(c, SD_K_INSERT, st, k_layout_text, dim3(nblk((n_tokens + layout_items(n_tokens) - 1) / layout_items(n_tokens))), dim3(TB), 0, d_tokens, d_offsets, n_seq, n_tokens, ntext, vocab, c->d_err, layout_items(n_tokens));
    {
        int64_t m = n_seq > SD_TEXT_PAD ? n_seq : SD_TEXT_PAD;
        SD_LAUNCH(c, SD_K_INSERT, st, k_layout_marks, dim3(nblk(m)), dim3(TB), 0, d_offsets, n_seq, M, ntext);
    }
    const int cur = build_sorted_positions(c, ntext, M, nullptr, st);
    if (cur < 0) return SD_ERR_HIP;
    // b_vals[cur]: new positions in order; b_flags: their ranks in the old array; merged arrays
    // go to b_vals[1 - cur] and b_rank, which then change places with g_sa and g_tok1
    uint32_t *dsa = c->b_vals[cur], *rank = c->b_flags;
    int32_t *sa_out = (int32_t *)c->b_vals[1 - cur], *tok1_out = (int32_t *)c->b_rank;
    SD_LAUNCH(c, SD_K_INSERT, st, k_insert_rank, dim3(nblk(M)), dim3(TB), 0, c->g_text, c->g_sa, N, c->g_bucket, dsa, M, N, c->cfg.D, rank);
    if (N > 0)
        SD_LAUNCH(c, SD_K_INSERT, st, k_insert_merge_old, dim3(nblk(N)), dim3(TB), 0, c->g_sa, c->g_tok1, N, rank, M, sa_out, tok1_out, c->g_tok1s);
    SD_LAUNCH(c, SD_K_INSERT, st, k_insert_merge_new, dim3(nblk(M)), dim3(TB), 0, c->g_text, dsa, rank, M, N, sa_out, tok1_out, c->g_tok1s);
    c->b_vals[1 - cur] = (uint32_t *)c->g_sa;
    c->b_rank = (uint32_t *)c->g_tok1;
    c->g_sa = sa_out;
    c->g_tok1 = tok1_out;
    c->g_N = N + M;
    c->g_tokens += n_tokens;
    c->g_docs += n_seq;
    SD_LAUNCH(c, SD_K_INSERT, st, k_bucket, dim3(nblk((int64_t)vocab + 2)), dim3(TB), 0, c->g_text, c->g_sa, c->g_N, vocab, c->g_bucket);
    return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}

sd_status sd_build_requests_impl(sd_ctx *c, const int32_t *d_slot_ids, const int32_t *d_tokens,
                                 const int64_t *d_offsets, int32_t n_seq, hipStream_t st) {
    if (n_seq == 0) return SD_OK;
    sd_span sp(c, SD_K_REQ_BUILD, st);
    hipLaunchKernelGGL(k_req_build, dim3((unsigned)n_seq), dim3(TB), 0, st, d_slot_ids, d_tokens,
                       d_offsets, c->r_text, c->r_len, c->r_stride, c->cfg.max_ctx_tokens,
                       c->cfg.max_batch_slots, c->cfg.vocab, c->d_err);
    return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}

sd_status sd_append_impl(sd_ctx *c, const int32_t *d_slot_ids, const int32_t *d_new_tokens,
                         const int32_t *d_new_offsets, int32_t n_slots, hipStream_t st) {
    if (n_slots == 0) return SD_OK;
    sd_span sp(c, SD_K_APPEND, st);
    hipLaunchKernelGGL(k_req_append, dim3((unsigned)n_slots), dim3(64), 0, st, d_slot_ids,
                       d_new_tokens, d_new_offsets, c->r_text, c->r_len, c->r_stride,
                       c->cfg.max_ctx_tokens, c->cfg.max_batch_slots, c->cfg.vocab, c->d_err);
    return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}

// used by sd_create to put every slot row into the "empty context" state
void sd_fill_i32(int32_t *p, int64_t n, int32_t v, hipStream_t st) {
    if (n > 0) hipLaunchKernelGGL(k_fill_i32, dim3(nblk(n)), dim3(TB), 0, st, p, n, v);
}
