/*
 * sd.h -- C ABI of the MI355X draft-generation library for SuffixDecoding
 * (arxiv 2411.04975).
 *
 * The library keeps two suffix indexes in device memory -- a GLOBAL one over
 * previously generated outputs and a PER-REQUEST one over each in-flight
 * request's prompt + output (Section 3, "Suffix Tree Construction") -- and,
 * for a batch of requests, produces one speculation tree per request
 * (Algorithm 1, GenerateCandidateTree) plus the greedy acceptance walk over a
 * verified tree (Section 2, "Speculative Decoding", step 2).
 *
 * Conventions
 *  - Every pointer named d_* is a DEVICE pointer owned by the caller (for
 *    example the storage of a torch tensor).  The library reads or writes it
 *    only through work enqueued on `hip_stream` by that call and never frees
 *    it.  Pointers without the prefix are host pointers.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *    sd_index_build, sd_index_append, sd_speculate and sd_accept only ENQUEUE
 *    work; they do not synchronise the device.  sd_create, sd_destroy and
 *    sd_get_stats synchronise.  sd_index_build of the global index and
 *    sd_index_insert wait for `hip_stream` while they enqueue (once for
 *    ordinary text, a few times for text with long repeats of frequent tokens:
 *    the host looks at what the first sorting rounds found to leave out device-wide
 *    sorts that are not needed), unless the stream is being captured into a
 *    graph: then they only enqueue.  Their last kernels are still in flight
 *    when they return.
 *  - Errors the host can see (bad arguments, sizes beyond the configured
 *    capacity) return a code at once and enqueue nothing.  Conditions only the
 *    device can see raise a sticky device flag that sd_get_stats reports: a
 *    token outside [0, vocab) is indexed as token 0 (the sequence is kept, so
 *    counts of paths through token 0 then include an occurrence that never
 *    existed: a caller that cannot rule such tokens out checks the flag); a
 *    sequence with a slot id out of range is skipped; a context, or an
 *    append to one, that would exceed max_ctx_tokens is skipped whole.
 *  - One sd_ctx belongs to one device; calls on one sd_ctx must not overlap.
 *  - Tokens are int32 in [0, vocab).  Sequence i of a (tokens, offsets) pair
 *    is tokens[offsets[i] .. offsets[i+1]).
 *  - Wherever a call takes d_slot_ids, NULL stands for the identity: sequence
 *    or request i is slot i.  A serving loop that keeps request i in slot i
 *    saves every drafting workgroup one dependent load that way.
 *
 * Readings of points the paper leaves open are part of this contract:
 *  - Depth bound D: the indexes hold every suffix cut to its first D tokens, so
 *    a path of D tokens has no continuation.  Requires 1 <= P < D.
 *  - Suffixes never run across a document (global) or past the end of the
 *    context (request).  COUNT is the number of occurrences by position.
 *  - C(N) = COUNT(N) / COUNT(PARENT(N)); D(N) is the product of C along the
 *    path from the matched node, computed in binary64 as
 *    parent_score * ((double)count_child / (double)count_parent).
 *  - The frontier of ExpandSpeculationTree is every not-yet-added child of any
 *    node already in the tree; ties go to the lower token id, then to the
 *    lower parent index.  A candidate scoring below min_score is never added.
 *  - The matched node N_p is not a draft node: sizes and SCORE count draft
 *    nodes only, at most floor(alpha * p) of them.
 *  - Between candidate trees a strictly greater SCORE wins, scanning the
 *    global index for p = 1..P first and the per-request index after it.
 *
 * Variants (sd_config): den_mode 1 uses the denominator as printed in Section 3,
 * C(N) = COUNT(N) / sum of COUNT over N's siblings (occurrences that stop at
 * the parent are left out); linear 1 is the "linear" speculation of the
 * baseline-comparison figure, which only grows one chain: after a node is
 * added, only its own children are candidates; tau is the threshold of the
 * hybrid scheme (Section 3, "Hybrid Suffix Speculative Decoding"): a request's
 * draft is flagged for use iff SCORE > tau.
 */
#ifndef SD_H
#define SD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sd_ctx sd_ctx; /* opaque; owns all index and scratch memory */

typedef enum {
    SD_OK = 0,
    SD_ERR_INVALID_ARG = 1,
    SD_ERR_OOM = 2,
    SD_ERR_HIP = 3,
    SD_ERR_CAPACITY = 4,
    SD_ERR_STATE = 5
} sd_status;

/* Limits checked by sd_create: den_mode and linear in {0, 1}, tau >= 0, 1 <= P < D <= 255, P <= 64, alpha > 0,
 * 1 <= floor(alpha*P) <= 256, 0 <= min_score <= 1, 1 <= vocab <= 2^24,
 * max_batch_slots >= 1, 1 <= max_ctx_tokens <= 2^25, 0 <= max_global_tokens (documents
 * included, each document costs one extra position) < 2^31 - 4096. */
typedef struct {
    int32_t vocab;
    int32_t D;               /* depth bound of both indexes                         */
    int32_t P;               /* longest pattern tried (Algorithm 1, "max pattern size") */
    double alpha;            /* MAX_SPEC = alpha * p (Section 3, "Adaptive Speculation Lengths") */
    double min_score;        /* per-node cut-off on D(N)                            */
    int32_t max_batch_slots; /* request slots 0 .. max_batch_slots-1                */
    int32_t max_ctx_tokens;  /* per slot, growth by sd_index_append included        */
    int64_t max_global_tokens;
    int32_t device;          /* HIP device ordinal                                  */
    int32_t den_mode;        /* 0: COUNT(parent) denominator; 1: sum over siblings  */
    int32_t linear;          /* 0: tree speculation; 1: single chain                */
    double tau;              /* hybrid threshold on SCORE (0 = always use the draft) */
} sd_config;

typedef enum { SD_SCOPE_GLOBAL = 0, SD_SCOPE_REQUESTS = 1 } sd_scope;

/* Speculation trees of a batch, all arrays caller-allocated on the device.
 * Request b owns entries [b*max_nodes, (b+1)*max_nodes) of the per-node arrays.
 * Draft node j of a request has token d_tokens[j], parent d_parents[j] (an
 * earlier node index, or -1 for a child of the matched node) and score
 * d_scores[j] = D(N); nodes appear in the order the greedy expansion added them.
 * Entries past d_n_nodes[b] are written as -1 / -1 / 0.0 so whole buffers can
 * be compared.  d_match_len[b] is the winning pattern length p (0 if none),
 * d_source[b] is 0 (global index), 1 (per-request index) or -1 (no tree),
 * d_tree_score[b] is SCORE = sum of node scores in node order (0.0 if none). */
typedef struct {
    int32_t *d_n_nodes;   /* [batch]             */
    int32_t *d_tokens;    /* [batch * max_nodes] */
    int32_t *d_parents;   /* [batch * max_nodes] */
    int32_t *d_match_len; /* [batch]             */
    int32_t *d_source;    /* [batch]             */
    double *d_scores;     /* [batch * max_nodes] */
    double *d_tree_score; /* [batch]             */
    int32_t max_nodes;    /* >= floor(alpha * P) */
    int32_t *d_use_draft; /* [batch] or NULL: 1 iff SCORE > tau (hybrid fallback gate) */
} sd_trees;

typedef struct {
    int64_t global_tokens;     /* tokens in the global index                    */
    int64_t global_docs;
    int32_t err_bad_token;     /* sticky: a token outside [0, vocab) was seen   */
    int32_t err_bad_slot;      /* sticky: a slot id outside the configured range */
    int32_t err_ctx_overflow;  /* sticky: a context would exceed max_ctx_tokens */
    int32_t reserved;
    int64_t index_bytes;       /* device bytes held by the global index         */
    int64_t scratch_bytes;     /* device bytes of scratch held by the context   */
    /* Counters of the drafting and acceptance calls, added up on the device by the kernels
     * themselves since sd_create (means are quotients of two of them; a caller that wants
     * them per call takes differences). */
    int64_t spec_requests;     /* requests drafted for (sd_speculate and the fused form)      */
    int64_t spec_trees;        /* of those: requests that got a tree of at least one node      */
    int64_t spec_nodes;        /* draft nodes of those trees                                   */
    int64_t spec_match_len;    /* winning pattern lengths p of those trees, added up           */
    int64_t spec_from_request; /* trees that came from the per-request index                   */
    int64_t spec_global_list;  /* requests whose global matches were settled for all pattern
                                  lengths at once from the suffixes of the last two tokens     */
    int64_t spec_global_search;/* requests whose pattern lengths were searched one by one      */
    int64_t spec_request_wide; /* requests with a per-request suffix list of more than 64
                                  occurrences (written to scratch memory)                      */
    int64_t spec_occ_in_memory;/* requests whose occurrence list was too long to sort in LDS   */
    int64_t spec_list_rounds;  /* extra rounds taken because such lists did not fit together   */
    int64_t accept_requests;   /* requests verified (sd_accept and the fused forms)            */
    int64_t accept_len;        /* accepted draft nodes, added up                               */
} sd_stats;

/* Validate the configuration, select `device`, allocate index capacity and
 * scratch.  On failure *out is NULL. */
sd_status sd_create(const sd_config *cfg, sd_ctx **out);
void sd_destroy(sd_ctx *ctx);
/* Text of the last host-side error of this context (owned by the context). */
const char *sd_last_error(const sd_ctx *ctx);
/* floor(alpha * P): the largest tree sd_speculate can emit (MAX_SPEC at p = P, Section 3,
 * "Adaptive Speculation Lengths"), i.e. the smallest sd_trees.max_nodes it accepts.  0 for a
 * null context. */
int32_t sd_max_nodes(const sd_ctx *ctx);

/* Build an index (Section 3, "Suffix Tree Construction").
 * SD_SCOPE_GLOBAL: the n_seq sequences are the documents of the corpus of
 *   previous outputs; the global index is replaced.  d_slot_ids is ignored.
 *   n_seq may be 0 (empty index).  Total tokens + n_seq must not exceed
 *   max_global_tokens (SD_ERR_CAPACITY).  `n_tokens` is the total token count
 *   (= offsets[n_seq], passed by the host so that no device read is needed).
 * SD_SCOPE_REQUESTS: sequence i becomes the whole context x_{1:t} of slot
 *   d_slot_ids[i], replacing what the slot held; other slots are untouched.
 *   Slot ids in one call must be distinct.
 * d_seq_offsets is int64[n_seq + 1] on the device. */
sd_status sd_index_build(sd_ctx *ctx, sd_scope scope, const int32_t *d_slot_ids,
                         const int32_t *d_tokens, const int64_t *d_seq_offsets, int32_t n_seq,
                         int64_t n_tokens, void *hip_stream);

/* Online insertion of finished outputs into the global index (Section 3: the
 * global structure is built offline from earlier outputs or kept up to date
 * online from finished requests; Appendix, "Effect of input distribution shift").  The n_seq
 * sequences (same layout and ownership as for sd_index_build: device tokens,
 * int64 device offsets, n_tokens = offsets[n_seq] given by the host) are added
 * as new documents.  Afterwards the global index holds exactly what
 * sd_index_build over the old and the new documents together would hold.
 * Cost: a sort of the new tokens plus one pass over the old index.
 * Total positions (tokens + documents) may not exceed max_global_tokens
 * (SD_ERR_CAPACITY; nothing is enqueued).  Like sd_index_build(GLOBAL), the
 * call changes sizes and buffers that later sd_speculate calls read on the
 * host side: work captured into a HIP graph before it must be captured anew. */
sd_status sd_index_insert(sd_ctx *ctx, const int32_t *d_tokens, const int64_t *d_seq_offsets,
                          int32_t n_seq, int64_t n_tokens, void *hip_stream);

/* Empirical entropy of the global index (Appendix, "Predicting SuffixDecoding
 * Effectiveness"): for every node of the depth-bounded suffix tree that has a
 * child (the root included), the entropy in bits of COUNT(child) / (sum of the
 * children's COUNTs); *h_mean_bits receives the average of these weighted by
 * that sum, *h_weight the total weight (= the number of (context, next token)
 * observations with contexts of 0..D-1 tokens).  Both are HOST pointers.
 * 0 / 0 for an empty index.  Enqueues its kernels on hip_stream, then
 * synchronises that stream.  Uses build scratch: not to be overlapped with
 * sd_index_build / sd_index_insert on another stream. */
sd_status sd_index_entropy(sd_ctx *ctx, double *h_mean_bits, double *h_weight, void *hip_stream);

/* Extend the contexts of n_slots distinct slots: slot d_slot_ids[i] receives
 * d_new_tokens[d_new_offsets[i] .. d_new_offsets[i+1]) (int32 offsets, device).
 * Afterwards the per-request index equals the one a fresh build over the longer
 * context would give (the online update of Section 3). */
sd_status sd_index_append(sd_ctx *ctx, const int32_t *d_slot_ids, const int32_t *d_new_tokens,
                          const int32_t *d_new_offsets, int32_t n_slots, void *hip_stream);

/* GenerateCandidateTree (Algorithm 1) for `batch` requests: request b uses the
 * current context of slot d_slot_ids[b].  For every pattern length p = 1..P
 * and both indexes it matches the last p context tokens (MatchPattern), grows
 * a tree of at most floor(alpha*p) nodes greedily by D(N)
 * (ExpandSpeculationTree) and keeps the tree with the highest SCORE.
 * batch <= max_batch_slots; out.max_nodes >= floor(alpha*P). */
sd_status sd_speculate(sd_ctx *ctx, const int32_t *d_slot_ids, int32_t batch, sd_trees out,
                       void *hip_stream);

/* sd_speculate for callers that cannot allocate device memory or may not touch memory that
 * was allocated at run time (code under HIP graph capture in a process whose allocator is
 * frozen, tight serving loops, harnesses that forbid hipMalloc): the same kernel with the same
 * results, but its working memory (occurrence records and suffix lists, 8 bytes per request
 * of the call and token of max_ctx_tokens) is a static array of SD_STATIC_SCRATCH_BYTES inside
 * the library's device code instead of buffers of the context; the call itself allocates and
 * frees nothing.  SD_ERR_CAPACITY, with nothing enqueued, if
 * batch * max_ctx_tokens * 8 > SD_STATIC_SCRATCH_BYTES.  Each device holds one such array
 * for the life of the process, shared by every context on it: calls that overlap on one
 * device (two streams, two contexts) race; calls that follow each other on one stream do
 * not, and nothing in the array has to survive from one call to the next. */
#define SD_STATIC_SCRATCH_BYTES (16u << 20)
sd_status sd_speculate_static(sd_ctx *ctx, const int32_t *d_slot_ids, int32_t batch, sd_trees out,
                              void *hip_stream);

/* Greedy verification walk (Section 2: drafted tokens are kept until the first
 * one the target model disagrees with; Section 4.1, simulated verifier).  d_target_tokens is
 * int32[batch * (max_nodes + 1)]: entry 0 of a request is the target model's
 * token after the context (at the tree root), entry 1+j its token after draft
 * node j.  From the root, the child whose token equals the target at the
 * current node is accepted and becomes the current node, until no child does.
 * d_accept_len[b] = number of accepted nodes, d_accept_path[b*max_nodes ..]
 * their indices in order (rest -1), d_bonus[b] = the target token at the last
 * accepted node (the token the target model contributes itself).
 * trees.max_nodes <= 256, batch <= max_batch_slots. */
sd_status sd_accept(sd_ctx *ctx, sd_trees trees, int32_t batch, const int32_t *d_target_tokens,
                    int32_t *d_accept_len, int32_t *d_accept_path, int32_t *d_bonus,
                    void *hip_stream);

/* sd_accept, and in the same launch sd_index_append of what it found: the
 * context of slot d_slot_ids[b] is extended by the tokens of request b's
 * accepted draft nodes, in path order, and then by its bonus token
 * (d_accept_len[b] + 1 tokens), which is how a decode step ends (Section 2,
 * step 2: the accepted tokens and the target model's own token join the
 * output; Section 3: the per-request structure follows the output online).
 * Outputs as for sd_accept.  Slot ids must be distinct.  A bad slot id, a
 * context that would outgrow max_ctx_tokens or a token outside [0, vocab)
 * raise the sticky flags of sd_get_stats, as sd_index_append does; the accept
 * outputs are written regardless.  batch <= max_batch_slots. */
sd_status sd_accept_append(sd_ctx *ctx, sd_trees trees, const int32_t *d_slot_ids, int32_t batch,
                           const int32_t *d_target_tokens, int32_t *d_accept_len,
                           int32_t *d_accept_path, int32_t *d_bonus, void *hip_stream);

/* sd_accept_append, and in the same launch sd_speculate for the same slots
 * from the contexts just extended: the end of one decoding step and the
 * beginning of the next (Section 2: verification, acceptance and the next
 * speculation follow each other for every request), with one kernel launch
 * between two calls of the target model instead of two.  `trees` is both
 * input (the drafts that were verified against d_target_tokens) and output
 * (the next drafts): every request's old tree is read before its new one is
 * written.  Results, flags and limits are those of sd_accept_append followed
 * by sd_speculate(ctx, d_slot_ids, batch, trees): trees.max_nodes must be
 * floor(alpha*P) <= max_nodes <= 256, slot ids distinct. */
sd_status sd_accept_append_speculate(sd_ctx *ctx, sd_trees trees, const int32_t *d_slot_ids,
                                     int32_t batch, const int32_t *d_target_tokens,
                                     int32_t *d_accept_len, int32_t *d_accept_path,
                                     int32_t *d_bonus, void *hip_stream);

/* Synchronises the device and copies counters and sticky flags to the host. */
sd_status sd_get_stats(sd_ctx *ctx, sd_stats *host_out);

/* Measurement hooks.  With profiling on, every kernel launch of the library is
 * bracketed by HIP events on the caller's stream (at most SD_PROF_MAX_SPANS
 * launches are kept between two reads).  mode 0 = off, 1 = time kernels,
 * 2 = time kernels and run the counting variant of the speculation kernel,
 * which adds up the bytes the algorithm asks for (context tokens scanned,
 * suffix-array words, text tokens, occurrence records, emitted nodes),
 * 3 = time kernels and run the timing variant of the speculation kernel,
 * which leaves wall-clock marks for the two sd_debug_read_*_ticks calls (calls of up to
 * SD_TICK_SLOTS requests: larger ones run the ordinary kernel).  sd_debug_profile_read
 * synchronises, reports per-kernel launch counts, total milliseconds and
 * counted bytes since the previous read, and clears them. */
enum {
    SD_K_SPECULATE = 0, SD_K_ACCEPT = 1, SD_K_APPEND = 2, SD_K_REQ_BUILD = 3, SD_K_SORT_HIST = 4,
    SD_K_SORT_SCAN = 5, SD_K_SORT_SCATTER = 6, SD_K_BUILD_OTHER = 7, SD_K_INSERT = 8,
    SD_K_ACCEPT_SPECULATE = 9, SD_K_COUNT = 10
};
#define SD_PROF_MAX_SPANS 8192
#define SD_TICK_SLOTS 1024
typedef struct {
    int64_t launches[SD_K_COUNT];
    double ms[SD_K_COUNT];
    int64_t algo_bytes[SD_K_COUNT];
} sd_profile;
sd_status sd_debug_profile(sd_ctx *ctx, int32_t mode);
sd_status sd_debug_profile_read(sd_ctx *ctx, sd_profile *host_out);

/* Latency profile: after an sd_speculate call made with profiling mode 3, copies four words
 * per (request, index, p) unit -- the ticks the unit spent merging tied single-occurrence
 * chains, then ticks since the unit started at the end of reading its match, of the first child
 * enumeration, and of the whole unit; unit
 * index = (b * 2 + index) * P + (p - 1), `count` = 4 * units -- and the tick rate in kHz.
 * Only units that were expanded are written (a pattern length whose tree is known from a
 * longer pattern of the same request is not); the others keep what the buffer held.
 * Synchronises. */
sd_status sd_debug_read_unit_ticks(sd_ctx *ctx, uint32_t *h_ticks, int64_t count, int32_t *khz);

/* Latency profile per request: after an sd_speculate call made with profiling mode 3, copies
 * 8 words for each of the 16 possible waves of each of the first `batch` requests of that call
 * (h_ticks holds batch * 16 * 8 words; waves that did not run leave their words untouched):
 * [0] the workgroup's start on the device-wide wall clock (low 32 bits), then ticks since that
 * start when [1] the request's occurrence lists and global matches were done, [2] the runs of
 * pattern lengths were set up, [3] this wave found no further run to take, [4] the workgroup's
 * closing barrier was passed; [5] runs of the request, [6] occurrences of its last token in its
 * context, [7] waves of the workgroup.  Also the tick rate in kHz.  Synchronises. */
sd_status sd_debug_read_request_ticks(sd_ctx *ctx, uint32_t *h_ticks, int32_t batch, int32_t *khz);

/* Test hook: synchronises, then copies the global index to host buffers:
 * the laid-out text (documents back to back, -1 after each) and the suffix
 * array over it, `*n_positions` entries each (tokens + documents).  Returns
 * SD_ERR_CAPACITY if `cap` entries are too few (only *n_positions is set). */
sd_status sd_debug_read_global(sd_ctx *ctx, int32_t *h_text, int32_t *h_sa, int64_t cap,
                               int64_t *n_positions);

#ifdef __cplusplus
}
#endif
#endif /* SD_H */
