// Internal declarations shared by the HIP translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>
#include <string>

#include "../../include/sd.h"

#define SD_WAVE 64
#define SD_TEXT_PAD 512      // sentinel tokens kept after the last real position of a text
#define SD_END_TOKEN (-1)    // sentinel: sorts below every token and never matches one

// sticky device-side error flags (indices into sd_ctx::d_err)
enum { SD_DEVERR_TOKEN = 0, SD_DEVERR_SLOT = 1, SD_DEVERR_CTX = 2, SD_DEVERR_N = 4 };
// device-side counters reported by sd_get_stats (indices into sd_ctx::d_counters, in the
// order of the sd_stats fields from spec_requests on)
enum {
    SD_CTR_REQUESTS = 0, SD_CTR_TREES, SD_CTR_NODES, SD_CTR_MATCH_LEN, SD_CTR_FROM_REQUEST,
    SD_CTR_GLOBAL_LIST, SD_CTR_GLOBAL_SEARCH, SD_CTR_REQUEST_WIDE, SD_CTR_OCC_IN_MEMORY,
    SD_CTR_LIST_ROUNDS, SD_CTR_ACCEPT_REQUESTS, SD_CTR_ACCEPT_LEN, SD_CTR_N
};
// Every request index b of a call has a row of its own (SD_CTR_STRIDE words, the first SD_CTR_N
// in use): the workgroup that serves request b reads the row early, adds its share and stores
// it with its results, plain loads and stores (calls on one context do not overlap, and a
// launch has one workgroup per b); sd_get_stats adds the rows up.  The counters of the
// drafting calls come first, those of acceptance behind them.  (Atomic adds were measured: on
// a dozen shared addresses they queue up, 15 us per launch at batch 512; spread over 256
// addresses each they still held the end of every launch up by 0.3 to 1 us.)
#define SD_CTR_STRIDE 16

struct sd_ctx {
    sd_config cfg;
    int max_nodes;           // floor(alpha * P)
    std::string last_error;

    // ---- global index -------------------------------------------------
    // g_text: documents laid out back to back, one SD_END_TOKEN after each, then padding.
    // g_sa:   positions of g_text (sentinel positions included, they sort first) ordered by
    //         the suffix starting there, compared on at least its first D tokens.
    // g_bucket[c] (c = token + 1, 0 for the sentinel): first g_sa index whose suffix starts
    //         with a token code >= c; g_bucket[vocab + 1] = g_N.
    int32_t *g_text = nullptr;
    int32_t *g_sa = nullptr;
    int32_t *g_bucket = nullptr;
    int32_t *g_tok1 = nullptr;   // g_tok1[i] = g_text[g_sa[i] + 1]: second token of suffix i
    int32_t *g_tok1s = nullptr;  // g_tok1s[j] = g_tok1[16 j]: every 16th entry of that column
    int64_t g_cap = 0;       // capacity in positions (tokens + documents)
    int64_t g_N = 0;         // positions in use
    int64_t g_tokens = 0, g_docs = 0;

    // build scratch (sized for g_cap)
    uint64_t *b_keys[2] = {nullptr, nullptr};
    uint32_t *b_vals[2] = {nullptr, nullptr};
    uint32_t *b_rank = nullptr;
    uint32_t *b_flags = nullptr;     // group numbers by place (one of two buffers, see b_gid2)
    uint32_t *b_gid2 = nullptr;      // the other one: a doubling round reads one and writes the other
    uint32_t *b_hist = nullptr;      // per-tile digit histograms
    uint32_t *b_partials = nullptr;  // scan partial sums
    int64_t b_hist_cap = 0, b_partials_cap = 0;

    // ---- per-request contexts -----------------------------------------
    int32_t *r_text = nullptr;       // [max_batch_slots][r_stride], SD_END_TOKEN after the context
    int32_t *r_len = nullptr;        // [max_batch_slots]
    int64_t r_stride = 0;

    // ---- speculate scratch (sized for max_batch_slots requests) -------
    uint32_t *s_occ = nullptr;       // [B][max_ctx]: end position e << 7 | common-suffix length L
    int32_t *s_unit_sa = nullptr;    // [B][max_ctx]: per-request room for suffix lists of more
                                     // than 64 occurrences (shared by the pattern lengths)
    int32_t tick_slots = 0;            // requests the tick buffers have room for: min(max_batch_slots, SD_TICK_SLOTS)
    uint32_t *s_unit_ticks = nullptr;  // [B][2P][4], written by the counting kernel variants

    void *static_scratch = nullptr;  // this device's address of the library's static scratch array
    int32_t *d_err = nullptr;        // [SD_DEVERR_N]
    unsigned long long *d_counters = nullptr;  // [max_batch_slots][SD_CTR_STRIDE]
    double *d_entropy = nullptr;     // [3] accumulators of sd_index_entropy
    int32_t *d_round_flag = nullptr; // [8] per doubling round: groups too long for the in-tile sort

    int n_cu = 0;                    // compute units of the device
    size_t lds_optin = 0;            // largest dynamic LDS size a workgroup may ask for
    size_t lds_cu = 0;               // LDS of one compute unit

    // ---- measurement hooks ---------------------------------------------
    int prof_mode = 0;
    hipEvent_t *prof_ev = nullptr;   // [2 * SD_PROF_MAX_SPANS]
    int prof_kind[SD_PROF_MAX_SPANS];
    int prof_n = 0;
    unsigned long long *d_algo_bytes = nullptr;  // [SD_K_COUNT]
    int64_t index_bytes = 0, scratch_bytes = 0;
};

// ---- launchers implemented in the other translation units ---------------
// radix sort of (key, value) pairs on bits [0, nbits); result ends in keys[out_idx]/vals[out_idx]
// every kernel of the sort returns at once if run_if is given and *run_if == 0 (device memory)
int sd_sort_pairs(sd_ctx *c, int64_t n, int nbits, int in_idx, hipStream_t st,
                  const int32_t *run_if = nullptr);
// gid[i] = 1 + index of the first entry of the run of equal keys that keys[i] belongs to (sorted
// array keys[0..n)), rank[vals[i]] = gid[i].  With gid_old (another buffer: the numbers the same
// places had before), rank is stored only where the number changed.
// Every kernel returns at once if run_if is given and *run_if == 0 (device memory).
void sd_group_ranks(sd_ctx *c, const uint64_t *keys, const uint32_t *vals, int64_t n,
                    uint32_t *rank, uint32_t *gid, const uint32_t *gid_old, hipStream_t st,
                    const int32_t *run_if = nullptr);

sd_status sd_build_global_impl(sd_ctx *c, const int32_t *d_tokens, const int64_t *d_offsets,
                               int32_t n_seq, int64_t n_tokens, hipStream_t st);
sd_status sd_insert_global_impl(sd_ctx *c, const int32_t *d_tokens, const int64_t *d_offsets,
                                int32_t n_seq, int64_t n_tokens, hipStream_t st);
void sd_fill_i32(int32_t *p, int64_t n, int32_t v, hipStream_t st);
sd_status sd_entropy_impl(sd_ctx *c, double *h_mean_bits, double *h_weight, hipStream_t st);
sd_status sd_build_requests_impl(sd_ctx *c, const int32_t *d_slot_ids, const int32_t *d_tokens,
                                 const int64_t *d_offsets, int32_t n_seq, hipStream_t st);
sd_status sd_append_impl(sd_ctx *c, const int32_t *d_slot_ids, const int32_t *d_new_tokens,
                         const int32_t *d_new_offsets, int32_t n_slots, hipStream_t st);
sd_status sd_speculate_setup(sd_ctx *c);  // device limits and kernel attributes, once per context
sd_status sd_speculate_impl(sd_ctx *c, const int32_t *d_slot_ids, int32_t batch, sd_trees out,
                            hipStream_t st);
sd_status sd_speculate_static_impl(sd_ctx *c, const int32_t *d_slot_ids, int32_t batch,
                                   sd_trees out, hipStream_t st);
sd_status sd_accept_impl(sd_ctx *c, sd_trees trees, int32_t batch, const int32_t *d_target,
                         int32_t *d_accept_len, int32_t *d_accept_path, int32_t *d_bonus,
                         hipStream_t st);

sd_status sd_accept_append_speculate_impl(sd_ctx *c, sd_trees trees, const int32_t *d_slot_ids,
                                          int32_t batch, const int32_t *d_target,
                                          int32_t *d_accept_len, int32_t *d_accept_path,
                                          int32_t *d_bonus, hipStream_t st);
sd_status sd_accept_append_impl(sd_ctx *c, sd_trees trees, const int32_t *d_slot_ids, int32_t batch,
                                const int32_t *d_target, int32_t *d_accept_len,
                                int32_t *d_accept_path, int32_t *d_bonus, hipStream_t st);

// event bracket around one kernel launch when profiling is on
struct sd_span {
    sd_ctx *c;
    hipStream_t st;
    int slot;
    sd_span(sd_ctx *ctx, int kind, hipStream_t stream) : c(ctx), st(stream), slot(-1) {
        if (c->prof_mode && c->prof_n < SD_PROF_MAX_SPANS) {
            slot = c->prof_n++;
            c->prof_kind[slot] = kind;
            (void)hipEventRecord(c->prof_ev[2 * slot], st);
        }
    }
    ~sd_span() {
        if (slot >= 0) (void)hipEventRecord(c->prof_ev[2 * slot + 1], st);
    }
};

#define SD_LAUNCH(c, kind, st, kernel, grid, block, lds, ...)              \
    do {                                                                    \
        sd_span sd_sp_(c, kind, st);                                        \
        hipLaunchKernelGGL(kernel, grid, block, lds, st, __VA_ARGS__);      \
    } while (0)

static inline int sd_bits_for(uint64_t max_value) {  // bits needed to hold values 0..max_value
    int b = 1;
    while (b < 64 && (max_value >> b) != 0) b++;
    return b;
}
