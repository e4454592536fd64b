// C ABI entry points: argument checks, memory ownership, stream plumbing.
#include <math.h>
#include <stdio.h>

#include <new>

#include "sd_internal.h"

void sd_fill_i32(int32_t *p, int64_t n, int32_t v, hipStream_t st);

namespace {

sd_status fail(sd_ctx *c, sd_status s, const char *msg) {
    if (c) c->last_error = msg;
    return s;
}

template <typename T>
bool dev_alloc(T **p, int64_t count, int64_t *acc) {
    *p = nullptr;
    if (count <= 0) count = 1;
    size_t bytes = (size_t)count * sizeof(T);
    if (hipMalloc((void **)p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        *p = nullptr;
        return false;
    }
    *acc += (int64_t)bytes;
    return true;
}

void free_all(sd_ctx *c) {
    void *ptrs[] = {c->g_text, c->g_sa, c->g_bucket, c->g_tok1, c->g_tok1s, c->b_keys[0], c->b_keys[1], c->b_vals[0],
                    c->b_vals[1], c->b_rank, c->b_flags, c->b_gid2, c->b_hist, c->b_partials, c->r_text,
                    c->r_len, c->s_occ, c->s_unit_sa, c->d_err, c->s_unit_ticks, c->d_entropy,
                    c->d_round_flag};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    if (c->d_algo_bytes) (void)hipFree(c->d_algo_bytes);
    if (c->prof_ev) {
        for (int i = 0; i < 2 * SD_PROF_MAX_SPANS; i++)
            if (c->prof_ev[i]) (void)hipEventDestroy(c->prof_ev[i]);
        delete[] c->prof_ev;
    }
}

}  // namespace

extern "C" {

sd_status sd_create(const sd_config *cfg, sd_ctx **out) {
    if (!out) return SD_ERR_INVALID_ARG;
    *out = nullptr;
    if (!cfg) return SD_ERR_INVALID_ARG;
    if (cfg->vocab < 1 || cfg->vocab > (1 << 24)) return SD_ERR_INVALID_ARG;
    if (cfg->P < 1 || cfg->P > 64 || cfg->D <= cfg->P || cfg->D > 255) return SD_ERR_INVALID_ARG;
    if (!(cfg->alpha > 0.0) || !(cfg->min_score >= 0.0) || !(cfg->min_score <= 1.0))
        return SD_ERR_INVALID_ARG;
    if (cfg->den_mode < 0 || cfg->den_mode > 1 || cfg->linear < 0 || cfg->linear > 1 ||
        !(cfg->tau >= 0.0))
        return SD_ERR_INVALID_ARG;
    const double mn = floor(cfg->alpha * (double)cfg->P);
    if (!(mn >= 1.0) || !(mn <= 256.0)) return SD_ERR_INVALID_ARG;
    if (cfg->max_batch_slots < 1 || cfg->max_ctx_tokens < 1 || cfg->max_global_tokens < 0 ||
        cfg->max_global_tokens >= (int64_t)2147483647 - 4096)
        return SD_ERR_INVALID_ARG;
    if (cfg->max_ctx_tokens > (1 << 25)) return SD_ERR_INVALID_ARG;  // occurrence records hold 25 bits of position
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev) {
        (void)hipGetLastError();
        return SD_ERR_HIP;
    }
    if (hipSetDevice(cfg->device) != hipSuccess) return SD_ERR_HIP;

    sd_ctx *c = new (std::nothrow) sd_ctx();
    if (!c) return SD_ERR_OOM;
    c->cfg = *cfg;
    c->max_nodes = (int)mn;
    const int64_t cap = cfg->max_global_tokens;
    c->g_cap = cap;
    const int64_t B = cfg->max_batch_slots, P = cfg->P, ctx = cfg->max_ctx_tokens;
    c->r_stride = ((ctx + SD_TEXT_PAD + 63) / 64) * 64;
    const int64_t tiles = (cap + 4095) / 4096 + 1;
    c->b_hist_cap = 256 * tiles + 256;  // (digit, tile) table + one total per digit
    const int64_t scan_n = c->b_hist_cap > cap ? c->b_hist_cap : cap;
    c->b_partials_cap = (scan_n + 4095) / 4096 + 1;
    bool ok = true;
    int64_t *ib = &c->index_bytes, *sb = &c->scratch_bytes;
    ok = ok && dev_alloc(&c->g_text, cap + SD_TEXT_PAD + 64, ib);
    // g_sa / g_tok1 change places with build scratch buffers on insertion: same sizes as those
    ok = ok && dev_alloc(&c->g_sa, cap + 64, ib);
    ok = ok && dev_alloc(&c->g_tok1, cap + 64, ib);
    ok = ok && dev_alloc(&c->g_tok1s, cap / 16 + 64, ib);
    ok = ok && dev_alloc(&c->g_bucket, (int64_t)cfg->vocab + 2, ib);
    ok = ok && dev_alloc(&c->b_keys[0], cap, sb) && dev_alloc(&c->b_keys[1], cap, sb);
    ok = ok && dev_alloc(&c->b_vals[0], cap + 64, sb) && dev_alloc(&c->b_vals[1], cap + 64, sb);
    ok = ok && dev_alloc(&c->b_rank, cap + 64, sb) && dev_alloc(&c->b_flags, cap, sb) &&
         dev_alloc(&c->b_gid2, cap, sb);
    ok = ok && dev_alloc(&c->b_hist, c->b_hist_cap, sb);
    ok = ok && dev_alloc(&c->b_partials, c->b_partials_cap, sb);
    ok = ok && dev_alloc(&c->r_text, B * c->r_stride, sb) && dev_alloc(&c->r_len, ((B + 31) / 32) * 32 + B * SD_CTR_STRIDE * 2, sb);
    ok = ok && dev_alloc(&c->s_occ, B * ctx, sb);
    ok = ok && dev_alloc(&c->s_unit_sa, B * ctx, sb);
    ok = ok && dev_alloc(&c->d_err, SD_DEVERR_N, sb) && dev_alloc(&c->d_entropy, 4, sb) &&
         dev_alloc(&c->d_round_flag, 8, sb);
    c->tick_slots = (int32_t)(B < SD_TICK_SLOTS ? B : SD_TICK_SLOTS);
    ok = ok && dev_alloc(&c->s_unit_ticks, (int64_t)c->tick_slots * (2 * P * 4 + 16 * 8), sb);
    ok = ok && dev_alloc(&c->d_algo_bytes, SD_K_COUNT, sb);
    if (!ok) {
        free_all(c);
        delete c;
        return SD_ERR_OOM;
    }
    if (sd_speculate_setup(c) != SD_OK) {
        free_all(c);
        delete c;
        return SD_ERR_HIP;
    }
    // empty global index, empty contexts, clear flags
    sd_fill_i32(c->g_text, SD_TEXT_PAD, SD_END_TOKEN, nullptr);
    sd_fill_i32(c->g_bucket, (int64_t)cfg->vocab + 2, 0, nullptr);
    sd_fill_i32(c->r_text, B * c->r_stride, SD_END_TOKEN, nullptr);
    sd_fill_i32(c->r_len, B, 0, nullptr);
    sd_fill_i32(c->d_err, SD_DEVERR_N, 0, nullptr);
    sd_fill_i32((int32_t *)c->d_algo_bytes, 2 * SD_K_COUNT, 0, nullptr);
    // the counters live behind the context lengths, in the same allocation: every workgroup
    // reads its length at its start, so the counters' page is one the compute unit has seen
    c->d_counters = reinterpret_cast<unsigned long long *>(c->r_len + ((B + 31) / 32) * 32);
    sd_fill_i32((int32_t *)c->d_counters, 2 * B * SD_CTR_STRIDE, 0, nullptr);
    if (hipDeviceSynchronize() != hipSuccess) {
        free_all(c);
        delete c;
        return SD_ERR_HIP;
    }
    *out = c;
    return SD_OK;
}

void sd_destroy(sd_ctx *c) {
    if (!c) return;
    (void)hipSetDevice(c->cfg.device);
    (void)hipDeviceSynchronize();
    free_all(c);
    delete c;
}

const char *sd_last_error(const sd_ctx *c) { return c ? c->last_error.c_str() : "null context"; }

int32_t sd_max_nodes(const sd_ctx *c) { return c ? c->max_nodes : 0; }

sd_status sd_index_build(sd_ctx *c, sd_scope scope, const int32_t *d_slot_ids,
                         const int32_t *d_tokens, const int64_t *d_seq_offsets, int32_t n_seq,
                         int64_t n_tokens, void *hip_stream) {
    if (!c) return SD_ERR_INVALID_ARG;
    if (n_seq < 0 || n_tokens < 0) return fail(c, SD_ERR_INVALID_ARG, "negative size");
    if (!d_seq_offsets) return fail(c, SD_ERR_INVALID_ARG, "d_seq_offsets is null");
    if (n_tokens > 0 && !d_tokens) return fail(c, SD_ERR_INVALID_ARG, "d_tokens is null");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    hipStream_t st = (hipStream_t)hip_stream;
    if (scope == SD_SCOPE_GLOBAL) {
        if (n_tokens + (int64_t)n_seq > c->g_cap)
            return fail(c, SD_ERR_CAPACITY, "corpus exceeds max_global_tokens");
        return sd_build_global_impl(c, d_tokens, d_seq_offsets, n_seq, n_tokens, st);
    }
    if (scope == SD_SCOPE_REQUESTS) {
        if (n_seq > c->cfg.max_batch_slots)
            return fail(c, SD_ERR_CAPACITY, "more sequences than request slots");
        return sd_build_requests_impl(c, d_slot_ids, d_tokens, d_seq_offsets, n_seq, st);
    }
    return fail(c, SD_ERR_INVALID_ARG, "unknown scope");
}

sd_status sd_index_insert(sd_ctx *c, const int32_t *d_tokens, const int64_t *d_seq_offsets,
                          int32_t n_seq, int64_t n_tokens, void *hip_stream) {
    if (!c) return SD_ERR_INVALID_ARG;
    if (n_seq < 0 || n_tokens < 0) return fail(c, SD_ERR_INVALID_ARG, "negative size");
    if (!d_seq_offsets) return fail(c, SD_ERR_INVALID_ARG, "d_seq_offsets is null");
    if (n_tokens > 0 && !d_tokens) return fail(c, SD_ERR_INVALID_ARG, "d_tokens is null");
    if (c->g_N + n_tokens + (int64_t)n_seq > c->g_cap)
        return fail(c, SD_ERR_CAPACITY, "corpus exceeds max_global_tokens");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    return sd_insert_global_impl(c, d_tokens, d_seq_offsets, n_seq, n_tokens,
                                 (hipStream_t)hip_stream);
}

sd_status sd_index_entropy(sd_ctx *c, double *h_mean_bits, double *h_weight, void *hip_stream) {
    if (!c) return SD_ERR_INVALID_ARG;
    if (!h_mean_bits || !h_weight) return fail(c, SD_ERR_INVALID_ARG, "null output pointer");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    sd_status rc = sd_entropy_impl(c, h_mean_bits, h_weight, (hipStream_t)hip_stream);
    return rc == SD_OK ? SD_OK : fail(c, rc, "entropy kernels failed");
}

sd_status sd_index_append(sd_ctx *c, const int32_t *d_slot_ids, const int32_t *d_new_tokens,
                          const int32_t *d_new_offsets, int32_t n_slots, void *hip_stream) {
    if (!c) return SD_ERR_INVALID_ARG;
    if (n_slots < 0) return fail(c, SD_ERR_INVALID_ARG, "negative size");
    if (n_slots > c->cfg.max_batch_slots)
        return fail(c, SD_ERR_CAPACITY, "more slots than configured");
    if (n_slots > 0 && (!d_new_offsets || !d_new_tokens))
        return fail(c, SD_ERR_INVALID_ARG, "null pointer");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    return sd_append_impl(c, d_slot_ids, d_new_tokens, d_new_offsets, n_slots,
                          (hipStream_t)hip_stream);
}

static bool trees_ok(const sd_trees &t) {
    return t.d_n_nodes && t.d_tokens && t.d_parents && t.d_match_len && t.d_source && t.d_scores &&
           t.d_tree_score;
}

sd_status sd_speculate(sd_ctx *c, const int32_t *d_slot_ids, int32_t batch, sd_trees out,
                       void *hip_stream) {
    if (!c) return SD_ERR_INVALID_ARG;
    if (batch < 0) return fail(c, SD_ERR_INVALID_ARG, "negative batch");
    if (batch > c->cfg.max_batch_slots)
        return fail(c, SD_ERR_CAPACITY, "batch exceeds max_batch_slots");
    if (batch == 0) return SD_OK;
    if (!trees_ok(out)) return fail(c, SD_ERR_INVALID_ARG, "null pointer");
    if (out.max_nodes < c->max_nodes)
        return fail(c, SD_ERR_INVALID_ARG, "trees.max_nodes below floor(alpha*P)");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    return sd_speculate_impl(c, d_slot_ids, batch, out, (hipStream_t)hip_stream);
}

sd_status sd_speculate_static(sd_ctx *c, const int32_t *d_slot_ids, int32_t batch, sd_trees out,
                              void *hip_stream) {
    if (!c) return SD_ERR_INVALID_ARG;
    if (batch < 0) return fail(c, SD_ERR_INVALID_ARG, "negative batch");
    if (batch > c->cfg.max_batch_slots)
        return fail(c, SD_ERR_CAPACITY, "batch exceeds max_batch_slots");
    if ((int64_t)batch * c->cfg.max_ctx_tokens * 8 > (int64_t)SD_STATIC_SCRATCH_BYTES)
        return fail(c, SD_ERR_CAPACITY,
                    "batch * max_ctx_tokens * 8 bytes exceeds SD_STATIC_SCRATCH_BYTES");
    if (batch == 0) return SD_OK;
    if (!trees_ok(out)) return fail(c, SD_ERR_INVALID_ARG, "null pointer");
    if (out.max_nodes < c->max_nodes)
        return fail(c, SD_ERR_INVALID_ARG, "trees.max_nodes below floor(alpha*P)");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    return sd_speculate_static_impl(c, d_slot_ids, batch, out, (hipStream_t)hip_stream);
}

sd_status sd_accept(sd_ctx *c, sd_trees trees, int32_t batch, const int32_t *d_target_tokens,
                    int32_t *d_accept_len, int32_t *d_accept_path, int32_t *d_bonus,
                    void *hip_stream) {
    if (!c) return SD_ERR_INVALID_ARG;
    if (batch < 0) return fail(c, SD_ERR_INVALID_ARG, "negative batch");
    if (batch > c->cfg.max_batch_slots)
        return fail(c, SD_ERR_CAPACITY, "batch exceeds max_batch_slots");
    if (batch == 0) return SD_OK;
    if (!trees.d_n_nodes || !trees.d_tokens || !trees.d_parents || trees.max_nodes < 1 ||
        !d_target_tokens || !d_accept_len || !d_accept_path || !d_bonus)
        return fail(c, SD_ERR_INVALID_ARG, "null pointer");
    if (trees.max_nodes > 256) return fail(c, SD_ERR_INVALID_ARG, "trees.max_nodes above 256");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    return sd_accept_impl(c, trees, batch, d_target_tokens, d_accept_len, d_accept_path, d_bonus,
                          (hipStream_t)hip_stream);
}

sd_status sd_accept_append(sd_ctx *c, sd_trees trees, const int32_t *d_slot_ids, int32_t batch,
                           const int32_t *d_target_tokens, int32_t *d_accept_len,
                           int32_t *d_accept_path, int32_t *d_bonus, void *hip_stream) {
    if (!c) return SD_ERR_INVALID_ARG;
    if (batch < 0) return fail(c, SD_ERR_INVALID_ARG, "negative batch");
    if (batch > c->cfg.max_batch_slots) return fail(c, SD_ERR_CAPACITY, "more slots than configured");
    if (batch == 0) return SD_OK;
    if (!trees.d_n_nodes || !trees.d_tokens || !trees.d_parents || trees.max_nodes < 1 ||
        !d_target_tokens || !d_accept_len || !d_accept_path || !d_bonus)
        return fail(c, SD_ERR_INVALID_ARG, "null pointer");
    if (trees.max_nodes > 256) return fail(c, SD_ERR_INVALID_ARG, "trees.max_nodes above 256");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    return sd_accept_append_impl(c, trees, d_slot_ids, batch, d_target_tokens, d_accept_len,
                                 d_accept_path, d_bonus, (hipStream_t)hip_stream);
}

sd_status sd_accept_append_speculate(sd_ctx *c, sd_trees trees, const int32_t *d_slot_ids,
                                     int32_t batch, const int32_t *d_target_tokens,
                                     int32_t *d_accept_len, int32_t *d_accept_path,
                                     int32_t *d_bonus, void *hip_stream) {
    if (!c) return SD_ERR_INVALID_ARG;
    if (batch < 0) return fail(c, SD_ERR_INVALID_ARG, "negative batch");
    if (batch > c->cfg.max_batch_slots) return fail(c, SD_ERR_CAPACITY, "more slots than configured");
    if (batch == 0) return SD_OK;
    if (!trees_ok(trees) || !d_target_tokens || !d_accept_len || !d_accept_path ||
        !d_bonus)
        return fail(c, SD_ERR_INVALID_ARG, "null pointer");
    if (trees.max_nodes < c->max_nodes)
        return fail(c, SD_ERR_INVALID_ARG, "trees.max_nodes below floor(alpha*P)");
    if (trees.max_nodes > 256) return fail(c, SD_ERR_INVALID_ARG, "trees.max_nodes above 256");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    return sd_accept_append_speculate_impl(c, trees, d_slot_ids, batch, d_target_tokens, d_accept_len,
                                           d_accept_path, d_bonus, (hipStream_t)hip_stream);
}

sd_status sd_get_stats(sd_ctx *c, sd_stats *o) {
    if (!c || !o) return SD_ERR_INVALID_ARG;
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    if (hipDeviceSynchronize() != hipSuccess) return fail(c, SD_ERR_HIP, "device synchronize failed");
    int32_t e[SD_DEVERR_N];
    if (hipMemcpy(e, c->d_err, sizeof(e), hipMemcpyDeviceToHost) != hipSuccess)
        return fail(c, SD_ERR_HIP, "hipMemcpy");
    o->global_tokens = c->g_tokens;
    o->global_docs = c->g_docs;
    o->err_bad_token = e[SD_DEVERR_TOKEN];
    o->err_bad_slot = e[SD_DEVERR_SLOT];
    o->err_ctx_overflow = e[SD_DEVERR_CTX];
    o->reserved = 0;
    o->index_bytes = c->index_bytes;
    o->scratch_bytes = c->scratch_bytes;
    const size_t rows = (size_t)c->cfg.max_batch_slots;
    unsigned long long *ctr = new (std::nothrow) unsigned long long[rows * SD_CTR_STRIDE];
    if (!ctr) return fail(c, SD_ERR_OOM, "host buffer for the counters");
    if (hipMemcpy(ctr, c->d_counters, rows * SD_CTR_STRIDE * sizeof(*ctr), hipMemcpyDeviceToHost) !=
        hipSuccess) {
        delete[] ctr;
        return fail(c, SD_ERR_HIP, "hipMemcpy");
    }
    int64_t *dst = &o->spec_requests;  // the counter fields follow each other in this order
    for (int i = 0; i < SD_CTR_N; i++) {
        dst[i] = 0;
        for (size_t r = 0; r < rows; r++) dst[i] += (int64_t)ctr[r * SD_CTR_STRIDE + i];
    }
    delete[] ctr;
    return SD_OK;
}

sd_status sd_debug_profile(sd_ctx *c, int32_t mode) {
    if (!c || mode < 0 || mode > 3) return SD_ERR_INVALID_ARG;
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    if (mode && !c->prof_ev) {
        c->prof_ev = new (std::nothrow) hipEvent_t[2 * SD_PROF_MAX_SPANS]();
        if (!c->prof_ev) return fail(c, SD_ERR_OOM, "event pool");
        for (int i = 0; i < 2 * SD_PROF_MAX_SPANS; i++)
            if (hipEventCreate(&c->prof_ev[i]) != hipSuccess) return fail(c, SD_ERR_HIP, "hipEventCreate");
    }
    c->prof_mode = mode;
    return SD_OK;
}

sd_status sd_debug_profile_read(sd_ctx *c, sd_profile *o) {
    if (!c || !o) return SD_ERR_INVALID_ARG;
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    if (hipDeviceSynchronize() != hipSuccess) return fail(c, SD_ERR_HIP, "device synchronize failed");
    for (int k = 0; k < SD_K_COUNT; k++) { o->launches[k] = 0; o->ms[k] = 0.0; o->algo_bytes[k] = 0; }
    for (int i = 0; i < c->prof_n; i++) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]) != hipSuccess)
            return fail(c, SD_ERR_HIP, "hipEventElapsedTime");
        o->launches[c->prof_kind[i]]++;
        o->ms[c->prof_kind[i]] += (double)ms;
    }
    c->prof_n = 0;
    unsigned long long ab[SD_K_COUNT];
    if (hipMemcpy(ab, c->d_algo_bytes, sizeof(ab), hipMemcpyDeviceToHost) != hipSuccess)
        return fail(c, SD_ERR_HIP, "hipMemcpy");
    for (int k = 0; k < SD_K_COUNT; k++) o->algo_bytes[k] = (int64_t)ab[k];
    if (hipMemset(c->d_algo_bytes, 0, sizeof(ab)) != hipSuccess) return fail(c, SD_ERR_HIP, "hipMemset");
    return SD_OK;
}

sd_status sd_debug_read_unit_ticks(sd_ctx *c, uint32_t *h_ticks, int64_t count, int32_t *khz) {
    if (!c || !h_ticks || !khz || count < 0) return SD_ERR_INVALID_ARG;
    if (count > (int64_t)c->tick_slots * 2 * c->cfg.P * 4)
        return fail(c, SD_ERR_CAPACITY, "more units than the tick buffers hold (SD_TICK_SLOTS requests)");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    if (hipDeviceSynchronize() != hipSuccess) return fail(c, SD_ERR_HIP, "device synchronize failed");
    int rate = 0;
    if (hipDeviceGetAttribute(&rate, hipDeviceAttributeWallClockRate, c->cfg.device) != hipSuccess)
        return fail(c, SD_ERR_HIP, "hipDeviceGetAttribute");
    *khz = rate;
    if (count && hipMemcpy(h_ticks, c->s_unit_ticks, (size_t)count * sizeof(uint32_t),
                           hipMemcpyDeviceToHost) != hipSuccess)
        return fail(c, SD_ERR_HIP, "hipMemcpy");
    return SD_OK;
}

sd_status sd_debug_read_request_ticks(sd_ctx *c, uint32_t *h_ticks, int32_t batch, int32_t *khz) {
    if (!c || !h_ticks || !khz || batch < 0) return SD_ERR_INVALID_ARG;
    if (batch > c->tick_slots)
        return fail(c, SD_ERR_CAPACITY, "more requests than the tick buffers hold (SD_TICK_SLOTS)");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    if (hipDeviceSynchronize() != hipSuccess) return fail(c, SD_ERR_HIP, "device synchronize failed");
    int rate = 0;
    if (hipDeviceGetAttribute(&rate, hipDeviceAttributeWallClockRate, c->cfg.device) != hipSuccess)
        return fail(c, SD_ERR_HIP, "hipDeviceGetAttribute");
    *khz = rate;
    const uint32_t *src = c->s_unit_ticks + (int64_t)c->tick_slots * 2 * c->cfg.P * 4;
    if (batch && hipMemcpy(h_ticks, src, (size_t)batch * 16 * 8 * sizeof(uint32_t),
                           hipMemcpyDeviceToHost) != hipSuccess)
        return fail(c, SD_ERR_HIP, "hipMemcpy");
    return SD_OK;
}

sd_status sd_debug_read_global(sd_ctx *c, int32_t *h_text, int32_t *h_sa, int64_t cap,
                               int64_t *n_positions) {
    if (!c || !n_positions) return SD_ERR_INVALID_ARG;
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, SD_ERR_HIP, "hipSetDevice");
    if (hipDeviceSynchronize() != hipSuccess) return fail(c, SD_ERR_HIP, "device synchronize failed");
    *n_positions = c->g_N;
    if (cap < c->g_N || !h_text || !h_sa) return fail(c, SD_ERR_CAPACITY, "host buffers too small");
    size_t bytes = (size_t)c->g_N * sizeof(int32_t);
    if (bytes && (hipMemcpy(h_text, c->g_text, bytes, hipMemcpyDeviceToHost) != hipSuccess ||
                  hipMemcpy(h_sa, c->g_sa, bytes, hipMemcpyDeviceToHost) != hipSuccess))
        return fail(c, SD_ERR_HIP, "hipMemcpy");
    return SD_OK;
}

}  // extern "C"
