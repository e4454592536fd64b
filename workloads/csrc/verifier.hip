// Synthetic serving-loop glue for benchmarks and tests: a simulated greedy target model and
// the collection of accepted tokens.  This is workload code, not part of the draft-generation
// library: it plays the role of the LLM verifier (Section 4.1, "Simulated Ablations": a
// drafted token is accepted iff it equals the ground-truth response token at that position).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// target[b][0] = future[b][pos[b]]; target[b][1+j] = future[b][pos[b] + depth(j)], where
// depth(j) is the number of draft nodes on the path from the tree root to node j (>= 1).
// With `advance` given, pos[b] first moves on by advance[b] + 1 (the tokens the previous step
// produced: its accepted draft tokens and the bonus token; -1 = nothing yet).
__global__ __launch_bounds__(64) void k_targets(const int32_t *__restrict__ n_nodes,
                                                const int32_t *__restrict__ parents, int max_nodes,
                                                const int32_t *__restrict__ future,
                                                int64_t future_stride, int32_t *__restrict__ pos,
                                                const int32_t *__restrict__ advance,
                                                int32_t *__restrict__ target) {
    __shared__ int32_t s_anc[256], s_dep[256];
    const int b = blockIdx.x, lane = threadIdx.x;
    const int32_t *par = parents + (int64_t)b * max_nodes;
    // everything that does not depend on another load is asked for at once
    int n = n_nodes[b];
    const int32_t pos0 = pos[b], adv = advance ? advance[b] + 1 : 0;
    const int32_t mypar = lane < max_nodes ? par[lane] : -1;
    if (n > 256) n = 256;
    const int32_t p0 = pos0 + adv;
    if (advance && lane == 0) pos[b] = p0;
    const int32_t *fut = future + (int64_t)b * future_stride + p0;
    int32_t *tgt = target + (int64_t)b * (max_nodes + 1);
    const int32_t f0 = fut[0];
    if (n <= 64) {
        // one node per lane: depth by pointer jumping over the parent links (a link must lead
        // to a lower index), links and depths in registers, log2(depth) rounds
        int32_t anc = (lane < n && mypar >= 0 && mypar < lane) ? mypar : -1, dep = lane < n ? 1 : 0;
        for (int round = 0; round < 6; round++) {
            if (!__ballot(anc >= 0)) break;
            const int src = anc >= 0 ? anc : lane;
            const int32_t da = __shfl(dep, src), aa = __shfl(anc, src);
            if (anc >= 0) { dep += da; anc = aa; }
        }
        const int32_t v = lane < n ? fut[dep] : f0;
        if (lane == 0) tgt[0] = f0;
        if (lane < max_nodes) tgt[1 + lane] = v;
        for (int j = 64 + lane; j < max_nodes; j += 64) tgt[1 + j] = f0;
        return;
    }
    // depth of every node by pointer jumping over the parent links (a link must lead to a
    // lower index): log2(depth) rounds instead of a walk of `depth` dependent steps
    for (int j = lane; j < n; j += 64) {
        const int32_t a = par[j];
        s_anc[j] = (a >= 0 && a < j) ? a : -1;
        s_dep[j] = 1;
    }
    __syncthreads();
    for (int round = 0; round < 8; round++) {
        int32_t nd[4], na[4];
        bool open = false;
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const int j = lane + 64 * r;
            nd[r] = 0; na[r] = -1;
            if (j < n) {
                const int32_t a = s_anc[j];
                nd[r] = s_dep[j];
                if (a >= 0) {
                    nd[r] += s_dep[a];
                    na[r] = s_anc[a];
                    open = true;
                }
            }
        }
        if (!__ballot(open)) break;
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const int j = lane + 64 * r;
            if (j < n) { s_dep[j] = nd[r]; s_anc[j] = na[r]; }
        }
        __syncthreads();
    }
    if (lane == 0) tgt[0] = f0;
    for (int j = lane; j < max_nodes; j += 64) tgt[1 + j] = j < n ? fut[s_dep[j]] : f0;
}

// one wavefront per request: new_offsets[b] = sum over earlier requests of (accept_len + 1);
// the new tokens of request b are its accepted draft tokens followed by the bonus token;
// pos[b] += accept_len[b] + 1.
__global__ __launch_bounds__(64) void k_collect(const int32_t *__restrict__ tokens, int max_nodes,
                                                const int32_t *__restrict__ accept_len,
                                                const int32_t *__restrict__ accept_path,
                                                const int32_t *__restrict__ bonus, int batch,
                                                int32_t *__restrict__ new_tokens,
                                                int32_t *__restrict__ new_offsets,
                                                int32_t *__restrict__ pos) {
    const int b = blockIdx.x, lane = threadIdx.x;
    int off = 0;
    for (int i = lane; i < b; i += 64) off += accept_len[i] + 1;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) off += __shfl_xor(off, o);
    const int L = accept_len[b];
    int32_t *dst = new_tokens + off;
    for (int i = lane; i < L; i += 64)
        dst[i] = tokens[(int64_t)b * max_nodes + accept_path[(int64_t)b * max_nodes + i]];
    if (lane == 0) {
        dst[L] = bonus[b];
        new_offsets[b] = off;
        pos[b] += L + 1;
        if (b == batch - 1) new_offsets[batch] = off + L + 1;
    }
}

// Plain streaming copy, 16 bytes per lane per trip, grid-stride: the reference rate that
// bandwidth figures of the other kernels are set against (and the known-size kernel that
// hardware byte counters are calibrated on).
__global__ __launch_bounds__(256) void k_stream_copy(const int4 *__restrict__ src,
                                                     int4 *__restrict__ dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        dst[i] = src[i];
}

// Dependent loads, one after the other, by a single lane: next[i] names the entry to read
// after entry i (entries 32 words apart: one memory line each).  The time per hop is the latency
// of a load whose address comes from the load before it, from whatever level of the memory
// system holds a working set of that size: the cost unit of the drafting kernel's probe chains.
__global__ __launch_bounds__(64) void k_chase(const uint32_t *__restrict__ next, uint32_t start,
                                              int hops, uint32_t *__restrict__ out) {
    if (threadIdx.x != 0) return;
    uint32_t i = start;
    for (int h = 0; h < hops; h++) i = __builtin_nontemporal_load(next + (size_t)i * 32);
    out[0] = i;
}

}  // namespace

extern "C" {

// follows d_next (uint32, one entry per 32 words, values are entry numbers) for `hops` loads
// from entry `start` on one lane; *d_out receives the last entry reached
int wl_chase(const void *d_next, uint32_t start, int hops, void *d_out, void *stream) {
    if (hops <= 0) return 0;
    hipLaunchKernelGGL(k_chase, dim3(1), dim3(64), 0, (hipStream_t)stream, (const uint32_t *)d_next,
                       start, hops, (uint32_t *)d_out);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// copies n_bytes (a multiple of 16, both pointers 16-byte aligned) from d_src to d_dst
int wl_stream_copy(const void *d_src, void *d_dst, int64_t n_bytes, void *stream) {
    if (n_bytes <= 0) return 0;
    if (n_bytes % 16 || ((uintptr_t)d_src & 15) || ((uintptr_t)d_dst & 15)) return 2;
    const int64_t n16 = n_bytes / 16;
    int64_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;  // 32 workgroups per compute unit, grid-stride
    hipLaunchKernelGGL(k_stream_copy, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const int4 *)d_src, (int4 *)d_dst, n16);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// all pointers are device pointers
int wl_targets(const int32_t *d_n_nodes, const int32_t *d_parents, int max_nodes,
               const int32_t *d_future, int64_t future_stride, int32_t *d_pos,
               const int32_t *d_advance, int batch, int32_t *d_target, void *stream) {
    if (batch <= 0) return 0;
    hipLaunchKernelGGL(k_targets, dim3((unsigned)batch), dim3(64), 0, (hipStream_t)stream, d_n_nodes,
                       d_parents, max_nodes, d_future, future_stride, d_pos, d_advance, d_target);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int wl_collect(const int32_t *d_tokens, int max_nodes, const int32_t *d_accept_len,
               const int32_t *d_accept_path, const int32_t *d_bonus, int batch,
               int32_t *d_new_tokens, int32_t *d_new_offsets, int32_t *d_pos, void *stream) {
    if (batch <= 0) return 0;
    hipLaunchKernelGGL(k_collect, dim3((unsigned)batch), dim3(64), 0, (hipStream_t)stream, d_tokens, max_nodes,
                       d_accept_len, d_accept_path, d_bonus, batch, d_new_tokens, d_new_offsets,
                       d_pos);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // extern "C"
