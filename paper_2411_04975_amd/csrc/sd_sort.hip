// LSD radix sort of (uint64 key, uint32 value) pairs and the numbering of the groups of a
// sorted key array (a device-wide prefix maximum), both hand-written for 64-wide wavefronts.
// Used by the suffix-array construction in sd_build.hip.
//
// One pass = three launches: per-tile digit histogram (one LDS add per key into the wave's own
// counters), per-digit prefix sums along the tiles, stable scatter.  Inside a tile the stable
// rank of a key among keys with the same digit comes from wave-wide ballots (all lanes holding
// the same digit find each other with one ballot per digit bit).  The scatter first
// orders the tile by digit in LDS, so that global writes go out as runs of neighbouring lanes.
#include "sd_internal.h"

namespace {

constexpr int RS_THREADS = 256;
constexpr int RS_WAVES = RS_THREADS / SD_WAVE;
constexpr int RS_ITEMS = 16;
constexpr int RS_TILE = RS_THREADS * RS_ITEMS;  // keys per workgroup
constexpr int RS_BITS = 8;
constexpr int RS_BINS = 1 << RS_BITS;

__device__ __forceinline__ uint64_t lanemask_lt() {
    return (1ull << (threadIdx.x & 63)) - 1ull;
}

// lanes (among `valid` ones) whose digit equals this lane's digit
__device__ __forceinline__ uint64_t match_digit(uint32_t d, bool valid) {
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < RS_BITS; b++) {
        bool bit = (d >> b) & 1u;
        uint64_t m = __ballot(valid && bit);
        peers &= bit ? m : ~m;
    }
    return peers;
}

// exclusive prefix sum of one value per thread over a 256-thread workgroup
__device__ __forceinline__ uint32_t block_excl_scan_256(uint32_t v, uint32_t *s_wave /*[RS_WAVES]*/,
                                                        uint32_t *total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    if (lane == 63) s_wave[w] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < RS_WAVES; i++) {
        uint32_t t = s_wave[i];
        if (i < w) base += t;
        tot += t;
    }
    __syncthreads();
    if (total) *total = tot;
    return base + inc - v;
}

__global__ __launch_bounds__(RS_THREADS) void k_radix_hist(const uint64_t *__restrict__ keys,
                                                           int64_t n, int shift,
                                                           uint32_t *__restrict__ tile_hist,
                                                           int64_t ntiles,
                                                           const int32_t *__restrict__ run_if) {
    __shared__ uint32_t s_cnt[RS_WAVES][RS_BINS];
    if (run_if && *run_if == 0) return;  // same for the whole grid: the pass is not needed
    const int tid = threadIdx.x, w = tid >> 6;
    for (int i = tid; i < RS_WAVES * RS_BINS; i += RS_THREADS) (&s_cnt[0][0])[i] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * RS_TILE;
    // all loads of the tile first, then one LDS add per key into the wave's own counters (the
    // counts need no order, unlike the ranks of the scatter)
    uint64_t key[RS_ITEMS];
#pragma unroll
    for (int k = 0; k < RS_ITEMS; k++) {
        int64_t idx = base + (int64_t)k * RS_THREADS + tid;
        key[k] = idx < n ? keys[idx] : 0ull;
    }
#pragma unroll
    for (int k = 0; k < RS_ITEMS; k++) {
        int64_t idx = base + (int64_t)k * RS_THREADS + tid;
        if (idx < n) atomicAdd(&s_cnt[w][(uint32_t)((key[k] >> shift) & (RS_BINS - 1))], 1u);
    }
    __syncthreads();
    uint32_t tot = 0;
#pragma unroll
    for (int i = 0; i < RS_WAVES; i++) tot += s_cnt[i][tid];
    tile_hist[(int64_t)tid * ntiles + blockIdx.x] = tot;
}

// One workgroup per digit: exclusive prefix sum along the digit's row of the (digit, tile)
// table, in place, and the row total.  The scatter adds the prefix over digit totals itself
// (256 values), so a pass needs no device-wide scan.
__global__ __launch_bounds__(RS_THREADS) void k_radix_rowscan(uint32_t *__restrict__ tile_hist,
                                                              int64_t ntiles,
                                                              uint32_t *__restrict__ row_total,
                                                              const int32_t *__restrict__ run_if) {
    __shared__ uint32_t s_wave[RS_WAVES];
    __shared__ uint32_t s_carry;
    if (run_if && *run_if == 0) return;
    uint32_t *row = tile_hist + (int64_t)blockIdx.x * ntiles;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    constexpr int PER = 8;
    for (int64_t base = 0; base < ntiles; base += RS_THREADS * PER) {
        const int64_t i0 = base + (int64_t)threadIdx.x * PER;
        uint32_t v[PER], sum = 0;
#pragma unroll
        for (int k = 0; k < PER; k++) {
            v[k] = i0 + k < ntiles ? row[i0 + k] : 0u;
            sum += v[k];
        }
        uint32_t tot;
        uint32_t ex = block_excl_scan_256(sum, s_wave, &tot) + s_carry;
#pragma unroll
        for (int k = 0; k < PER; k++) {
            if (i0 + k < ntiles) row[i0 + k] = ex;
            ex += v[k];
        }
        __syncthreads();
        if (threadIdx.x == 0) s_carry += tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) row_total[blockIdx.x] = s_carry;
}

__global__ __launch_bounds__(RS_THREADS) void k_radix_scatter(
    const uint64_t *__restrict__ kin, const uint32_t *__restrict__ vin, uint64_t *__restrict__ kout,
    uint32_t *__restrict__ vout, int64_t n, int shift, const uint32_t *__restrict__ row_excl,
    const uint32_t *__restrict__ row_total, int64_t ntiles, const int32_t *__restrict__ run_if) {
    // 52 KB of LDS, so that three workgroups share a compute unit (with 54 KB two did): the
    // per-wave digit counts are 16-bit (a tile has 4096 keys), and the block scans' partial
    // sums sit where the keys go afterwards
    __shared__ uint64_t s_keys[RS_TILE];
    __shared__ uint32_t s_vals[RS_TILE];
    __shared__ volatile uint16_t s_wcnt[RS_WAVES][RS_BINS];
    __shared__ uint32_t s_excl[RS_BINS];
    __shared__ uint32_t s_gbase[RS_BINS];
    uint32_t *s_wave = reinterpret_cast<uint32_t *>(s_keys);  // (the keys arrive later)
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (run_if && *run_if == 0) return;
    for (int i = tid; i < RS_WAVES * RS_BINS; i += RS_THREADS) (&s_wcnt[0][0])[i] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * RS_TILE;
    const int cnt = (int)((n - base) < RS_TILE ? (n - base) : RS_TILE);
    static_assert(RS_TILE <= 65535, "16-bit digit counts");
    const uint64_t lt = lanemask_lt();

    uint64_t key[RS_ITEMS];
    uint32_t val[RS_ITEMS];
    uint32_t rnk[RS_ITEMS];
    // wave w owns keys [w*1024, (w+1)*1024) of the tile, item k of lane l is key k*64 + l of
    // that range: the stable order is (wave, item, lane).
#pragma unroll
    for (int k = 0; k < RS_ITEMS; k++) {
        int j = w * (RS_ITEMS * 64) + k * 64 + lane;
        bool valid = j < cnt;
        key[k] = valid ? kin[base + j] : 0ull;
        val[k] = valid ? vin[base + j] : 0u;
    }
#pragma unroll
    for (int k = 0; k < RS_ITEMS; k++) {
        int j = w * (RS_ITEMS * 64) + k * 64 + lane;
        bool valid = j < cnt;
        uint32_t d = (uint32_t)((key[k] >> shift) & (RS_BINS - 1));
        uint64_t peers = match_digit(d, valid);
        uint32_t pre = s_wcnt[w][d];
        uint32_t below = (uint32_t)__popcll(peers & lt);
        if (valid && below == 0) s_wcnt[w][d] = (uint16_t)(pre + (uint32_t)__popcll(peers));
        rnk[k] = pre + below;
    }
    __syncthreads();
    {
        const int d = tid;
        uint32_t acc = 0;
#pragma unroll
        for (int i = 0; i < RS_WAVES; i++) {
            uint32_t c = s_wcnt[i][d];
            s_wcnt[i][d] = (uint16_t)acc;  // keys of digit d held by earlier waves of this tile
            acc += c;
        }
        uint32_t ex = block_excl_scan_256(acc, s_wave, nullptr);
        s_excl[d] = ex;
        // keys with a smaller digit anywhere + keys with this digit in earlier tiles
        uint32_t digit_base = block_excl_scan_256(row_total[d], s_wave, nullptr);
        s_gbase[d] = digit_base + row_excl[(int64_t)d * ntiles + blockIdx.x];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < RS_ITEMS; k++) {
        int j = w * (RS_ITEMS * 64) + k * 64 + lane;
        if (j < cnt) {
            uint32_t d = (uint32_t)((key[k] >> shift) & (RS_BINS - 1));
            uint32_t pos = s_excl[d] + s_wcnt[w][d] + rnk[k];
            s_keys[pos] = key[k];
            s_vals[pos] = val[k];
        }
    }
    __syncthreads();
#pragma unroll 4
    for (int k = 0; k < RS_ITEMS; k++) {
        int j = k * RS_THREADS + tid;
        if (j < cnt) {
            uint64_t kk = s_keys[j];
            uint32_t d = (uint32_t)((kk >> shift) & (RS_BINS - 1));
            uint32_t out = s_gbase[d] + ((uint32_t)j - s_excl[d]);
            kout[out] = kk;
            vout[out] = s_vals[j];
        }
    }
}

// ---- tiles of the device-wide scans ------------------------------------------------------
constexpr int SC_THREADS = 256;
constexpr int SC_ITEMS = 16;
constexpr int SC_TILE = SC_THREADS * SC_ITEMS;

// exclusive prefix maximum of one value per thread over a 256-thread workgroup
__device__ __forceinline__ uint32_t block_excl_scanmax_256(uint32_t v, uint32_t *s_wave /*[RS_WAVES]*/,
                                                           uint32_t *total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t t = __shfl_up(inc, o);
        if (lane >= o) inc = t > inc ? t : inc;
    }
    uint32_t ex = __shfl_up(inc, 1);
    if (lane == 0) ex = 0;
    if (lane == 63) s_wave[w] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < RS_WAVES; i++) {
        uint32_t t = s_wave[i];
        if (i < w) base = t > base ? t : base;
        tot = t > tot ? t : tot;
    }
    __syncthreads();
    if (total) *total = tot;
    return base > ex ? base : ex;
}

// single workgroup: partials[i] <- maximum of partials[0..i) (exclusive, 0 for i = 0), any length
__global__ __launch_bounds__(SC_THREADS) void k_scanmax_partials(uint32_t *partials, int64_t m,
                                                                 const int32_t *__restrict__ run_if) {
    __shared__ uint32_t s_wave[SC_THREADS / 64];
    __shared__ uint32_t s_carry;
    if (run_if && *run_if == 0) return;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < m; base += SC_THREADS) {
        int64_t i = base + threadIdx.x;
        uint32_t v = i < m ? partials[i] : 0u;
        uint32_t tot;
        uint32_t ex = block_excl_scanmax_256(v, s_wave, &tot);
        uint32_t carry = s_carry;
        if (i < m) partials[i] = carry > ex ? carry : ex;
        __syncthreads();
        if (threadIdx.x == 0) s_carry = carry > tot ? carry : tot;
        __syncthreads();
    }
}

// ---- group numbers of a sorted key array, written by position -------------------------------
// A group (a run of equal keys) is numbered by where it starts: gid[i] = 1 + index of the first
// entry of i's group (0 stays free for "beyond the end"), and rank[vals[i]] = gid[i].  Numbers of
// that kind keep the order of the groups, and they change only for the entries that a split
// moves out of the front part of their group: given the numbers the places had before
// (gid_old; places keep their group from round to round, the build only reorders inside
// groups), only those entries are written to `rank` (by position: a random 4-byte store each).  Two passes over the keys: the last group start of every
// tile, a prefix maximum over the tiles, then numbers and stores.
__global__ __launch_bounds__(SC_THREADS) void k_rank_tile_last(const uint64_t *__restrict__ keys,
                                                               int64_t n,
                                                               uint32_t *__restrict__ partials,
                                                               const int32_t *__restrict__ run_if) {
    __shared__ uint32_t s_wave[SC_THREADS / 64];
    if (run_if && *run_if == 0) return;
    const int64_t base = (int64_t)blockIdx.x * SC_TILE;
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < SC_ITEMS; k++) {
        int64_t i = base + (int64_t)k * SC_THREADS + threadIdx.x;
        if (i < n && (i == 0 || keys[i] != keys[i - 1])) s = (uint32_t)(i + 1) > s ? (uint32_t)(i + 1) : s;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t t = __shfl_xor(s, o);
        s = t > s ? t : s;
    }
    if ((threadIdx.x & 63) == 0) s_wave[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int i = 0; i < SC_THREADS / 64; i++) t = s_wave[i] > t ? s_wave[i] : t;
        partials[blockIdx.x] = t;
    }
}

// (Entry k * SC_THREADS + t of the tile belongs to thread t: every load and store of a wave
// covers neighbouring words.  With SC_ITEMS consecutive entries per thread each load
// instruction touched 64 lines, and the kernel took 311 us for 10M entries, most of it for
// that and not for the scatter.)
__global__ __launch_bounds__(SC_THREADS) void k_rank_apply(const uint64_t *__restrict__ keys,
                                                           const uint32_t *__restrict__ vals,
                                                           int64_t n,
                                                           const uint32_t *__restrict__ partials,
                                                           uint32_t *__restrict__ rank,
                                                           uint32_t *__restrict__ gid,
                                                           const uint32_t *__restrict__ gid_old,
                                                           const int32_t *__restrict__ run_if) {
    constexpr int NW = SC_THREADS / 64;
    static_assert(SC_ITEMS * NW == 64, "one wave scans the parts of a tile");
    __shared__ uint64_t s_edge[SC_ITEMS][NW];  // key of the last lane of (row k, wave w)
    __shared__ uint32_t s_tot[SC_ITEMS * NW];  // group starts: maximum over (row k, wave w), then
                                               // over everything before it in the tile
    if (run_if && *run_if == 0) return;
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int64_t base = (int64_t)blockIdx.x * SC_TILE;
    uint64_t key[SC_ITEMS];
#pragma unroll
    for (int k = 0; k < SC_ITEMS; k++) {
        const int64_t i = base + (int64_t)k * SC_THREADS + t;
        key[k] = i < n ? keys[i] : 0ull;
    }
    const uint64_t before_tile = base > 0 ? keys[base - 1] : 0ull;
#pragma unroll
    for (int k = 0; k < SC_ITEMS; k++)
        if (lane == 63) s_edge[k][w] = key[k];
    __syncthreads();
    uint32_t inc[SC_ITEMS];  // running maximum of the group starts inside (row k, wave w)
#pragma unroll
    for (int k = 0; k < SC_ITEMS; k++) {
        const int64_t i = base + (int64_t)k * SC_THREADS + t;
        uint64_t prev = __shfl_up(key[k], 1);
        if (lane == 0) prev = w > 0 ? s_edge[k][w - 1] : (k > 0 ? s_edge[k > 0 ? k - 1 : 0][NW - 1] : before_tile);
        uint32_t v = i < n && (i == 0 || key[k] != prev) ? (uint32_t)(i + 1) : 0u;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t u = __shfl_up(v, o);
            if (lane >= o) v = u > v ? u : v;
        }
        inc[k] = v;
        if (lane == 63) s_tot[k * NW + w] = v;
    }
    __syncthreads();
    if (t < 64) {  // exclusive running maximum over the SC_ITEMS * NW = 64 parts, in array order
        uint32_t v = s_tot[t];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t u = __shfl_up(v, o);
            if (lane >= o) v = u > v ? u : v;
        }
        uint32_t ex = __shfl_up(v, 1);
        if (lane == 0) ex = 0;
        const uint32_t before = partials[blockIdx.x];
        s_tot[t] = before > ex ? before : ex;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < SC_ITEMS; k++) {
        const int64_t i = base + (int64_t)k * SC_THREADS + t;
        const uint32_t carry = s_tot[k * NW + w];
        const uint32_t g = inc[k] > carry ? inc[k] : carry;
        if (i < n) {
            if (!gid_old || gid_old[i] != g) rank[vals[i]] = g;
            gid[i] = g;
        }
    }
}

}  // namespace

void sd_group_ranks(sd_ctx *c, const uint64_t *keys, const uint32_t *vals, int64_t n,
                    uint32_t *rank, uint32_t *gid, const uint32_t *gid_old, hipStream_t st,
                    const int32_t *run_if) {
    if (n <= 0) return;
    int64_t nt = (n + SC_TILE - 1) / SC_TILE;
    sd_span sp(c, run_if ? SD_K_BUILD_OTHER : SD_K_SORT_SCAN, st);
    hipLaunchKernelGGL(k_rank_tile_last, dim3((unsigned)nt), dim3(SC_THREADS), 0, st, keys, n,
                       c->b_partials, run_if);
    hipLaunchKernelGGL(k_scanmax_partials, dim3(1), dim3(SC_THREADS), 0, st, c->b_partials, nt, run_if);
    hipLaunchKernelGGL(k_rank_apply, dim3((unsigned)nt), dim3(SC_THREADS), 0, st, keys, vals, n,
                       c->b_partials, rank, gid, gid_old, run_if);
}


// (Passes that a device-side switch may turn into no-ops are timed under "other build kernels",
// so that the sort kernels' own figures hold real passes only.)
int sd_sort_pairs(sd_ctx *c, int64_t n, int nbits, int in_idx, hipStream_t st, const int32_t *run_if) {
    int cur = in_idx;
    if (n <= 0) return cur;
    int64_t ntiles = (n + RS_TILE - 1) / RS_TILE;
    for (int shift = 0; shift < nbits; shift += RS_BITS) {
        {
            sd_span sp(c, run_if ? SD_K_BUILD_OTHER : SD_K_SORT_HIST, st);
            hipLaunchKernelGGL(k_radix_hist, dim3((unsigned)ntiles), dim3(RS_THREADS), 0, st,
                               c->b_keys[cur], n, shift, c->b_hist, ntiles, run_if);
        }
        {
            sd_span sp(c, run_if ? SD_K_BUILD_OTHER : SD_K_SORT_SCAN, st);
            hipLaunchKernelGGL(k_radix_rowscan, dim3(RS_BINS), dim3(RS_THREADS), 0, st, c->b_hist,
                               ntiles, c->b_hist + (int64_t)RS_BINS * ntiles, run_if);
        }
        {
            sd_span sp(c, run_if ? SD_K_BUILD_OTHER : SD_K_SORT_SCATTER, st);
            hipLaunchKernelGGL(k_radix_scatter, dim3((unsigned)ntiles), dim3(RS_THREADS), 0, st,
                               c->b_keys[cur], c->b_vals[cur], c->b_keys[cur ^ 1],
                               c->b_vals[cur ^ 1], n, shift, c->b_hist,
                               c->b_hist + (int64_t)RS_BINS * ntiles, ntiles, run_if);
        }
        cur ^= 1;
    }
    return cur;
}
