// Point -> cell assignment (Eq. 6) and stable bucketing of samples by network id (Sec. 3.5:
// inputs are ordered so that consecutive inputs belong to the same network).
//
// Bucketing is a least-significant-digit radix sort on 8-bit digits of the key (network id, with
// N standing for "outside"), each pass = per-block digit histogram -> exclusive scan of the
// (digit, block) table -> stable scatter.  Inside a block, stability comes from ranking each
// 64-element row of a wavefront with ballot-built peer masks and wave-private LDS counters.
// Bucket counts and the tile list of the grouped MLP are then read off the sorted keys.
#include "kn_common.h"

namespace {

// The number of keys is either known on the host, or (render waves) only on the device; in the
// second case the host passes an upper bound for grid sizing and a pointer to the real count.
__device__ __forceinline__ int64_t real_count(int64_t m_bound, const int32_t *m_dev)
{
    return m_dev ? (int64_t)*m_dev : m_bound;
}

constexpr int RS_THREADS = 256;
#ifndef KN_RS_ROWS
#define KN_RS_ROWS 16
#endif
constexpr int RS_ROWS = KN_RS_ROWS;               // 64-element rows per wavefront
constexpr int RS_WAVES = RS_THREADS / KN_WAVE;    // 4
constexpr int RS_TILE = RS_THREADS * RS_ROWS;     // 4096 keys per block
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

// ---------------------------------------------------------------------------------------------
__global__ void k_fill_i32(int32_t *p, int64_t n, int32_t v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void k_cell_ids(const float *__restrict__ pts, int64_t M, KnGrid g, const int32_t *__restrict__ cell_net,
                           int32_t *__restrict__ ids, int32_t *__restrict__ keys, int32_t N, int32_t *__restrict__ zero,
                           int64_t n_zero)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_zero) zero[i] = 0; // scratch counters of the sort that follows
    if (i >= M) return;
    float x = pts[3 * i], y = pts[3 * i + 1], z = pts[3 * i + 2];
    int32_t id = kn_net_of_cell(cell_net, kn_grid_index(g, x, y, z)); // Eq. 6, then the table of a sparse grid
    if (ids) ids[i] = id;
    if (keys) keys[i] = id < 0 ? N : id;
}

__global__ void k_ids_to_keys(const int32_t *__restrict__ ids, int64_t M, int32_t N, int32_t *__restrict__ keys)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    int32_t id = ids[i];
    keys[i] = (id < 0 || id > N) ? N : id;
}

// ---------------------------------------------------------------------------------------------
// block-wide exclusive scan helper (256 threads), returns the exclusive prefix of v and the total
__device__ __forceinline__ int32_t block_exclusive_scan(int32_t v, int32_t *lds /*RS_WAVES+1*/, int32_t &total)
{
    const int lane = threadIdx.x & (KN_WAVE - 1), w = threadIdx.x / KN_WAVE;
    int32_t inc = v;
#pragma unroll
    for (int d = 1; d < KN_WAVE; d <<= 1) {
        int32_t o = __shfl_up(inc, d, KN_WAVE);
        if (lane >= d) inc += o;
    }
    __syncthreads(); // protects lds reuse between consecutive calls
    if (lane == KN_WAVE - 1) lds[w] = inc;
    __syncthreads();
    int32_t wbase = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < SCAN_THREADS / KN_WAVE; ++i) {
        int32_t s = lds[i];
        if (i < w) wbase += s;
        tot += s;
    }
    total = tot;
    return wbase + inc - v;
}

__global__ void __launch_bounds__(SCAN_THREADS) k_scan_sums(const int32_t *__restrict__ in, int64_t n,
                                                            int32_t *__restrict__ sums)
{
    __shared__ int32_t lds[8];
    int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    int32_t s = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i)
        if (base + i < n) s += in[base + i];
    int32_t total;
    block_exclusive_scan(s, lds, total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ void __launch_bounds__(SCAN_THREADS) k_scan_apply(const int32_t *__restrict__ in, int32_t *__restrict__ out,
                                                             int64_t n, const int32_t *__restrict__ sums,
                                                             int32_t n_sums, int32_t *__restrict__ total_out)
{
    __shared__ int32_t lds[8];
    // prefix of the block sums in front of this block (and the grand total for block 0)
    int32_t before = 0, all = 0;
    for (int32_t i = threadIdx.x; i < n_sums; i += SCAN_THREADS) {
        int32_t s = sums[i];
        all += s;
        if (i < (int32_t)blockIdx.x) before += s;
    }
    int32_t tot_before, tot_all;
    block_exclusive_scan(before, lds, tot_before);
    block_exclusive_scan(all, lds, tot_all);
    if (blockIdx.x == 0 && threadIdx.x == 0 && total_out) *total_out = tot_all;

    int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    int32_t v[SCAN_ITEMS], s = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        v[i] = (base + i < n) ? in[base + i] : 0;
        s += v[i];
    }
    int32_t dummy;
    int32_t run = tot_before + block_exclusive_scan(s, lds, dummy);
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        if (base + i < n) out[base + i] = run;
        run += v[i];
    }
}

// ---------------------------------------------------------------------------------------------
// radix pass, step 1: digit histogram of each 4096-key block -> table[digit * n_blocks + block].
// With `grp` given, the block also adds its counts to per-digit sums over groups of GRP_BLOCKS
// blocks (integer atomics: the sums do not depend on arrival order), from which the scatter kernel
// derives its own base offsets without a separate scan of the table.  Counters that many blocks
// hit share few cache lines, and same-line atomics serialise, so nothing finer is accumulated.
constexpr int GRP_BLOCKS = 32;
__global__ void __launch_bounds__(RS_THREADS) k_radix_hist(const int32_t *__restrict__ keys, int64_t M_bound,
                                                           const int32_t *__restrict__ M_dev, int shift,
                                                           int32_t n_blocks, int32_t *__restrict__ table,
                                                           int32_t *__restrict__ grp, int32_t n_grp)
{
    __shared__ int32_t hist[256];
    const int64_t M = real_count(M_bound, M_dev);
    int64_t base = (int64_t)blockIdx.x * RS_TILE;
    if (grp && base >= M) return; // nobody reads this block's table column in that mode
    hist[threadIdx.x] = 0;
    __syncthreads();
    int32_t kv[RS_ROWS];
#pragma unroll
    for (int r = 0; r < RS_ROWS; ++r) {
        const int64_t i = base + (int64_t)r * RS_THREADS + threadIdx.x;
        kv[r] = (i < M) ? keys[i] : -1;
    }
#pragma unroll
    for (int r = 0; r < RS_ROWS; ++r)
        if (kv[r] >= 0) atomicAdd(&hist[((uint32_t)kv[r] >> shift) & 255u], 1);
    __syncthreads();
    const int32_t h = hist[threadIdx.x];
    table[(int64_t)threadIdx.x * n_blocks + blockIdx.x] = h;
    if (grp && h) atomicAdd(&grp[(int64_t)threadIdx.x * n_grp + blockIdx.x / GRP_BLOCKS], h);
}

// radix pass, step 3: stable scatter.  Wavefront w of block b owns keys
// [b*4096 + w*1024, +1024) as 16 rows of 64; order of keys = (block, wave, row, lane).
__global__ void __launch_bounds__(RS_THREADS)
    k_radix_scatter(const int32_t *__restrict__ keys_in, const int32_t *__restrict__ vals_in,
                    int32_t *__restrict__ keys_out, int32_t *__restrict__ vals_out, int64_t M_bound,
                    const int32_t *__restrict__ M_dev, int shift, int32_t n_blocks,
                    const int32_t *__restrict__ table /*scanned if grp == nullptr, raw counts otherwise*/,
                    const int32_t *__restrict__ grp, int32_t n_grp)
{
    __shared__ int32_t cnt[RS_WAVES][256];
    __shared__ int32_t scan_lds[8];
    const int64_t M = real_count(M_bound, M_dev);
    if ((int64_t)blockIdx.x * RS_TILE >= M) return;
    const int lane = threadIdx.x & (KN_WAVE - 1), w = threadIdx.x / KN_WAVE;
#pragma unroll
    for (int i = 0; i < RS_WAVES; ++i) cnt[i][threadIdx.x] = 0;
    // thread d: global position of this block's first key with digit d (loads issued before the ranking
    // loop so that their latency overlaps with it)
    int32_t digit_base;
    {
        const int d = threadIdx.x;
        if (grp) {
            // keys with smaller digits + same digit in earlier groups + same digit earlier in my group
            const int g = blockIdx.x / GRP_BLOCKS;
            const int g_used = (int)((M + (int64_t)RS_TILE * GRP_BLOCKS - 1) / ((int64_t)RS_TILE * GRP_BLOCKS));
            int32_t total = 0, before = 0;
            // fixed-size batches of independent loads: a loop with a data-dependent trip count would pay one
            // memory round trip per element
            const int32_t *gp = grp + (int64_t)d * n_grp;
            for (int g0 = 0; g0 < g_used; g0 += 16) {
                int32_t v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = gp[min(g0 + u, n_grp - 1)]; // unconditional loads batch up
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = (g0 + u < g_used) ? v[u] : 0;
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    total += v[u];
                    if (g0 + u < g) before += v[u];
                }
            }
            {
                const int32_t *tp = table + (int64_t)d * n_blocks + g * GRP_BLOCKS;
                const int in_grp = (int)blockIdx.x - g * GRP_BLOCKS;
                int32_t v[GRP_BLOCKS];
#pragma unroll
                for (int u = 0; u < GRP_BLOCKS; ++u) v[u] = tp[min(u, max(in_grp - 1, 0))];
#pragma unroll
                for (int u = 0; u < GRP_BLOCKS; ++u) v[u] = (u < in_grp) ? v[u] : 0;
#pragma unroll
                for (int u = 0; u < GRP_BLOCKS; ++u) before += v[u];
            }
            int32_t all;
            digit_base = block_exclusive_scan(total, scan_lds, all) + before;
        } else {
            digit_base = table[(int64_t)d * n_blocks + blockIdx.x];
        }
    }
    __syncthreads();

    const int64_t wbase = (int64_t)blockIdx.x * RS_TILE + (int64_t)w * (RS_ROWS * KN_WAVE);
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int32_t key[RS_ROWS], rank[RS_ROWS], val[RS_ROWS];

    // all loads first: the ranking loop below contains scheduling barriers that loads cannot cross
#pragma unroll
    for (int r = 0; r < RS_ROWS; ++r) {
        const int64_t i = min(wbase + r * KN_WAVE + lane, M - 1);
        key[r] = keys_in[i];
        val[r] = vals_in ? vals_in[i] : (int32_t)i;
    }
#pragma unroll
    for (int r = 0; r < RS_ROWS; ++r) {
        const int64_t i = wbase + r * KN_WAVE + lane;
        const bool valid = i < M;
        const uint32_t d = ((uint32_t)key[r] >> shift) & 255u;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (d >> b) & 1u;
            const uint64_t m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        int32_t prior = 0;
        if (valid) prior = cnt[w][d];
        __builtin_amdgcn_wave_barrier();
        const int n_peers = __popcll(peers);
        const bool leader = valid && (lane == 63 - __clzll(peers));
        if (leader) cnt[w][d] = prior + n_peers;
        __builtin_amdgcn_wave_barrier();
        rank[r] = prior + __popcll(peers & lt_mask);
    }
    __syncthreads();
    {
        // thread d: per-wave digit counts -> global positions of each wave's first key with digit d
        const int d = threadIdx.x;
        int32_t run = digit_base;
#pragma unroll
        for (int i = 0; i < RS_WAVES; ++i) {
            int32_t c = cnt[i][d];
            cnt[i][d] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RS_ROWS; ++r) {
        const int64_t i = wbase + r * KN_WAVE + lane;
        if (i < M) {
            const uint32_t d = ((uint32_t)key[r] >> shift) & 255u;
            const int32_t dst = cnt[w][d] + rank[r];
            if (keys_out) keys_out[dst] = key[r];
            vals_out[dst] = val[r];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// offsets[n] = first position of bucket n in the sorted list, for all n in [0, N+1] (offsets[N+1] = M).
// Each boundary of the sorted keys defines the offsets of every bucket between the two keys (empty
// buckets included), so each entry is written exactly once; runs of empty buckets are filled by
// the whole wavefront together.
__global__ void __launch_bounds__(256)
    k_bucket_offsets(const int32_t *__restrict__ sorted_keys, int64_t M_bound, const int32_t *__restrict__ M_dev, int32_t N,
                     int32_t *__restrict__ offsets, int32_t *__restrict__ user_offsets)
{
    const int64_t M = real_count(M_bound, M_dev);
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & (KN_WAVE - 1);
    if (M == 0) {
        if (blockIdx.x == 0)
            for (int32_t n = threadIdx.x; n <= N + 1; n += blockDim.x) {
                offsets[n] = 0;
                if (user_offsets) user_offsets[n] = 0;
            }
        return;
    }
    if ((int64_t)blockIdx.x * blockDim.x >= M) return;
    const bool valid = i < M;
    const int32_t k = valid ? sorted_keys[i] : 0;
    const int32_t prev = (!valid || i == 0) ? -1 : sorted_keys[i - 1];
    const bool boundary = valid && k != prev;
    if (boundary) {
        offsets[k] = (int32_t)i;
        if (user_offsets) user_offsets[k] = (int32_t)i;
    }
    // empty buckets prev+1 .. k-1 take the same offset; after the last key everything up to N+1 takes M
    const bool last = valid && i == M - 1;
    unsigned long long gaps = __ballot(boundary && k - prev > 1);
    while (gaps) {
        const int src = __ffsll((long long)gaps) - 1;
        gaps &= gaps - 1;
        const int32_t lo = __shfl(prev, src, KN_WAVE) + 1, hi = __shfl(k, src, KN_WAVE);
        const int32_t val = (int32_t)__shfl((int)i, src, KN_WAVE);
        for (int32_t n = lo + lane; n < hi; n += KN_WAVE) {
            offsets[n] = val;
            if (user_offsets) user_offsets[n] = val;
        }
    }
    const unsigned long long tail = __ballot(last);
    if (tail) {
        const int src = __ffsll((long long)tail) - 1;
        const int32_t lo = __shfl(k, src, KN_WAVE) + 1;
        for (int32_t n = lo + lane; n <= N + 1; n += KN_WAVE) {
            offsets[n] = (int32_t)M;
            if (user_offsets) user_offsets[n] = (int32_t)M;
        }
    }
}

// counts and the tile list of the grouped MLP, one thread per bucket.  Tile slots are handed out
// with one atomic per wavefront (the order of tiles is free; nothing observable depends on it).
__global__ void __launch_bounds__(256)
    k_bucket_tiles(const int32_t *__restrict__ offsets, int32_t N, int32_t tile_len, int32_t *__restrict__ counts,
                   int32_t *__restrict__ user_counts, KnTile *__restrict__ tiles, int32_t *__restrict__ n_tiles)
{
    const int32_t n = blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & (KN_WAVE - 1);
    int32_t a = 0, c = 0;
    if (n <= N) {
        a = offsets[n];
        c = offsets[n + 1] - a;
        counts[n] = c;
        if (user_counts) user_counts[n] = c;
    }
    const int32_t mine = (n < N) ? (c + tile_len - 1) / tile_len : 0; // bucket N (outside / unused) gets none
    int32_t inc = mine;
#pragma unroll
    for (int d = 1; d < KN_WAVE; d <<= 1) {
        const int32_t o = __shfl_up(inc, d, KN_WAVE);
        if (lane >= d) inc += o;
    }
    const int32_t wave_total = __shfl(inc, KN_WAVE - 1, KN_WAVE);
    int32_t base = 0;
    if (lane == 0 && wave_total > 0) base = atomicAdd(n_tiles, wave_total);
    base = __shfl(base, 0, KN_WAVE) + inc - mine;
    for (int32_t t = 0; t < mine; ++t) {
        KnTile tl;
        tl.net = n;
        tl.start = a + t * tile_len;
        tl.len = min(tile_len, c - t * tile_len);
        tl.pad = 0;
        tiles[base + t] = tl;
    }
}

int launch_1d(int64_t n, int threads, dim3 &grid)
{
    int64_t blocks = kn_div_up(n, threads);
    if (blocks > 0x7fffffffLL) return KN_E_UNSUPPORTED;
    grid = dim3((unsigned)blocks);
    return KN_OK;
}

} // namespace

// ---------------------------------------------------------------------------------------------
int kn_fill_i32(hipStream_t st, int32_t *p, int64_t n, int32_t v)
{
    if (n <= 0) return KN_OK;
    dim3 grid;
    KN_TRY(launch_1d(n, 256, grid));
    hipLaunchKernelGGL(k_fill_i32, grid, dim3(256), 0, st, p, n, v);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

int64_t kn_scan_tmp_len(int64_t n) { return kn_div_up(n > 0 ? n : 1, SCAN_TILE); }

int kn_exclusive_scan_i32(hipStream_t st, const int32_t *in, int32_t *out, int64_t n, int32_t *tmp, int32_t *total)
{
    if (n <= 0) {
        if (total) KN_TRY(kn_fill_i32(st, total, 1, 0));
        return KN_OK;
    }
    int64_t nb = kn_div_up(n, SCAN_TILE);
    if (nb > (1 << 24)) return KN_E_UNSUPPORTED;
    hipLaunchKernelGGL(k_scan_sums, dim3((unsigned)nb), dim3(SCAN_THREADS), 0, st, in, n, tmp);
    KN_CHECK_LAUNCH();
    hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)nb), dim3(SCAN_THREADS), 0, st, in, out, n, tmp, (int32_t)nb, total);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

static int radix_passes(int32_t N)
{
    int bits = 1;
    while ((1ll << bits) < (int64_t)N + 1) ++bits;
    return (bits + 7) / 8;
}

int64_t kn_max_tiles(int64_t M, int32_t N, int32_t tile_len)
{
    return M / tile_len + (M < N ? M : N) + 1;
}


struct BucketWs {
    int32_t *keys_a, *keys_b, *vals_a, *vals_b, *table, *table_s, *scan_tmp, *atomics, *counts, *offsets, *n_tiles;
    KnTile *tiles;
    int64_t nblk, n_grp, n_atomics;
};

static void carve_bucket(KnCarver &c, int64_t M, int32_t N, BucketWs &w)
{
    w.nblk = kn_div_up(M > 0 ? M : 1, RS_TILE);
    w.n_grp = kn_div_up(w.nblk, GRP_BLOCKS);
    w.n_atomics = 4 * 256 * w.n_grp + 1; // per-digit group sums for up to 4 passes, then the tile counter
    w.keys_a = c.carve<int32_t>(M);
    w.keys_b = c.carve<int32_t>(M);
    w.vals_a = c.carve<int32_t>(M);
    w.vals_b = c.carve<int32_t>(M);
    w.table = c.carve<int32_t>(256 * w.nblk);
    w.table_s = c.carve<int32_t>(256 * w.nblk);
    w.scan_tmp = c.carve<int32_t>(kn_scan_tmp_len(256 * w.nblk));
    w.atomics = c.carve<int32_t>(w.n_atomics);
    w.counts = c.carve<int32_t>(N + 1);
    w.offsets = c.carve<int32_t>(N + 2);
    w.tiles = c.carve<KnTile>(kn_max_tiles(M, N, 64));
    w.n_tiles = w.atomics ? w.atomics + 4 * 256 * w.n_grp : nullptr;
}

int64_t kn_bucket_ws_bytes(int64_t M, int32_t N)
{
    KnCarver c((void *)256, INT64_MAX / 2);
    BucketWs w;
    carve_bucket(c, M, N, w);
    return c.used;
}

void kn_bucket_scratch(KnCarver ws, int64_t M, int32_t N, int32_t **atomics, int64_t *n_atomics)
{
    BucketWs w;
    carve_bucket(ws, M, N, w);
    *atomics = w.atomics;
    *n_atomics = w.n_atomics;
}

int kn_bucket_run(hipStream_t st, int32_t *keys, int64_t M, const int32_t *M_dev, int32_t N, int32_t tile_len,
                  int32_t *user_counts, int32_t *user_offsets, int32_t *user_perm, KnCarver &ws, KnBucketOut *out,
                  bool atomics_zeroed, int64_t self_base_blocks)
{
    if (M < 0 || M > (1ll << 30) || N < 1 || tile_len < 64) return KN_E_INVALID_ARG;
    BucketWs w;
    carve_bucket(ws, M, N, w);
    if (!ws.ok()) return KN_E_WORKSPACE;
    const int64_t nblk = w.nblk;
    // up to this many blocks the scatter derives its offsets from per-group sums; beyond, the (digit, block) table is scanned
    const bool self_base = nblk <= self_base_blocks;

    const int passes = radix_passes(N);
    const int32_t *kin = keys;
    const int32_t *vin = nullptr;
    int32_t *sorted_keys = w.keys_b;
    int32_t *perm = w.vals_b;
    if (!atomics_zeroed) KN_TRY(kn_fill_i32(st, w.atomics, w.n_atomics, 0));
    if (M > 0) {
        for (int p = 0; p < passes; ++p) {
            const bool last = (p == passes - 1);
            int32_t *kout = (p & 1) ? w.keys_a : w.keys_b;
            int32_t *vout = (p & 1) ? w.vals_a : w.vals_b;
            if (last && user_perm) vout = user_perm;
            int32_t *grp = self_base ? w.atomics + p * 256 * w.n_grp : nullptr;
            hipLaunchKernelGGL(k_radix_hist, dim3((unsigned)nblk), dim3(RS_THREADS), 0, st, kin, M, M_dev, 8 * p, (int32_t)nblk,
                               w.table, grp, (int32_t)w.n_grp);
            KN_CHECK_LAUNCH();
            const int32_t *tbl = w.table;
            if (!self_base) {
                KN_TRY(kn_exclusive_scan_i32(st, w.table, w.table_s, 256 * nblk, w.scan_tmp, nullptr));
                tbl = w.table_s;
            }
            hipLaunchKernelGGL(k_radix_scatter, dim3((unsigned)nblk), dim3(RS_THREADS), 0, st, kin, vin, kout, vout, M, M_dev,
                               8 * p, (int32_t)nblk, tbl, grp, (int32_t)w.n_grp);
            KN_CHECK_LAUNCH();
            kin = kout;
            vin = vout;
            sorted_keys = kout;
            perm = vout;
        }
    }
    {
        dim3 grid;
        KN_TRY(launch_1d(M > 0 ? M : 1, 256, grid));
        hipLaunchKernelGGL(k_bucket_offsets, grid, dim3(256), 0, st, sorted_keys, M, M_dev, N, w.offsets, user_offsets);
        KN_CHECK_LAUNCH();
        hipLaunchKernelGGL(k_bucket_tiles, dim3((unsigned)kn_div_up(N + 1, 256)), dim3(256), 0, st, w.offsets, N, tile_len,
                           w.counts, user_counts, w.tiles, w.n_tiles);
        KN_CHECK_LAUNCH();
    }
    out->perm = perm;
    out->counts = w.counts;
    out->offsets = w.offsets;
    out->tiles = w.tiles;
    out->n_tiles = w.n_tiles;
    return KN_OK;
}

// ---------------------------------------------------------------------------------------------
// C ABI: stage entry points of this file
extern "C" int kn_cell_ids(const kn_scene *sc, void *stream, const float *points, int64_t M, int32_t *ids)
{
    if (!sc || M < 0 || (M > 0 && (!points || !ids))) return KN_E_INVALID_ARG;
    if (M == 0) return KN_OK;
    dim3 grid;
    KN_TRY(launch_1d(M, 256, grid));
    hipLaunchKernelGGL(k_cell_ids, grid, dim3(256), 0, (hipStream_t)stream, points, M, sc->net_grid, sc->cell_net, ids,
                       (int32_t *)nullptr, sc->N, (int32_t *)nullptr, (int64_t)0);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

// used by kn_eval_grouped: ids (optional) and sort keys in one pass over the points
int kn_cell_keys(const kn_scene *sc, hipStream_t st, const float *points, int64_t M, int32_t *ids, int32_t *keys,
                 int32_t *zero, int64_t n_zero)
{
    if (M == 0 && n_zero == 0) return KN_OK;
    dim3 grid;
    KN_TRY(launch_1d(M > n_zero ? M : n_zero, 256, grid));
    hipLaunchKernelGGL(k_cell_ids, grid, dim3(256), 0, st, points, M, sc->net_grid, sc->cell_net, ids, keys, sc->N, zero,
                       n_zero);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

extern "C" int kn_bucket(kn_ctx *ctx, const kn_scene *sc, void *stream, const int32_t *ids, int64_t M, int32_t *counts,
                         int32_t *offsets, int32_t *perm, void *workspace, int64_t workspace_bytes)
{
    if (!ctx || !sc || M < 0 || (M > 0 && (!ids || !perm))) return KN_E_INVALID_ARG;
    if (M > (1ll << 30)) return KN_E_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < kn_bucket_ws_bytes(M, sc->N) + kn_align_up(M * 4, 256))
        return KN_E_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    KnCarver ws(workspace, workspace_bytes);
    int32_t *keys = ws.carve<int32_t>(M);
    if (M > 0) {
        dim3 grid;
        KN_TRY(launch_1d(M, 256, grid));
        hipLaunchKernelGGL(k_ids_to_keys, grid, dim3(256), 0, st, ids, M, sc->N, keys);
        KN_CHECK_LAUNCH();
    }
    KnBucketOut bo;
    return kn_bucket_run(st, keys, M, nullptr, sc->N, 64, counts, offsets, perm, ws, &bo, false, kn_knobs(ctx).radix_self_base_blocks);
}
