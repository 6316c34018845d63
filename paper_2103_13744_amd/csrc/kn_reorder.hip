// Physical re-ordering of a batch of points by network (Sec. 3.5: the inputs are ordered so that the inputs of one
// network are consecutive in memory) for kn_eval_grouped.
//
// The points arrive in the caller's order.  Sorting indices alone leaves the grouped-MLP kernel with one random
// 12-byte gather per position and per direction and one scattered write per result; here the sample itself
// travels: two 16-byte halves, (x, y, z, key) and (dx, dy, dz, caller index), each in an array of its own, are moved
// by a stable least-significant-digit radix sort of at most two passes (keys are below 2^16), after which the
// kernel reads its samples with two contiguous 16-byte loads per lane.
//
// A pass's scatter does not store a record where its rank says: 64 lanes would write to some 40 different runs, one
// memory transaction each, and the pass would run at the rate of a random scatter.  The block first brings its
// records into sorted order in LDS, one half at a time; then consecutive lanes write consecutive addresses, a few
// runs per store instruction.
//
// One pass = (digit, block) count table -> per-digit exclusive scan over the blocks -> stable scatter of the records.
// The table of the first pass is counted by the kernel that computes the cell ids (Eq. 6); the first scatter also
// leaves the keys alone in their new order (4 bytes each), from which the table of the second pass is counted.
// (Counting it with one atomic per record from inside the first scatter was tried: 4 M device atomics on a 130 KB
// table take longer than both scatters together.)  Inside a block, stability comes from ranking each 64-record row
// of a wavefront with ballot-built peer masks and wave-private counters, as in the index sort.
// Bucket offsets, counts and the kernel's tile list are then found by a 16-way search over the sorted keys, one
// 16-lane group per network.
//
// Results: a random 16-byte store costs one memory transaction, an unaligned 12-byte one several, so the MLP kernel
// writes (r, g, b, sigma) as one 16-byte store at the sample's caller index into a staging array, and a streaming
// kernel splits that array into the caller's sigma and rgb arrays.
#include "kn_common.h"

namespace {

constexpr int RO_THREADS = 256;
constexpr int RO_WAVES = RO_THREADS / KN_WAVE; // 4
constexpr int RO_ROWS = 16;                    // 64-record rows per wavefront
constexpr int RO_TILE = RO_THREADS * RO_ROWS;  // 4096 records per block

typedef uint32_t u4 __attribute__((ext_vector_type(4)));

// Eq. 6 for RO_TILE points per block: ids (optional), sort keys (network id, N = outside), and the block's count of
// each value of the keys' lowest digit.  Also clears `zero` (the counter that a later kernel of the call adds to) and
// writes the (zero) results of the points that have no network into the staging array of the results.
__global__ void __launch_bounds__(RO_THREADS)
    k_keys_hist(const float *__restrict__ pts, int64_t M, KnGrid g, const int32_t *__restrict__ cell_net, int32_t *__restrict__ ids,
                int32_t *__restrict__ keys, int32_t N, uint32_t digit_mask, int32_t nblk, int32_t *__restrict__ table,
                int32_t *__restrict__ zero, int64_t n_zero, float *__restrict__ out4)
{
    __shared__ int32_t hist[256];
    for (int64_t i = (int64_t)blockIdx.x * RO_THREADS + threadIdx.x; i < n_zero; i += (int64_t)gridDim.x * RO_THREADS) zero[i] = 0;
    hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * RO_TILE + threadIdx.x;
    float p[RO_ROWS][3];
#pragma unroll
    for (int r = 0; r < RO_ROWS; ++r) {
        const int64_t i = min(base + r * RO_THREADS, M - 1);
#pragma unroll
        for (int c = 0; c < 3; ++c) p[r][c] = pts[3 * i + c];
    }
#pragma unroll
    for (int r = 0; r < RO_ROWS; ++r) {
        const int64_t i = base + r * RO_THREADS;
        if (i < M) {
            const int32_t id = kn_net_of_cell(cell_net, kn_grid_index(g, p[r][0], p[r][1], p[r][2]));
            const int32_t key = id < 0 ? N : id;
            if (ids) ids[i] = id;
            keys[i] = key;
            if (id < 0) *(float4 *)(out4 + 4 * i) = make_float4(0.0f, 0.0f, 0.0f, 0.0f); // no network: the result is zero
            atomicAdd(&hist[(uint32_t)key & digit_mask], 1);
        }
    }
    __syncthreads();
    if (threadIdx.x <= digit_mask) table[(int64_t)threadIdx.x * nblk + blockIdx.x] = hist[threadIdx.x];
}

// Row d of the (digit, block) table -> exclusive prefix along the blocks (in place), totals[d] = the row's sum.
// One workgroup per digit.
__global__ void __launch_bounds__(RO_THREADS) k_digit_scan(int32_t *__restrict__ table, int32_t nblk, int32_t *__restrict__ totals)
{
    __shared__ int32_t lds[16];
    int32_t *row = table + (int64_t)blockIdx.x * nblk;
    int32_t carry = 0;
    for (int32_t base = 0; base < nblk; base += RO_THREADS * 4) {
        const int32_t i0 = base + threadIdx.x * 4;
        int32_t v[4], s = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[k] = i0 + k < nblk ? row[i0 + k] : 0;
            s += v[k];
        }
        int32_t tot;
        int32_t run = carry + kn_block_exclusive_scan(s, lds, tot);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i0 + k < nblk) row[i0 + k] = run;
            run += v[k];
        }
        carry += tot;
    }
    if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}

// (digit, block) counts of a later pass, from the keys in the order the pass before left them
__global__ void __launch_bounds__(RO_THREADS)
    k_key_hist(const int32_t *__restrict__ keys, int64_t M, int shift, uint32_t mask, int32_t nblk, int32_t *__restrict__ table)
{
    __shared__ int32_t hist[256];
    hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * RO_TILE + 4 * (int64_t)threadIdx.x;
#pragma unroll
    for (int r = 0; r < RO_ROWS / 4; ++r) {
        const int64_t i = base + r * (4 * RO_THREADS);
        if (i + 3 < M) {
            const int4 k = *(const int4 *)(keys + i);
            atomicAdd(&hist[((uint32_t)k.x >> shift) & mask], 1);
            atomicAdd(&hist[((uint32_t)k.y >> shift) & mask], 1);
            atomicAdd(&hist[((uint32_t)k.z >> shift) & mask], 1);
            atomicAdd(&hist[((uint32_t)k.w >> shift) & mask], 1);
        } else {
            for (int64_t j = i; j < M && j < i + 4; ++j) atomicAdd(&hist[((uint32_t)keys[j] >> shift) & mask], 1);
        }
    }
    __syncthreads();
    if (threadIdx.x <= mask) table[(int64_t)threadIdx.x * nblk + blockIdx.x] = hist[threadIdx.x];
}

// Stable scatter of one radix pass.  Wavefront w of block b owns records [b*RO_TILE + w*RO_ROWS*64, +RO_ROWS*64) as rows
// of 64; order of records = (block, wave, row, lane).  `keys`: the keys in the order of the input.
//   FROM_REC false: the halves are formed here from the caller's arrays (points, dirs), caller index = position.
//   keys_out (nullable): the keys alone in the new order; perm_out (nullable): the caller indices in the new order.
// Dynamic LDS: RO_TILE * 16 bytes (the staging buffer of one half).
template <bool FROM_REC>
__global__ void __launch_bounds__(RO_THREADS)
    k_reorder_scatter(const int32_t *__restrict__ keys, const float *__restrict__ pts, const float *__restrict__ dirs,
                      const u4 *__restrict__ pin, const u4 *__restrict__ din, u4 *__restrict__ pout, u4 *__restrict__ dout,
                      int32_t *__restrict__ keys_out, int32_t *__restrict__ perm_out, int64_t M, int shift, int bits, int32_t nblk,
                      const int32_t *__restrict__ table_s, const int32_t *__restrict__ totals)
{
    constexpr int TILE = RO_TILE, ROWS = RO_ROWS;
    extern __shared__ u4 stage[]; // TILE halves in the block's sorted order
    __shared__ int32_t cnt[RO_WAVES][256];
    __shared__ int32_t delta[256]; // digit d: (global position) - (position in the block's sorted order) of its records
    __shared__ int32_t scan_lds[16];
    const int lane = threadIdx.x & (KN_WAVE - 1), w = threadIdx.x / KN_WAVE;
    const uint32_t mask = (1u << bits) - 1u;
#pragma unroll
    for (int i = 0; i < RO_WAVES; ++i) cnt[i][threadIdx.x] = 0;
    // thread d: position of this block's first record with digit d = records with smaller digits + records with
    // this digit in earlier blocks
    int32_t digit_base;
    {
        const bool has = threadIdx.x <= mask;
        const int32_t total = has ? totals[threadIdx.x] : 0;
        const int32_t mine = has ? table_s[(int64_t)threadIdx.x * nblk + blockIdx.x] : 0;
        int32_t all;
        digit_base = kn_block_exclusive_scan(total, scan_lds, all) + mine; // (contains the barrier that orders the clearing above)
    }
    const int64_t bbase = (int64_t)blockIdx.x * TILE;
    const int64_t wbase = bbase + (int64_t)w * (ROWS * KN_WAVE);
    const int32_t n_here = (int32_t)min((int64_t)TILE, M - bbase); // records of this block (>= 1)
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    uint32_t key[ROWS];
    int32_t lpos[ROWS]; // rank among the wavefront's records of the same digit, then position in the block's sorted order
#pragma unroll
    for (int r = 0; r < ROWS; ++r) key[r] = (uint32_t)keys[min(wbase + r * KN_WAVE + lane, M - 1)];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const bool valid = wbase + r * KN_WAVE + lane < M;
        const uint32_t d = (key[r] >> shift) & mask;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            if (b < bits) { // uniform
                const bool bit = (d >> b) & 1u;
                const uint64_t m = __ballot(bit);
                peers &= bit ? m : ~m;
            }
        }
        int32_t prior = 0;
        if (valid) prior = cnt[w][d];
        __builtin_amdgcn_wave_barrier();
        const int n_peers = __popcll(peers);
        const bool leader = valid && (lane == 63 - __clzll(peers));
        if (leader) cnt[w][d] = prior + n_peers;
        __builtin_amdgcn_wave_barrier();
        lpos[r] = prior + __popcll(peers & lt_mask);
    }
    __syncthreads();
    {
        // thread d: where the digit's records start in the block's sorted order, and each wavefront's share of them
        const int d = threadIdx.x;
        int32_t c[RO_WAVES], sum = 0;
#pragma unroll
        for (int i = 0; i < RO_WAVES; ++i) {
            c[i] = cnt[i][d];
            sum += c[i];
        }
        int32_t all;
        int32_t run = kn_block_exclusive_scan(sum, scan_lds, all);
        delta[d] = digit_base - run;
#pragma unroll
        for (int i = 0; i < RO_WAVES; ++i) {
            cnt[i][d] = run;
            run += c[i];
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ROWS; ++r) lpos[r] += cnt[w][(key[r] >> shift) & mask];

    // first halves: (x, y, z, key)
    {
        u4 h[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const int64_t i = min(wbase + r * KN_WAVE + lane, M - 1);
            if constexpr (FROM_REC) {
                h[r] = pin[i];
            } else {
                const float *p = pts + 3 * i;
                h[r] = (u4){__float_as_uint(p[0]), __float_as_uint(p[1]), __float_as_uint(p[2]), key[r]};
            }
        }
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
            if (wbase + r * KN_WAVE + lane < M) stage[lpos[r]] = h[r];
    }
    __syncthreads();
    int32_t dst[ROWS];
#pragma unroll
    for (int k = 0; k < ROWS; ++k) {
        const int32_t sp = k * RO_THREADS + threadIdx.x; // position in the block's sorted order
        if (sp < n_here) {
            const u4 v = stage[sp];
            dst[k] = sp + delta[(v[3] >> shift) & mask];
            pout[dst[k]] = v;
            if (keys_out) keys_out[dst[k]] = (int32_t)v[3];
        }
    }
    __syncthreads();
    // second halves: (dx, dy, dz, caller index)
    {
        u4 h[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const int64_t i = min(wbase + r * KN_WAVE + lane, M - 1);
            if constexpr (FROM_REC) {
                h[r] = din[i];
            } else {
                const float *q = dirs + 3 * i;
                h[r] = (u4){__float_as_uint(q[0]), __float_as_uint(q[1]), __float_as_uint(q[2]), (uint32_t)i};
            }
        }
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
            if (wbase + r * KN_WAVE + lane < M) stage[lpos[r]] = h[r];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < ROWS; ++k) {
        const int32_t sp = k * RO_THREADS + threadIdx.x;
        if (sp < n_here) {
            const u4 v = stage[sp];
            dout[dst[k]] = v;
            if (perm_out) perm_out[dst[k]] = (int32_t)v[3];
        }
    }
}

// Bucket offsets, counts and the tile list of the grouped MLP from the sorted keys (word 3 of each first half).
// One 16-lane group per network n = 0 .. N (N: the points without a network) finds offsets[n] and offsets[n+1] (the
// number of records whose key is below n, n+1) by a 16-way search, two searches at a time; counts[n] is their
// difference, and the group writes the network's tiles (chunks of at most tile_len records) into slots that its
// wavefront takes from the zeroed counter n_tiles with one atomic (the order of tiles is free: nothing observable
// depends on it).  offsets has N + 2 entries; the group of n = N writes the last two.
__global__ void __launch_bounds__(256)
    k_offsets_tiles(const u4 *__restrict__ rec, int64_t M, int32_t N, int32_t tile_len, int32_t *__restrict__ offsets,
                    int32_t *__restrict__ counts, int32_t *__restrict__ user_counts, KnTile *__restrict__ tiles, int32_t *__restrict__ n_tiles)
{
    const int lane = threadIdx.x & (KN_WAVE - 1), t = lane & 15, sub = lane >> 4;
    const int32_t n = (blockIdx.x * blockDim.x + threadIdx.x) >> 4;
    const bool mine = n <= N;
    const uint32_t *key_of = (const uint32_t *)rec + 3;
    // two lower bounds per group: lb[0] for n, lb[1] for n + 1; each interval [lo, hi] holds its answer
    int64_t lo[2] = {0, 0}, hi[2] = {mine ? M : 0, mine ? M : 0};
    while (__any(hi[0] > lo[0] || hi[1] > lo[1])) { // each round cuts an interval to a seventeenth; uniform in the wavefront
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const uint32_t bound = (uint32_t)(n + q);
            const int64_t len = hi[q] - lo[q];
            bool below = false;
            if (len <= 16) {
                const int64_t pos = lo[q] + t;
                if (pos < hi[q]) below = key_of[4 * pos] < bound;
            } else {
                const int64_t pos = lo[q] + (int64_t)(t + 1) * len / 17; // strictly inside, increasing in t, distinct (len > 16)
                below = key_of[4 * pos] < bound;
            }
            const int c = __popcll((__ballot(below) >> (16 * sub)) & 0xffffull); // keys are sorted: lanes 0 .. c-1
            if (len <= 16) {
                lo[q] = hi[q] = lo[q] + c;
            } else {
                const int64_t p_below = lo[q] + (int64_t)c * len / 17;       // probe c-1 (if c > 0): the last one below
                const int64_t p_above = lo[q] + (int64_t)(c + 1) * len / 17; // probe c (if c < 16): the first one not below
                if (c < 16) hi[q] = p_above;
                if (c > 0) lo[q] = p_below + 1;
            }
        }
    }
    const int32_t first = (int32_t)lo[0], count = (int32_t)(lo[1] - lo[0]);
    if (mine && t == 0) {
        offsets[n] = first;
        if (n == N) offsets[N + 1] = (int32_t)lo[1]; // = M
        counts[n] = count;
        if (user_counts) user_counts[n] = count;
    }
    // tiles: bucket N (no network) gets none
    const int32_t n_mine = (mine && n < N) ? (count + tile_len - 1) / tile_len : 0;
    int32_t before = 0, wave_total = 0; // tiles of the groups in front of mine in the wavefront
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int32_t v = __shfl(n_mine, 16 * g, KN_WAVE);
        if (g < sub) before += v;
        wave_total += v;
    }
    int32_t base = 0;
    if (lane == 0 && wave_total > 0) base = atomicAdd(n_tiles, wave_total);
    base = __shfl(base, 0, KN_WAVE) + before;
    for (int32_t k = t; k < n_mine; k += 16) {
        KnTile tl;
        tl.net = n;
        tl.start = first + k * tile_len;
        tl.len = min(tile_len, count - k * tile_len);
        tl.pad = 0;
        tiles[base + k] = tl;
    }
}

// staging array (r, g, b, sigma per point, caller order) -> the caller's sigma and rgb arrays; 4 points per thread
__global__ void __launch_bounds__(256) k_split_results(const float *__restrict__ out4, int64_t M, float *__restrict__ sigma, float *__restrict__ rgb)
{
    const int64_t i = 4 * ((int64_t)blockIdx.x * blockDim.x + threadIdx.x);
    if (i >= M) return;
    if (i + 3 < M && (((uintptr_t)sigma | (uintptr_t)rgb) & 15) == 0) {
        float4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = *(const float4 *)(out4 + 4 * (i + k));
        *(float4 *)(sigma + i) = make_float4(v[0].w, v[1].w, v[2].w, v[3].w);
        float4 *c = (float4 *)(rgb + 3 * i);
        c[0] = make_float4(v[0].x, v[0].y, v[0].z, v[1].x);
        c[1] = make_float4(v[1].y, v[1].z, v[2].x, v[2].y);
        c[2] = make_float4(v[2].z, v[3].x, v[3].y, v[3].z);
    } else {
        for (int64_t j = i; j < M && j < i + 4; ++j) {
            const float4 v = *(const float4 *)(out4 + 4 * j);
            sigma[j] = v.w;
            rgb[3 * j] = v.x;
            rgb[3 * j + 1] = v.y;
            rgb[3 * j + 2] = v.z;
        }
    }
}

struct ReorderWs {
    int32_t *keys, *keys_b, *table, *totals, *n_tiles, *counts, *offsets;
    u4 *pos_a, *dir_a, *pos_b, *dir_b; // the two halves of the records, before and after the second pass
    float *out4;
    KnTile *tiles;
    int64_t nblk;
};

int key_bits(int32_t N)
{
    int bits = 1;
    while ((1ll << bits) < (int64_t)N + 1) ++bits;
    return bits;
}

void carve_reorder(KnCarver &c, int64_t M, int32_t N, ReorderWs &w)
{
    w.nblk = kn_div_up(M > 0 ? M : 1, RO_TILE);
    const bool two = key_bits(N) > 8;
    w.n_tiles = c.carve<int32_t>(1);
    w.table = c.carve<int32_t>(256 * w.nblk);
    w.totals = c.carve<int32_t>(256);
    w.keys = c.carve<int32_t>(M);
    w.keys_b = two ? c.carve<int32_t>(M) : nullptr;
    w.counts = c.carve<int32_t>(N + 1);
    w.offsets = c.carve<int32_t>(N + 2);
    w.tiles = c.carve<KnTile>(kn_max_tiles(M, N, 64));
    w.pos_a = c.carve<u4>(M);
    w.dir_a = c.carve<u4>(M);
    w.pos_b = two ? c.carve<u4>(M) : nullptr;
    w.dir_b = two ? c.carve<u4>(M) : nullptr;
    w.out4 = c.carve<float>(4 * M);
}

} // namespace

int64_t kn_reorder_ws_bytes(int64_t M, int32_t N)
{
    KnCarver c((void *)256, INT64_MAX / 2);
    ReorderWs w;
    carve_reorder(c, M, N, w);
    return c.used;
}

int kn_reorder_run(const kn_scene *sc, hipStream_t st, const float *points, const float *dirs, int64_t M, int32_t tile_len,
                   int32_t *user_ids, int32_t *user_counts, int32_t *user_perm, KnCarver &ws, KnBucketOut *out,
                   const uint32_t *records[2], float **out4, KnStageTimer *tm)
{
    const int32_t N = sc->N;
    if (M < 1 || M > (1ll << 30) || N < 1 || N > 65535 || tile_len < 64) return KN_E_INVALID_ARG;
    ReorderWs w;
    carve_reorder(ws, M, N, w);
    if (!ws.ok()) return KN_E_WORKSPACE;
    const int bits = key_bits(N); // <= 16
    const bool two = bits > 8;
    const int bits0 = two ? bits / 2 : bits, bits1 = bits - bits0; // (the last pass takes the larger digit: N itself is a key)
    const int32_t nblk = (int32_t)w.nblk;
    const dim3 grid((unsigned)nblk), block(RO_THREADS);

    hipLaunchKernelGGL(k_keys_hist, grid, block, 0, st, points, M, sc->net_grid, sc->cell_net, user_ids, w.keys, N, (1u << bits0) - 1u,
                       nblk, w.table, w.n_tiles, (int64_t)1, w.out4);
    KN_CHECK_LAUNCH();
    if (tm) tm->mark(KN_ST_CELL);
    hipLaunchKernelGGL(k_digit_scan, dim3(1u << bits0), block, 0, st, w.table, nblk, w.totals);
    KN_CHECK_LAUNCH();
    const u4 *sorted_pos = w.pos_a, *sorted_dir = w.dir_a;
    constexpr size_t stage_bytes = (size_t)RO_TILE * sizeof(u4);
    hipLaunchKernelGGL((k_reorder_scatter<false>), grid, block, stage_bytes, st, w.keys, points, dirs, (const u4 *)nullptr,
                       (const u4 *)nullptr, w.pos_a, w.dir_a, w.keys_b, two ? (int32_t *)nullptr : user_perm, M, 0, bits0, nblk, w.table,
                       w.totals);
    KN_CHECK_LAUNCH();
    if (two) {
        hipLaunchKernelGGL(k_key_hist, grid, block, 0, st, w.keys_b, M, bits0, (1u << bits1) - 1u, nblk, w.table);
        KN_CHECK_LAUNCH();
        hipLaunchKernelGGL(k_digit_scan, dim3(1u << bits1), block, 0, st, w.table, nblk, w.totals);
        KN_CHECK_LAUNCH();
        hipLaunchKernelGGL((k_reorder_scatter<true>), grid, block, stage_bytes, st, w.keys_b, (const float *)nullptr,
                           (const float *)nullptr, w.pos_a, w.dir_a, w.pos_b, w.dir_b, (int32_t *)nullptr, user_perm, M, bits0, bits1,
                           nblk, w.table, w.totals);
        KN_CHECK_LAUNCH();
        sorted_pos = w.pos_b;
        sorted_dir = w.dir_b;
    }
    hipLaunchKernelGGL(k_offsets_tiles, dim3((unsigned)kn_div_up(((int64_t)N + 1) * 16, 256)), dim3(256), 0, st, sorted_pos, M, N, tile_len,
                       w.offsets, w.counts, user_counts, w.tiles, w.n_tiles);
    KN_CHECK_LAUNCH();
    out->perm = nullptr; // the records are the sorted list
    out->counts = w.counts;
    out->offsets = w.offsets;
    out->tiles = w.tiles;
    out->n_tiles = w.n_tiles;
    records[0] = (const uint32_t *)sorted_pos;
    records[1] = (const uint32_t *)sorted_dir;
    *out4 = w.out4;
    return KN_OK;
}

int kn_reorder_split_results(hipStream_t st, const float *out4, int64_t M, float *sigma, float *rgb)
{
    hipLaunchKernelGGL(k_split_results, dim3((unsigned)kn_div_up(kn_div_up(M, 4), 256)), dim3(256), 0, st, out4, M, sigma, rgb);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

// the scatter's staging buffer is above the default limit of dynamic LDS (once per device, from kn_create)
int kn_reorder_configure()
{
    const int bytes = (int)(RO_TILE * sizeof(u4));
    KN_HIP(hipFuncSetAttribute((const void *)k_reorder_scatter<false>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    KN_HIP(hipFuncSetAttribute((const void *)k_reorder_scatter<true>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    return KN_OK;
}
