// Stable ordering of a batch by network (Sec. 3.5: the inputs are ordered so that the inputs of one network are
// consecutive in memory): a least-significant-digit radix sort of at most two passes (keys are below 2^16), in two forms.
//
// kn_reorder_run (kn_eval_grouped) moves the samples themselves.  The points arrive in the caller's order; sorting
// indices alone leaves the grouped-MLP kernel with one random 12-byte gather per position and per direction and
// one scattered write per result.  Here two 16-byte halves per sample, (x, y, z, key) and (dx, dy, dz, caller index),
// each in an array of its own, travel through the passes, after which the kernel reads its samples with two
// contiguous 16-byte loads per lane.
// kn_bucket_run (the stage call kn_bucket, the layer-at-a-time and the static-scratch evaluation) sorts (key, index)
// pairs and leaves the permutation.
//
// One pass = (digit, block) count table -> per-digit exclusive scan over the blocks -> stable scatter.  Inside a
// block, stability comes from ranking each 64-element row of a wavefront with ballot-built peer masks and
// wave-private counters: no atomics in the ordering path, so the order is the unique stable one.
// A scatter does not store an element where its rank says: 64 lanes would write to some 40 different runs, one
// memory transaction each, and the pass would run at the rate of a random scatter.  The block first brings its
// elements into sorted order in LDS; then consecutive lanes write consecutive addresses, a few runs per store
// instruction.
// The table of the first pass of kn_reorder_run is counted by the kernel that computes the cell ids (Eq. 6); every
// scatter also leaves the keys alone in their new order (4 bytes each), from which the table of the next pass is
// counted.  (Counting it with one atomic per record from inside the first scatter was tried: 4 M device atomics on
// a 130 KB table take longer than both scatters together.)
// Bucket offsets, counts and the kernel's tile list are then found by a 16-way search over the sorted keys, one
// 16-lane group per network.
//
// Results of kn_eval_grouped: a random 16-byte store costs one memory transaction, an unaligned 12-byte one several,
// so the MLP kernel writes (r, g, b, sigma) as one 16-byte store at the sample's caller index into a staging array,
// and a streaming kernel splits that array into the caller's sigma and rgb arrays.
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
    // one point: id, key, the zero result of a point without a network, the digit count
    auto point = [&](int64_t i, float x, float y, float z) -> int32_t {
        const int32_t id = kn_net_of_cell(cell_net, kn_grid_index(g, x, y, z));
        const int32_t key = id < 0 ? N : id;
        if (ids) ids[i] = id;
        if (id < 0) *(float4 *)(out4 + 4 * i) = make_float4(0.0f, 0.0f, 0.0f, 0.0f); // no network: the result is zero
        atomicAdd(&hist[(uint32_t)key & digit_mask], 1);
        return key;
    };
    const int64_t tile0 = (int64_t)blockIdx.x * RO_TILE;
    if (tile0 + RO_TILE <= M && ((uintptr_t)pts & 15) == 0) { // (uniform) a whole tile of a 16-byte aligned array
        // four consecutive points per thread and step: three 16-byte loads, one 16-byte store of the keys
#pragma unroll
        for (int r = 0; r < RO_ROWS / 4; ++r) {
            const int64_t i = tile0 + 4 * ((int64_t)r * RO_THREADS + threadIdx.x);
            const float4 a = *(const float4 *)(pts + 3 * i), b = *(const float4 *)(pts + 3 * i + 4), c = *(const float4 *)(pts + 3 * i + 8);
            int4 k;
            k.x = point(i, a.x, a.y, a.z);
            k.y = point(i + 1, a.w, b.x, b.y);
            k.z = point(i + 2, b.z, b.w, c.x);
            k.w = point(i + 3, c.y, c.z, c.w);
            *(int4 *)(keys + i) = k;
        }
    } else {
        const int64_t base = tile0 + threadIdx.x;
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
            if (i < M) keys[i] = point(i, p[r][0], p[r][1], p[r][2]);
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

// (digit, block) counts of a pass from the keys alone, in the order the pass reads them.  Also clears `zero`.
__global__ void __launch_bounds__(RO_THREADS)
    k_key_hist(const int32_t *__restrict__ keys, int64_t M, int shift, uint32_t mask, int32_t nblk, int32_t *__restrict__ table,
               int32_t *__restrict__ zero, int64_t n_zero)
{
    __shared__ int32_t hist[256];
    for (int64_t i = (int64_t)blockIdx.x * RO_THREADS + threadIdx.x; i < n_zero; i += (int64_t)gridDim.x * RO_THREADS) zero[i] = 0;
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

// Ranking step shared by the scatter kernels.  Wavefront w of block b owns elements [b*RO_TILE + w*RO_ROWS*64,
// +RO_ROWS*64) as rows of 64; order of elements = (block, wave, row, lane).  In: key[r] of the lane's element of row r
// (clamped loads beyond M).  Out: lpos[r], the element's position in the block's sorted order (digit, then input
// order), and delta[d] = (global position) - (position in the block's sorted order) for the elements of digit d.
// cnt and delta are LDS arrays of the caller; contains block barriers: every thread of the block calls it.
__device__ __forceinline__ void rank_block(const uint32_t (&key)[RO_ROWS], int32_t (&lpos)[RO_ROWS], int64_t M, int shift, int bits,
                                           int32_t nblk, const int32_t *__restrict__ table_s, const int32_t *__restrict__ totals,
                                           int32_t (*cnt)[256], int32_t *delta, int32_t *scan_lds)
{
    const int lane = threadIdx.x & (KN_WAVE - 1), w = threadIdx.x / KN_WAVE;
    const uint32_t mask = (1u << bits) - 1u;
#pragma unroll
    for (int i = 0; i < RO_WAVES; ++i) cnt[i][threadIdx.x] = 0;
    // thread d: position of this block's first element with digit d = elements with smaller digits + elements with
    // this digit in earlier blocks
    int32_t digit_base;
    {
        const bool has = threadIdx.x <= mask;
        const int32_t total = has ? totals[threadIdx.x] : 0;
        const int32_t mine = has ? table_s[(int64_t)threadIdx.x * nblk + blockIdx.x] : 0;
        int32_t all;
        digit_base = kn_block_exclusive_scan(total, scan_lds, all) + mine; // (contains the barrier that orders the clearing above)
    }
    const int64_t wbase = (int64_t)blockIdx.x * RO_TILE + (int64_t)w * (RO_ROWS * KN_WAVE);
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int r = 0; r < RO_ROWS; ++r) {
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
        lpos[r] = prior + __popcll(peers & lt_mask); // rank among the wavefront's elements of the same digit
    }
    __syncthreads();
    {
        // thread d: where the digit's elements start in the block's sorted order, and each wavefront's share of them
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
    for (int r = 0; r < RO_ROWS; ++r) lpos[r] += cnt[w][(key[r] >> shift) & mask];
}

// Stable scatter of one radix pass over (key, value) pairs.  vals == nullptr: the values are the positions (first pass).
__global__ void __launch_bounds__(RO_THREADS)
    k_index_scatter(const int32_t *__restrict__ keys, const int32_t *__restrict__ vals, int32_t *__restrict__ keys_out,
                    int32_t *__restrict__ vals_out, int64_t M, int shift, int bits, int32_t nblk, const int32_t *__restrict__ table_s,
                    const int32_t *__restrict__ totals)
{
    __shared__ uint2 stage[RO_TILE]; // (key, value) in the block's sorted order
    __shared__ int32_t cnt[RO_WAVES][256];
    __shared__ int32_t delta[256];
    __shared__ int32_t scan_lds[16];
    const int lane = threadIdx.x & (KN_WAVE - 1), w = threadIdx.x / KN_WAVE;
    const uint32_t mask = (1u << bits) - 1u;
    const int64_t bbase = (int64_t)blockIdx.x * RO_TILE;
    const int64_t wbase = bbase + (int64_t)w * (RO_ROWS * KN_WAVE);
    const int32_t n_here = (int32_t)min((int64_t)RO_TILE, M - bbase); // elements of this block (>= 1)
    uint32_t key[RO_ROWS];
    int32_t val[RO_ROWS], lpos[RO_ROWS];
#pragma unroll
    for (int r = 0; r < RO_ROWS; ++r) {
        const int64_t i = min(wbase + r * KN_WAVE + lane, M - 1);
        key[r] = (uint32_t)keys[i];
        val[r] = vals ? vals[i] : (int32_t)i;
    }
    rank_block(key, lpos, M, shift, bits, nblk, table_s, totals, cnt, delta, scan_lds);
#pragma unroll
    for (int r = 0; r < RO_ROWS; ++r)
        if (wbase + r * KN_WAVE + lane < M) stage[lpos[r]] = make_uint2(key[r], (uint32_t)val[r]);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < RO_ROWS; ++k) {
        const int32_t sp = k * RO_THREADS + threadIdx.x; // position in the block's sorted order
        if (sp < n_here) {
            const uint2 v = stage[sp];
            const int32_t dst = sp + delta[(v.x >> shift) & mask];
            keys_out[dst] = (int32_t)v.x;
            vals_out[dst] = (int32_t)v.y;
        }
    }
}

// Stable scatter of one radix pass over the samples themselves.  `keys`: the keys in the order of the input.
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
    constexpr int ROWS = RO_ROWS;
    extern __shared__ u4 stage[]; // RO_TILE halves in the block's sorted order
    __shared__ int32_t cnt[RO_WAVES][256];
    __shared__ int32_t delta[256];
    __shared__ int32_t scan_lds[16];
    const int lane = threadIdx.x & (KN_WAVE - 1), w = threadIdx.x / KN_WAVE;
    const uint32_t mask = (1u << bits) - 1u;
    const int64_t bbase = (int64_t)blockIdx.x * RO_TILE;
    const int64_t wbase = bbase + (int64_t)w * (ROWS * KN_WAVE);
    const int32_t n_here = (int32_t)min((int64_t)RO_TILE, M - bbase); // records of this block (>= 1)
    uint32_t key[ROWS];
    int32_t lpos[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) key[r] = (uint32_t)keys[min(wbase + r * KN_WAVE + lane, M - 1)];
    rank_block(key, lpos, M, shift, bits, nblk, table_s, totals, cnt, delta, scan_lds);

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

// Bucket offsets, counts and the tile list of the grouped MLP from the sorted keys (key j at key_of[key_stride * j]:
// word 3 of each first half of the re-ordered samples, or a plain array).
// A wavefront takes three networks n0, n0+1, n0+2 (n = 0 .. N; N: the points without a network): its four 16-lane
// groups find the number of keys below n0 .. n0+3 by a 16-way search (one load per lane and round, five or six rounds
// for 2^22 keys), so that groups 0..2 know both ends of their bucket; each writes offsets[n] and counts[n], and its
// network's tiles (chunks of at most tile_len records) into slots that the workgroup takes from the zeroed counter
// n_tiles with one atomic (the order of tiles is free: nothing observable depends on it).  offsets has N + 2 entries;
// the group of n = N writes the last two.
constexpr int OT_NETS_PER_WAVE = 3, OT_THREADS = 1024, OT_WAVES = OT_THREADS / KN_WAVE;
__global__ void __launch_bounds__(OT_THREADS)
    k_offsets_tiles(const uint32_t *__restrict__ key_of, int key_stride, int64_t M, int32_t N, int32_t tile_len,
                    int32_t *__restrict__ offsets, int32_t *__restrict__ user_offsets, int32_t *__restrict__ counts,
                    int32_t *__restrict__ user_counts, KnTile *__restrict__ tiles, int32_t *__restrict__ n_tiles)
{
    const int lane = threadIdx.x & (KN_WAVE - 1), t = lane & 15, sub = lane >> 4;
    const int32_t wave_id = (blockIdx.x * blockDim.x + threadIdx.x) / KN_WAVE;
    const int32_t n = wave_id * OT_NETS_PER_WAVE + sub; // the bound this group searches; groups 0..2 own network n
    const bool searches = n <= N + 1;
    const uint32_t bound = (uint32_t)n;
    int64_t lo = 0, hi = searches ? M : 0; // the number of keys below `bound` lies in [lo, hi]
    while (__any(hi > lo)) { // each round cuts the interval to a seventeenth; uniform trip count in the wavefront
        const int64_t len = hi - lo;
        const bool last = len <= 16;
        // probes: strictly inside, increasing in t, distinct (len > 16); the last round tests every position left
        const int64_t pos = last ? lo + t : lo + (int64_t)(t + 1) * len / 17;
        bool below = false;
        if (pos < hi) below = key_of[(int64_t)key_stride * pos] < bound;
        const int c = __popcll((__ballot(below) >> (16 * sub)) & 0xffffull); // keys are sorted: lanes 0 .. c-1
        if (last) {
            lo = hi = lo + c;
        } else {
            const int64_t p_below = lo + (int64_t)c * len / 17;       // probe c-1 (if c > 0): the last one below
            const int64_t p_above = lo + (int64_t)(c + 1) * len / 17; // probe c (if c < 16): the first one not below
            if (c < 16) hi = p_above;
            if (c > 0) lo = p_below + 1;
        }
    }
    const int32_t first = (int32_t)lo;
    const int32_t next = __shfl(first, (lane + 16) & (KN_WAVE - 1), KN_WAVE); // the following group's bound
    const bool mine = sub < OT_NETS_PER_WAVE && n <= N;
    const int32_t count = mine ? next - first : 0;
    if (mine && t == 0) {
        offsets[n] = first;
        if (user_offsets) user_offsets[n] = first;
        if (n == N) {
            offsets[N + 1] = next; // = M
            if (user_offsets) user_offsets[N + 1] = next;
        }
        counts[n] = count;
        if (user_counts) user_counts[n] = count;
    }
    // tiles: bucket N (no network) gets none
    const int32_t n_mine = (mine && n < N) ? (count + tile_len - 1) / tile_len : 0;
    int32_t before = 0, wave_total = 0; // tiles of the groups in front of mine in the wavefront
#pragma unroll
    for (int g = 0; g < OT_NETS_PER_WAVE; ++g) {
        const int32_t v = __shfl(n_mine, 16 * g, KN_WAVE);
        if (g < sub) before += v;
        wave_total += v;
    }
    // one atomic per workgroup: atomics on one address execute one after the other (11 ns each)
    __shared__ int32_t wave_tiles[OT_WAVES], block_base;
    const int wv = threadIdx.x / KN_WAVE;
    if (lane == 0) wave_tiles[wv] = wave_total;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t all = 0;
        for (int i = 0; i < OT_WAVES; ++i) all += wave_tiles[i];
        block_base = all > 0 ? atomicAdd(n_tiles, all) : 0;
    }
    __syncthreads();
    int32_t base = block_base + before;
    for (int i = 0; i < wv; ++i) base += wave_tiles[i];
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

// workgroups of k_offsets_tiles: OT_WAVES wavefronts of OT_NETS_PER_WAVE networks each, for the networks 0 .. N
int64_t offsets_tiles_blocks(int32_t N) { return kn_div_up(kn_div_up((int64_t)N + 1, OT_NETS_PER_WAVE), OT_WAVES); }

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
        hipLaunchKernelGGL(k_key_hist, grid, block, 0, st, w.keys_b, M, bits0, (1u << bits1) - 1u, nblk, w.table, (int32_t *)nullptr,
                           (int64_t)0);
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
    hipLaunchKernelGGL(k_offsets_tiles, dim3((unsigned)offsets_tiles_blocks(N)), dim3(OT_THREADS), 0, st,
                       (const uint32_t *)sorted_pos + 3, 4, M, N, tile_len, w.offsets, (int32_t *)nullptr, w.counts, user_counts, w.tiles,
                       w.n_tiles);
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

// ---------------------------------------------------------------------------------------------
// index sort
namespace {
struct BucketWs {
    int32_t *keys_b, *vals_a, *vals_b, *table, *totals, *n_tiles, *counts, *offsets;
    KnTile *tiles;
    int64_t nblk;
};
void carve_bucket(KnCarver &c, int64_t M, int32_t N, BucketWs &w)
{
    w.nblk = kn_div_up(M > 0 ? M : 1, RO_TILE);
    w.n_tiles = c.carve<int32_t>(1);
    w.table = c.carve<int32_t>(256 * w.nblk);
    w.totals = c.carve<int32_t>(256);
    w.keys_b = c.carve<int32_t>(M);
    w.vals_a = c.carve<int32_t>(M);
    w.vals_b = c.carve<int32_t>(M);
    w.counts = c.carve<int32_t>(N + 1);
    w.offsets = c.carve<int32_t>(N + 2);
    w.tiles = c.carve<KnTile>(kn_max_tiles(M, N, 64));
}
} // namespace

int64_t kn_bucket_ws_bytes(int64_t M, int32_t N)
{
    KnCarver c((void *)256, INT64_MAX / 2);
    BucketWs w;
    carve_bucket(c, M, N, w);
    return c.used;
}

int kn_bucket_run(hipStream_t st, int32_t *keys, int64_t M, int32_t N, int32_t tile_len, int32_t *user_counts, int32_t *user_offsets,
                  int32_t *user_perm, KnCarver &ws, KnBucketOut *out)
{
    if (M < 0 || M > (1ll << 30) || N < 1 || N > 65535 || tile_len < 64) return KN_E_INVALID_ARG;
    BucketWs w;
    carve_bucket(ws, M, N, w);
    if (!ws.ok()) return KN_E_WORKSPACE;
    const int bits = key_bits(N);
    const bool two = bits > 8;
    const int bits0 = two ? bits / 2 : bits, bits1 = bits - bits0;
    const int32_t nblk = (int32_t)w.nblk;
    const dim3 grid((unsigned)nblk), block(RO_THREADS);
    const int32_t *sorted_keys = keys;
    const int32_t *perm = w.vals_a;
    // the first kernel clears the tile counter (with no keys there are no passes: a fill does it)
    if (M == 0) KN_TRY(kn_fill_i32(st, w.n_tiles, 1, 0));
    if (M > 0) {
        hipLaunchKernelGGL(k_key_hist, grid, block, 0, st, keys, M, 0, (1u << bits0) - 1u, nblk, w.table, w.n_tiles, (int64_t)1);
        KN_CHECK_LAUNCH();
        hipLaunchKernelGGL(k_digit_scan, dim3(1u << bits0), block, 0, st, w.table, nblk, w.totals);
        KN_CHECK_LAUNCH();
        int32_t *v1 = (!two && user_perm) ? user_perm : w.vals_a;
        hipLaunchKernelGGL(k_index_scatter, grid, block, 0, st, keys, (const int32_t *)nullptr, w.keys_b, v1, M, 0, bits0, nblk, w.table,
                           w.totals);
        KN_CHECK_LAUNCH();
        sorted_keys = w.keys_b;
        perm = v1;
        if (two) {
            hipLaunchKernelGGL(k_key_hist, grid, block, 0, st, w.keys_b, M, bits0, (1u << bits1) - 1u, nblk, w.table, (int32_t *)nullptr,
                               (int64_t)0);
            KN_CHECK_LAUNCH();
            hipLaunchKernelGGL(k_digit_scan, dim3(1u << bits1), block, 0, st, w.table, nblk, w.totals);
            KN_CHECK_LAUNCH();
            int32_t *v2 = user_perm ? user_perm : w.vals_b;
            // (the caller's key array is free by now: it takes the keys in final order)
            hipLaunchKernelGGL(k_index_scatter, grid, block, 0, st, w.keys_b, v1, keys, v2, M, bits0, bits1, nblk, w.table, w.totals);
            KN_CHECK_LAUNCH();
            sorted_keys = keys;
            perm = v2;
        }
    }
    hipLaunchKernelGGL(k_offsets_tiles, dim3((unsigned)offsets_tiles_blocks(N)), dim3(OT_THREADS), 0, st,
                       (const uint32_t *)sorted_keys, 1, M, N, tile_len, w.offsets, user_offsets, w.counts, user_counts, w.tiles, w.n_tiles);
    KN_CHECK_LAUNCH();
    out->perm = perm;
    out->counts = w.counts;
    out->offsets = w.offsets;
    out->tiles = w.tiles;
    out->n_tiles = w.n_tiles;
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
