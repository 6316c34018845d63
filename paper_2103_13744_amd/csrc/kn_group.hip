// Grouping of a render wave's samples by network (Sec. 3.5 "Implementation": points are ordered so
// that the inputs of one network are contiguous before the networks are evaluated).
//
// The renderer does not need the stable order that kn_bucket guarantees: a sample's network output does
// not depend on where it sits inside its group, nor on the order of the groups.  Samples of neighbouring
// rays fall into few cells, so instead of sorting the keys every workgroup counts the keys of a contiguous
// range of rows in LDS and touches global memory only for the bins it met:
//   histogram   per-network sample counts of the wave, accumulated by the marching kernel itself.
//   offsets     exclusive prefix sums of the histogram and the tile list.  Small grids: every workgroup of
//               the fill pass derives the offsets it needs from the histogram, the first few also write the
//               tiles; otherwise k_group_offsets (one workgroup) and k_group_tiles (one thread per group).
//   fill        a workgroup reserves, per bin it met, a range inside the group with one integer atomic and
//               writes the slot numbers of its samples there.
//
// Input is the wave's row layout: row i holds cnt[i] samples in slots i*S .. i*S + cnt[i] - 1.
#include "kn_common.h"
#include <type_traits>

namespace {

constexpr int GROUP_THREADS = 256;
constexpr int GROUP_FUSED_MAX_BINS = KN_GROUP_FUSED_MAX_BINS; // largest grid whose histogram the fill pass scans by itself
constexpr int GROUP_HASH_PROBES = 16;      // slots tried before a bin is handled through global memory instead

// tiles of c samples; tile_len is a power of two (the host checks it)
__device__ __forceinline__ int32_t tiles_of(int32_t c, int32_t tile_len) { return (c + tile_len - 1) >> (31 - __builtin_clz(tile_len)); }

// tiles of one group: the owner lane has written the first; groups of several tiles are finished by the
// whole wavefront (every lane of the wavefront must call this, with its own group or nt == 0)
__device__ __forceinline__ void write_tiles(KnTile *__restrict__ tiles, int32_t b, int32_t off, int32_t c, int32_t nt,
                                            int32_t tpos, int32_t tile_len, int lane)
{
    if (nt > 0) tiles[tpos] = KnTile{b, off, min(tile_len, c), 0};
    unsigned long long big = __ballot(nt > 1);
    while (big) {
        const int srcl = __builtin_ctzll(big);
        big &= big - 1;
        // (the source lane is the same for the whole wavefront: scalar reads, no lane exchange)
        const int32_t gb = __builtin_amdgcn_readlane(b, srcl), go = __builtin_amdgcn_readlane(off, srcl),
                      gc = __builtin_amdgcn_readlane(c, srcl), gt = __builtin_amdgcn_readlane(tpos, srcl),
                      gn = __builtin_amdgcn_readlane(nt, srcl);
        for (int32_t k = 1 + lane; k < gn; k += KN_WAVE)
            tiles[gt + k] = KnTile{gb, go + k * tile_len, min(tile_len, gc - k * tile_len), 0};
    }
}

// MODE 1: (large grids) `global` holds each group's absolute fill cursor; reserve and fill this workgroup's ranges of
//         `perm`.  A counter per network would not fit in LDS, and neighbouring rays meet few networks, so the
//         counters live in an LDS hash table (bins_cap slots, linear probing) keyed by network; a bin that finds no
//         slot within GROUP_HASH_PROBES is reserved through global memory run by run.
// MODE 2: (small grids) bins_cap = N direct counters; `hist` holds the finished histogram and `global` zeroed fill counters:
//         derive the group offsets here (groups are laid out in the order bin % 256, bin / 256), reserve and
//         fill; the first N / 256 workgroups also write the tile list.
//
// A workgroup covers an equal share of consecutive rows, 256 >> g_log2 of them at a time with 1 << g_log2 lanes
// per row.  A lane reads its row four keys at a time (chunks g, g + G, ...), and a run of equal keys inside a
// chunk (consecutive samples of a ray mostly share their cell) costs one LDS atomic.
template <int MODE>
__global__ void __launch_bounds__(GROUP_THREADS)
    k_group_pass(const int32_t *__restrict__ row_keys, const int32_t *__restrict__ cnt, const int32_t *__restrict__ ctl,
                 int32_t N, int32_t bins_cap, int32_t *__restrict__ global,
                 int32_t *__restrict__ perm, const int32_t *__restrict__ hist, int32_t tile_len,
                 KnTile *__restrict__ tiles, int32_t *__restrict__ n_tiles)
{
    typedef int32_t i4 __attribute__((ext_vector_type(4)));
    extern __shared__ int32_t bins[]; // MODE 2: counters [N], then the wave's histogram [N]; else hash keys, counts [bins_cap] each
    __shared__ int32_t scan_lds[GROUP_THREADS / KN_WAVE];
    const int tid = threadIdx.x, lane = tid & (KN_WAVE - 1);
    // the wave's shape comes from device memory (ctl[0] rows of ctl[1] slots): the launch may have been enqueued
    // before it was known.  Lanes per row: enough that a lane meets about two chunks of four keys.
    const int32_t n_rows = ctl[0], S = ctl[1];
    int g_log2 = 0;
    while (g_log2 < 6 && (8 << g_log2) < S) ++g_log2;
    const int32_t set_s = GROUP_THREADS >> g_log2; // rows per set if the rows were full
    const int32_t rows_per_block = ((n_rows + (int32_t)gridDim.x - 1) / (int32_t)gridDim.x + set_s - 1) / set_s * set_s;
    const int32_t r0 = min((int64_t)blockIdx.x * rows_per_block, (int64_t)n_rows);
    const int32_t nr = min(rows_per_block, n_rows - r0);
    // Rows of later waves are long but mostly far from full: the lanes per row follow the average sample count of
    // this workgroup's rows instead of the row length (more rows side by side, fewer idle lanes).
    if (S > 64 && nr > 0) {
        int32_t mine = 0;
        for (int32_t t = tid; t < nr; t += GROUP_THREADS) mine += cnt[r0 + t];
        const int32_t avg = kn_block_sum(mine, scan_lds) / nr;
        int fit = 0;
        while (fit < g_log2 && (8 << fit) < avg) ++fit;
        g_log2 = fit;
        __syncthreads(); // scan_lds is used again below
    }
    const int G = 1 << g_log2, g = tid & (G - 1), sub = tid >> g_log2, rows_per_set = GROUP_THREADS >> g_log2;
    const bool vec = (S & 3) == 0; // rows start on 16-byte boundaries
    const int32_t row_chunks = (S + 3) >> 2;

    int32_t *hcl = bins + bins_cap; // MODE 2: the wave's histogram [N]

    // four keys of chunk ch of the row at `base` (unconditional, clamped inside the row buffer).  VEC (rows start on
    // 16-byte boundaries) is a compile-time choice: with a branch around the loads the compiler cannot count the loads in
    // flight, and waits for all of them wherever it waits for one, which undoes every prefetch below.
    auto load_chunk = [&](auto VEC, int64_t base, int32_t ch) -> i4 {
        const int32_t c = min(ch, row_chunks - 1);
        if constexpr (decltype(VEC)::value) {
            return *(const i4 *)(row_keys + base + 4 * c);
        } else {
            i4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = row_keys[base + min(4 * c + q, S - 1)];
            return v;
        }
    };
    // runs of equal keys among the (up to four) samples j0.. of a chunk; f(key, first j, length) per run
    auto chunk_runs = [&](i4 v, int32_t j0, int32_t c, int32_t w0, int32_t nb, auto &&f) {
        int32_t run_key = -1, run_j = 0, run_len = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int32_t k = v[q] - w0;
            if (j0 + q >= c || (uint32_t)k >= (uint32_t)nb) k = -1;
            if (k == run_key) {
                ++run_len;
            } else {
                if (run_key >= 0) f(run_key, run_j, run_len);
                run_key = k;
                run_j = j0 + q;
                run_len = 1;
            }
        }
        if (run_key >= 0) f(run_key, run_j, run_len);
    };
    // One pass over the rows of the workgroup.  The sample count and the first two chunks of the next set of rows
    // are fetched before the current set is processed, so that only the first set waits for memory.
    struct RowLoad { int32_t c; int64_t base; i4 va, vb; };
    auto fetch_rows = [&](auto VEC, int32_t rs) -> RowLoad {
        RowLoad q;
        const int32_t row = rs + sub;
        const int32_t i = max(r0 + min(row, nr - 1), 0); // (a workgroup without rows reads row 0 and ignores it)
        q.base = (int64_t)i * S;
        const int32_t c = cnt[i]; // (every lane loads: rows beyond the workgroup's share read its last row and drop it)
        q.c = row < nr ? c : 0;
        q.va = load_chunk(VEC, q.base, g);
        q.vb = load_chunk(VEC, q.base, g + G);
        return q;
    };
    auto sweep = [&](auto VEC, int32_t w0, int32_t nb, RowLoad next /* = fetch_rows(0) */, auto &&f) {
        for (int32_t rs = 0; rs < nr; rs += rows_per_set) {
            const RowLoad cur = next;
            next = fetch_rows(VEC, rs + rows_per_set); // (unconditional: past the last set it reads the last row again)
            auto both = [&](i4 va, i4 vb, int32_t ch) {
                chunk_runs(va, 4 * ch, cur.c, w0, nb, [&](int32_t k, int32_t j, int32_t len) { f(k, cur.base + j, len); });
                chunk_runs(vb, 4 * (ch + G), cur.c, w0, nb, [&](int32_t k, int32_t j, int32_t len) { f(k, cur.base + j, len); });
            };
            if (4 * g < cur.c) both(cur.va, cur.vb, g);
            for (int32_t ch = g + 2 * G; 4 * ch < cur.c; ch += 2 * G) // rows longer than two chunks per lane
                both(load_chunk(VEC, cur.base, ch), load_chunk(VEC, cur.base, ch + G), ch);
        }
    };

    // the first rows of the counting sweep are requested before the histogram is staged: one round trip for both
    RowLoad first_rows = vec ? fetch_rows(std::true_type{}, 0) : fetch_rows(std::false_type{}, 0);
    int32_t own_sum = 0; // MODE 2: samples in the bins tid, tid + 256, ..., which this thread lays out below
    if constexpr (MODE == 2) {
        for (int32_t b0 = 0; b0 < N; b0 += 8 * GROUP_THREADS) {
            int32_t v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = hist[min(b0 + u * GROUP_THREADS + tid, N - 1)]; // loads issued together
#pragma unroll
            for (int u = 0; u < 8; ++u) // (the counters are cleared while the histogram is on its way)
                if (b0 + u * GROUP_THREADS + tid < N) bins[b0 + u * GROUP_THREADS + tid] = 0;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (b0 + u * GROUP_THREADS + tid < N) {
                    hcl[b0 + u * GROUP_THREADS + tid] = v[u];
                    own_sum += v[u];
                }
        }
    }

    if constexpr (MODE != 2) {
        int32_t *hkeys = bins, *hcnt = bins + bins_cap;
        const uint32_t hmask = (uint32_t)bins_cap - 1u;
        const int hshift = __builtin_clz((uint32_t)bins_cap) + 1; // 32 - log2(bins_cap)
        for (int32_t b = tid; b < bins_cap; b += GROUP_THREADS) {
            hkeys[b] = -1;
            hcnt[b] = 0;
        }
        __syncthreads();
        // slot of bin k, claimed on first use; -1 when the probed slots all belong to other bins (they never become
        // free again, so the answer for a bin is the same throughout the kernel)
        auto slot_of = [&](int32_t k) -> int32_t {
            uint32_t h = ((uint32_t)k * 2654435761u) >> hshift;
            for (int probe = 0; probe < GROUP_HASH_PROBES; ++probe) {
                int32_t old = hkeys[h];
                if (old == -1) old = atomicCAS(&hkeys[h], -1, k);
                if (old == -1 || old == k) return (int32_t)h;
                h = (h + 1u) & hmask;
            }
            return -1;
        };
        auto count = [&](int32_t k, int64_t, int32_t len) {
            const int32_t sl = slot_of(k);
            if (sl >= 0) atomicAdd(&hcnt[sl], len);
        };
        if (nr > 0) {
            if (vec) sweep(std::true_type{}, 0, N, first_rows, count);
            else sweep(std::false_type{}, 0, N, first_rows, count);
        }
        __syncthreads();
        // the first rows of the filling sweep are requested in front of the reservation's atomics: their round trip runs
        // under the atomics' longer one
        const RowLoad fill_first = vec ? fetch_rows(std::true_type{}, 0) : fetch_rows(std::false_type{}, 0);
        // first position of this workgroup's range inside each group it met: the returning atomics of a thread's eight
        // table slots are in flight together
        for (int32_t q0 = 0; q0 < bins_cap; q0 += 8 * GROUP_THREADS) {
            int32_t k[8], c[8], base[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int32_t q = q0 + u * GROUP_THREADS + tid;
                k[u] = q < bins_cap ? hkeys[q] : -1;
                c[u] = q < bins_cap ? hcnt[q] : 0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) base[u] = (k[u] >= 0 && c[u] > 0) ? atomicAdd(&global[k[u]], c[u]) : 0;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (k[u] >= 0 && c[u] > 0) hcnt[q0 + u * GROUP_THREADS + tid] = base[u];
        }
        __syncthreads();
        auto fill = [&](int32_t k, int64_t slot, int32_t len) {
            const int32_t sl = slot_of(k);
            const int32_t pos = sl >= 0 ? atomicAdd(&hcnt[sl], len) : atomicAdd(&global[k], len);
            for (int32_t t = 0; t < len; ++t) perm[pos + t] = (int32_t)slot + t;
        };
        if (nr > 0) {
            if (vec) sweep(std::true_type{}, 0, N, fill_first, fill);
            else sweep(std::false_type{}, 0, N, fill_first, fill);
        }
    } else {
        __syncthreads(); // counters cleared, histogram staged
        // heads and lengths of the runs of equal keys among the eight samples of a lane's two chunks (straight-line code)
        auto runs8 = [&](i4 va, i4 vb, int32_t ja, int32_t jb, int32_t c, int32_t (&key)[8], int32_t (&len)[8], bool (&valid)[8],
                         bool (&head)[8]) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                key[q] = q < 4 ? va[q] : vb[q - 4];
                valid[q] = (q < 4 ? ja + q : jb + q - 4) < c && (uint32_t)key[q] < (uint32_t)N;
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) head[q] = valid[q] && ((q & 3) == 0 || !valid[q - 1] || key[q - 1] != key[q]);
#pragma unroll
            for (int q = 7; q >= 0; --q) len[q] = valid[q] ? 1 + (((q & 3) != 3 && valid[q + 1] && !head[q + 1]) ? len[q + 1] : 0) : 0;
        };
        // f(current row set, its two chunks, their first sample numbers) for every pair of chunks of the workgroup's rows
        auto pairs = [&](auto VEC, RowLoad next /* = fetch_rows(0) */, auto &&f) {
            for (int32_t rs = 0; rs < nr; rs += rows_per_set) {
                const RowLoad cur = next;
                next = fetch_rows(VEC, rs + rows_per_set); // (unconditional: past the last set it reads the last row again)
                if (4 * g < cur.c) f(cur, cur.va, cur.vb, 4 * g, 4 * (g + G));
                for (int32_t ch = g + 2 * G; 4 * ch < cur.c; ch += 2 * G) // rows longer than two chunks per lane
                    f(cur, load_chunk(VEC, cur.base, ch), load_chunk(VEC, cur.base, ch + G), 4 * ch, 4 * (ch + G));
            }
        };
        auto count = [&](const RowLoad &cur, i4 va, i4 vb, int32_t ja, int32_t jb) {
            int32_t key[8], len[8];
            bool valid[8], head[8];
            runs8(va, vb, ja, jb, cur.c, key, len, valid, head);
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (head[q]) atomicAdd(&bins[key[q]], len[q]);
        };
        if (nr > 0) {
            if (vec) pairs(std::true_type{}, first_rows, count);
            else pairs(std::false_type{}, first_rows, count);
        }
        __syncthreads();
        // exclusive offsets of all groups: thread t owns the bins t, t + 256, ... and lays them out in a row
        int32_t total;
        const int32_t fused_off0 = kn_block_exclusive_scan(own_sum, scan_lds, total);
        // the first rows of the filling sweep are requested in front of the reservation's atomics: their round trip runs
        // under the atomics' longer one
        const RowLoad fill_first = vec ? fetch_rows(std::true_type{}, 0) : fetch_rows(std::false_type{}, 0);
        {
            // first position of this workgroup's range inside each group it met: the returning atomics of a thread's
            // eight bins are in flight together (a workgroup meets few networks: most threads issue none)
            int32_t off = fused_off0;
            for (int32_t b0 = 0; b0 < N; b0 += 8 * GROUP_THREADS) {
                int32_t c[8], h[8], base[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int32_t b = b0 + u * GROUP_THREADS + tid;
                    c[u] = b < N ? bins[b] : 0;
                    h[u] = b < N ? hcl[b] : 0;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) base[u] = c[u] ? atomicAdd(&global[b0 + u * GROUP_THREADS + tid], c[u]) : 0;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (c[u]) bins[b0 + u * GROUP_THREADS + tid] = off + base[u];
                    off += h[u];
                }
            }
        }
        // tile list: slice k = the bins 256 k .. 256 k + 255, one workgroup per slice (tile positions follow
        // the same layout order as the offsets)
        for (int64_t slice = blockIdx.x; slice * GROUP_THREADS < N; slice += gridDim.x) {
            const int32_t mine_b = (int32_t)slice * GROUP_THREADS + tid;
            int32_t my_tiles = 0, tiles_before = 0, off_mine = fused_off0;
            for (int32_t b = tid; b < N; b += GROUP_THREADS) {
                const int32_t c = hcl[b];
                const int32_t nt = tiles_of(c, tile_len);
                if (b < mine_b) {
                    tiles_before += nt;
                    off_mine += c;
                }
                my_tiles += nt;
            }
            const int32_t tpos = kn_block_exclusive_scan(my_tiles, scan_lds, total) + tiles_before;
            if (slice == 0 && tid == 0) *n_tiles = total;
            const int32_t c = mine_b < N ? hcl[mine_b] : 0;
            write_tiles(tiles, mine_b, off_mine, c, tiles_of(c, tile_len), tpos, tile_len, lane);
        }
        __syncthreads(); // every bin this workgroup met holds the absolute position of its first sample
        // Filling sweep: the first sample of every run takes the run's place with one returning LDS atomic, and all of
        // a lane's are issued before the first result is used (taken run by run, each atomic's latency sat in front of
        // the next).
        auto fill = [&](const RowLoad &cur, i4 va, i4 vb, int32_t ja, int32_t jb) {
            int32_t key[8], len[8], pos[8];
            bool valid[8], head[8];
            runs8(va, vb, ja, jb, cur.c, key, len, valid, head);
#pragma unroll
            for (int q = 0; q < 8; ++q) pos[q] = head[q] ? atomicAdd(&bins[key[q]], len[q]) : 0;
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (valid[q] && !head[q]) pos[q] = pos[q - 1] + 1;
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (valid[q]) perm[pos[q]] = (int32_t)(cur.base + (q < 4 ? ja + q : jb + q - 4));
        };
        if (nr > 0) {
            if (vec) pairs(std::true_type{}, fill_first, fill);
            else pairs(std::false_type{}, fill_first, fill);
        }
    }
}

// histogram -> group offsets (also the fill cursors) and tile positions.  One workgroup; a thread scans 16 contiguous
// bins (one 64-byte line, read and written as four 16-byte accesses), 16,384 bins per round.  The histogram entries
// are replaced by the groups' first tile positions, totals[0] = tiles, totals[1] = samples; k_group_tiles writes the
// tiles from that and clears the histogram for the next use.
__global__ void __launch_bounds__(1024)
    k_group_offsets(int32_t *__restrict__ hist, int32_t N, int32_t tile_len, int32_t *__restrict__ cursor,
                    int32_t *__restrict__ totals)
{
    constexpr int T = 1024, PER = 16;
    typedef int32_t i4 __attribute__((ext_vector_type(4)));
    __shared__ int32_t lds[T / KN_WAVE];
    const int tid = threadIdx.x;
    int32_t carry_s = 0, carry_t = 0;
    for (int32_t b0 = 0; b0 < N; b0 += T * PER) {
        const int32_t e0 = b0 + PER * tid;
        // (16-byte accesses only where both arrays are 16-byte aligned: the cursors start N ints behind the histogram)
        const bool full = e0 + PER <= N && (N & 3) == 0;
        int32_t c[PER];
        if (full) {
#pragma unroll
            for (int u = 0; u < PER / 4; ++u) {
                const i4 q = *(const i4 *)(hist + e0 + 4 * u);
                c[4 * u] = q[0]; c[4 * u + 1] = q[1]; c[4 * u + 2] = q[2]; c[4 * u + 3] = q[3];
            }
        } else {
#pragma unroll
            for (int u = 0; u < PER; ++u) c[u] = e0 + u < N ? hist[e0 + u] : 0;
        }
        int32_t sum_s = 0, sum_t = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            sum_s += c[u];
            sum_t += tiles_of(c[u], tile_len);
        }
        int32_t tot_s, tot_t;
        int32_t off = carry_s + kn_block_exclusive_scan(sum_s, lds, tot_s);
        int32_t tpos = carry_t + kn_block_exclusive_scan(sum_t, lds, tot_t);
        int32_t o[PER], t[PER];
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            o[u] = off;
            t[u] = tpos;
            off += c[u];
            tpos += tiles_of(c[u], tile_len);
        }
        if (full) {
#pragma unroll
            for (int u = 0; u < PER / 4; ++u) {
                *(i4 *)(cursor + e0 + 4 * u) = (i4){o[4 * u], o[4 * u + 1], o[4 * u + 2], o[4 * u + 3]};
                *(i4 *)(hist + e0 + 4 * u) = (i4){t[4 * u], t[4 * u + 1], t[4 * u + 2], t[4 * u + 3]};
            }
        } else {
#pragma unroll
            for (int u = 0; u < PER; ++u)
                if (e0 + u < N) {
                    cursor[e0 + u] = o[u];
                    hist[e0 + u] = t[u];
                }
        }
        carry_s += tot_s;
        carry_t += tot_t;
    }
    if (tid == 0) {
        totals[0] = carry_t;
        totals[1] = carry_s;
    }
}

// one thread per group; groups of several tiles are finished by the whole wavefront
__global__ void __launch_bounds__(GROUP_THREADS)
    k_group_tiles(int32_t *__restrict__ hist, int32_t N, int32_t tile_len, const int32_t *__restrict__ cursor,
                  const int32_t *__restrict__ totals, KnTile *__restrict__ tiles)
{
    const int32_t b = blockIdx.x * GROUP_THREADS + threadIdx.x;
    const int lane = threadIdx.x & (KN_WAVE - 1);
    int32_t off = 0, c = 0, tpos = 0;
    if (b < N) {
        off = cursor[b];
        c = (b + 1 < N ? cursor[b + 1] : totals[1]) - off;
        tpos = hist[b];
        hist[b] = 0;
    }
    write_tiles(tiles, b, off, c, tiles_of(c, tile_len), tpos, tile_len, lane);
}

} // namespace

// the fill kernels may need more dynamic LDS than the default limit (once per device, from kn_create)
int kn_group_configure()
{
    const int most = (int)(sizeof(int32_t) * 2 * GROUP_FUSED_MAX_BINS);
    KN_HIP(hipFuncSetAttribute((const void *)k_group_pass<1>, hipFuncAttributeMaxDynamicSharedMemorySize, most));
    KN_HIP(hipFuncSetAttribute((const void *)k_group_pass<2>, hipFuncAttributeMaxDynamicSharedMemorySize, most));
    return KN_OK;
}

static void carve_group(KnCarver &c, int64_t slots, int32_t N, KnGroupWs &w)
{
    w.hist = c.carve<int32_t>(2 * (int64_t)N); // histogram, then the fill cursors
    w.cursor = w.hist ? w.hist + N : nullptr;
    w.n_tiles = c.carve<int32_t>(2); // [1]: the sample total (large grids)
    w.perm = c.carve<int32_t>(slots);
    w.tiles = c.carve<KnTile>(kn_max_tiles(slots, N, 64));
}

int64_t kn_group_ws_bytes(int64_t slots, int32_t N)
{
    KnCarver c((void *)256, INT64_MAX / 2);
    KnGroupWs w;
    carve_group(c, slots, N, w);
    return c.used;
}

void kn_group_carve(KnCarver &ws, int64_t slots, int32_t N, KnGroupWs *w) { carve_group(ws, slots, N, *w); }

int kn_group_run(hipStream_t st, const KnKnobs &knobs, const int32_t *row_keys, const int32_t *cnt, const int32_t *ctl,
                 int64_t max_rows, int32_t N, int32_t tile_len, const KnGroupWs &w, KnBucketOut *out)
{
    if (!ctl || max_rows < 0 || max_rows > 0x7fffffffLL || N < 1 || tile_len < 64 || (tile_len & (tile_len - 1)) != 0)
        return KN_E_INVALID_ARG; // (tile counts are taken with a shift)
    if (!w.hist || !w.cursor || !w.n_tiles || !w.perm || !w.tiles) return KN_E_WORKSPACE;
    const bool fused = kn_group_fused(knobs, N);
    const int32_t bins_cap = fused ? N : knobs.group_hash_slots; // direct counters, or hash slots
    int64_t blocks = kn_div_up(max_rows > 0 ? max_rows : 1, 16);
    if (blocks > 1024) blocks = 1024;
    const size_t lds_bytes = sizeof(int32_t) * (size_t)bins_cap * 2;
    const dim3 grid((unsigned)blocks), block(GROUP_THREADS);
    if (fused) {
        hipLaunchKernelGGL(k_group_pass<2>, grid, block, lds_bytes, st, row_keys, cnt, ctl, N, bins_cap, w.cursor, w.perm,
                           (const int32_t *)w.hist, tile_len, w.tiles, w.n_tiles);
        KN_CHECK_LAUNCH();
    } else {
        hipLaunchKernelGGL(k_group_offsets, dim3(1), dim3(1024), 0, st, w.hist, N, tile_len, w.cursor, w.n_tiles);
        KN_CHECK_LAUNCH();
        hipLaunchKernelGGL(k_group_tiles, dim3((unsigned)kn_div_up(N, GROUP_THREADS)), dim3(GROUP_THREADS), 0, st, w.hist, N,
                           tile_len, (const int32_t *)w.cursor, (const int32_t *)w.n_tiles, w.tiles);
        KN_CHECK_LAUNCH();
        hipLaunchKernelGGL(k_group_pass<1>, grid, block, lds_bytes, st, row_keys, cnt, ctl, N, bins_cap, w.cursor, w.perm,
                           (const int32_t *)nullptr, tile_len, (KnTile *)nullptr, (int32_t *)nullptr);
        KN_CHECK_LAUNCH();
    }
    out->perm = w.perm;
    out->counts = nullptr;
    out->offsets = nullptr;
    out->tiles = w.tiles;
    out->n_tiles = w.n_tiles;
    return KN_OK;
}

