// Ray marching with empty-space skipping, alpha blending with early ray termination, and the
// wave loop that ties them to bucketing and the grouped MLP (Sec. 3.1 Eq. 1-4, Sec. 3.4).
//
// A wave gives every live ray up to S samples.  Marching is cooperative: a group of G lanes (8 or 16)
// owns one ray and tests G consecutive lattice points per iteration, so the latency of the
// dependent index arithmetic + occupancy load is paid once per G points.  A coarse skip field
// (Chebyshev distance, in blocks of 4^3 voxels, to the nearest occupied block) lets a group jump
// over lattice points that provably lie in empty blocks; every point that could be kept is still
// tested with the exact arithmetic of Eq. 6, so the kept set equals the plain per-point definition.
// Kept samples go to the ray's row of the wave's buffers (network id and packed (ray, k) record per slot, a
// count per row); the grouping and the MLP kernel address samples by slot number, so the rows are never
// compacted into a list.
#include "kn_common.h"
#include "kn_dir_encode.h"

#include <math.h>

#include <chrono>

namespace {

constexpr int MARCH_G = 16;    // lanes per ray of the stage kernel and of the blend of long rows
constexpr int LIST_GROUP = 16; // rows per group in which the blend counts survivors and the next march compacts the list

struct MarchParams {
    KnGrid net, occ;
    KnGrid content; // box around everything occupied (res 0: nothing is); rays are clipped against it
    const uint32_t *occ_bits;
    const uint8_t *skip_dist;
    int32_t skip_res[3];
    float skip_inv[3];   // 1 / (edge of a skip block) per axis
    float skip_edge_min; // shortest edge of a skip block
    float skip_margin;   // safety margin on the jump radius (position rounding)
    int32_t has_occ;
    // >= 0 on every axis: the occupancy grid refines the network grid by 2^net_shift[a] (same box), so that the
    // network cell of a point is its voxel coordinate shifted right, exactly (scaling the cell edge by a power of two
    // scales the fp32 quotient of Eq. 6 by the same power of two without a rounding difference)
    int32_t net_shift[3];
    float t_near, step;
    int32_t K;
    const int32_t *cell_net; // sparse network grid: cell -> network or -1 (kernels built with OPT_SPARSE read it)
    uint32_t seed_key;       // stratified sampling: kn_mix32(seed) (kernels built with OPT_STRAT use it)
};

// Variants of the marching kernels, chosen at compile time so that the plain path carries none of their cost:
// a sparse network grid (a table look-up per kept point; points in cells without a network are dropped) and
// stratified sampling (lattice points at their drawn offsets instead of the middle of their intervals).
constexpr int OPT_SPARSE = 1, OPT_STRAT = 2;

// One axis of Eq. 6 without the division when the result cannot depend on it: u' = rel * (1/cell)
// differs from the correctly rounded quotient by a few ulp (less than 4.8e-7 |u'|); only when u' sits that close
// to an integer is the division itself evaluated.  `guard` is that bound for the largest |u'| that matters,
// res + 1: beyond it both u' and the quotient are outside [0, res) whatever their last bits are, and callers only
// ask whether the result is inside that range, and which integer it is if so.  Returns floor(quotient) as a float
// (for values inside the range; some value outside the range otherwise; NaN and inf stay what they are).
__device__ __forceinline__ float axis_floor(float rel, float cell, float inv_cell, float guard, float one_minus_guard)
{
    const float u = rel * inv_cell;
    const float f = floorf(u);
    const float frac = u - f;
    if (frac <= guard || frac >= one_minus_guard) return floorf(rel / cell); // (both false for NaN / inf)
    return f;
}

struct GridFast {
    float bmin[3], cell[3], inv[3], resf[3], guard[3], one_minus_guard[3];
    int32_t res1, res2;
};

__device__ __forceinline__ GridFast make_fast(const KnGrid &g)
{
    GridFast f;
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        f.bmin[a] = g.bmin[a];
        f.cell[a] = g.cell[a];
        f.inv[a] = 1.0f / g.cell[a];
        f.resf[a] = (float)g.res[a];
        f.guard[a] = ((float)g.res[a] + 1.0f) * 4.8e-7f + 1e-30f;
        f.one_minus_guard[a] = 1.0f - f.guard[a];
    }
    f.res1 = g.res[1];
    f.res2 = g.res[2];
    return f;
}

// Eq. 6 per axis: integer cell coordinates of a point, false when it is outside the grid
__device__ __forceinline__ bool grid_coords_fast(const GridFast &g, float x, float y, float z, int32_t &ix, int32_t &iy,
                                                 int32_t &iz)
{
    const float fx = axis_floor(x - g.bmin[0], g.cell[0], g.inv[0], g.guard[0], g.one_minus_guard[0]);
    const float fy = axis_floor(y - g.bmin[1], g.cell[1], g.inv[1], g.guard[1], g.one_minus_guard[1]);
    const float fz = axis_floor(z - g.bmin[2], g.cell[2], g.inv[2], g.guard[2], g.one_minus_guard[2]);
    const bool in = (fx >= 0.0f) && (fx < g.resf[0]) && (fy >= 0.0f) && (fy < g.resf[1]) && (fz >= 0.0f) &&
                    (fz < g.resf[2]);
    ix = (int32_t)fx;
    iy = (int32_t)fy;
    iz = (int32_t)fz;
    return in;
}

__device__ __forceinline__ int32_t grid_index_fast(const GridFast &g, float x, float y, float z)
{
    const float fx = axis_floor(x - g.bmin[0], g.cell[0], g.inv[0], g.guard[0], g.one_minus_guard[0]);
    const float fy = axis_floor(y - g.bmin[1], g.cell[1], g.inv[1], g.guard[1], g.one_minus_guard[1]);
    const float fz = axis_floor(z - g.bmin[2], g.cell[2], g.inv[2], g.guard[2], g.one_minus_guard[2]);
    const bool in = (fx >= 0.0f) && (fx < g.resf[0]) && (fy >= 0.0f) && (fy < g.resf[1]) && (fz >= 0.0f) &&
                    (fz < g.resf[2]);
    if (!in) return -1;
    return ((int32_t)fx * g.res1 + (int32_t)fy) * g.res2 + (int32_t)fz;
}

// Conservative range [k_lo, k_hi) of lattice indices whose point can lie inside the AABB (slab
// test widened by the rounding error of x_k = fma(t_k, d, o) and two steps).  Every index
// outside the range is provably outside the box; indices inside it are still tested exactly.
__device__ __forceinline__ void clip_ray(const KnGrid &g, const float o[3], const float d[3], float t_near, float step,
                                         int32_t K, int32_t &k_lo, int32_t &k_hi)
{
    if (g.res[0] == 0) { // empty box
        k_lo = k_hi = 0;
        return;
    }
    float tmin = -INFINITY, tmax = INFINITY;
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        if (d[a] != 0.0f) {
            const float lo = g.bmin[a], hi = g.bmin[a] + g.cell[a] * (float)g.res[a];
            const float inv = 1.0f / d[a];
            float t0 = (lo - o[a]) * inv, t1 = (hi - o[a]) * inv;
            if (t0 > t1) { float s = t0; t0 = t1; t1 = s; }
            const float mag = fabsf(lo) + fabsf(hi) + fabsf(o[a]) + g.cell[a];
            const float margin = mag * 2.4e-7f * fabsf(inv) + 1e-6f * (fabsf(t0) + fabsf(t1));
            tmin = fmaxf(tmin, t0 - margin);
            tmax = fminf(tmax, t1 + margin);
        }
    }
    // k such that t_near + (k + 1/2) step lies in [tmin, tmax], widened by two steps
    float a = floorf((tmin - t_near) / step - 0.5f) - 2.0f;
    float b = ceilf((tmax - t_near) / step - 0.5f) + 3.0f;
    a = fminf(fmaxf(a, 0.0f), (float)K); // NaN -> 0
    b = fminf(fmaxf(b, 0.0f), (float)K);
    if (!(tmin <= tmax)) { // empty -> nothing; NaN -> stay conservative (full range)
        if (tmin > tmax) { a = 0.0f; b = 0.0f; } else { a = 0.0f; b = (float)K; }
    }
    k_lo = (int32_t)a;
    k_hi = (int32_t)b;
}

// Jump length bookkeeping shared by the two users of the skip field.  A point whose block has
// Chebyshev distance dist >= 2 to the nearest occupied block lies in an empty block, and so does
// every point within Euclidean distance (dist-1) * (shortest block edge) of it, minus a rounding
// margin: jump(dist) is how many further lattice indices that covers.
struct SkipJump {
    float a, b;
    bool use;
    // strat: with stratified sampling point k + j lies up to j + 1 steps from point k, one more than on the
    // midpoint lattice
    __device__ __forceinline__ SkipJump(const MarchParams &p, const float o[3], const float d[3], bool strat)
    {
        const float dlen = sqrtf(d[0] * d[0] + d[1] * d[1] + d[2] * d[2]);
        const float inv_step_len = 1.0f / (p.step * dlen); // 1 / distance covered by one lattice step
        a = p.skip_edge_min * inv_step_len;
        b = (p.skip_margin + 1e-6f * (fabsf(o[0]) + fabsf(o[1]) + fabsf(o[2]))) * inv_step_len + (strat ? 2.0f : 1.0f);
        use = p.skip_dist != nullptr && isfinite(inv_step_len);
    }
    __device__ __forceinline__ int32_t jump(int32_t dist) const { return (int32_t)fmaxf(floorf((float)(dist - 1) * a - b), 0.0f); }
};

// skip-field value at a point; -1 = the point is (up to rounding) outside the field
__device__ __forceinline__ int32_t skip_lookup(const MarchParams &p, float x, float y, float z)
{
    const float cx = floorf((x - p.occ.bmin[0]) * p.skip_inv[0]);
    const float cy = floorf((y - p.occ.bmin[1]) * p.skip_inv[1]);
    const float cz = floorf((z - p.occ.bmin[2]) * p.skip_inv[2]);
    if (cx >= 0.0f && cx < (float)p.skip_res[0] && cy >= 0.0f && cy < (float)p.skip_res[1] && cz >= 0.0f &&
        cz < (float)p.skip_res[2])
        return p.skip_dist[((int32_t)cx * p.skip_res[1] + (int32_t)cy) * p.skip_res[2] + (int32_t)cz];
    return -1;
}

// One thread walks a ray through provably empty space: returns the first index in [k, k_hi) whose
// point is not known to be empty (or k_hi).  No index it passes over can be a kept sample.
template <int OPT>
__device__ __forceinline__ int32_t skip_to_content(const MarchParams &p, const GridFast &go, const float o[3],
                                                   const float d[3], int32_t k, int32_t k_hi, uint32_t ray_key)
{
    constexpr bool STRAT = (OPT & OPT_STRAT) != 0;
    if (k >= k_hi) return k_hi; // the ray misses the content box: nothing to walk through
    const SkipJump sj(p, o, d, STRAT);
    if (!sj.use) return k;
    while (k < k_hi) {
        float x, y, z;
        kn_lattice_point<STRAT>(o[0], o[1], o[2], d[0], d[1], d[2], p.t_near, p.step, k, x, y, z, ray_key);
        const int32_t dist = skip_lookup(p, x, y, z);
        if (dist >= 2) {
            k += 1 + sj.jump(dist);
        } else if (dist < 0 && grid_index_fast(go, x, y, z) < 0) {
            k += 1; // exactly outside the AABB (the clip range starts a little before the box)
        } else {
            break;
        }
    }
    return min(k, k_hi);
}

// Largest value among the G lanes of a marching group, in every lane of the group.  A group is one row (16 lanes) or
// half a row (8) of the data-parallel-primitive network, so a few permutations inside the row do it, without the LDS
// crossbar that general lane exchanges go through.  All lanes of the group must be active.
template <int G> __device__ __forceinline__ int32_t group_max(int32_t v)
{
    static_assert(G == 16 || G == 8, "a marching group is a DPP row or half of one");
    constexpr int ROW_ROR = 0x120;                     // dpp_ctrl of row_ror:n is 0x120 + n
    constexpr int QUAD_1032 = 0xB1, QUAD_2301 = 0x4E;  // quad_perm:[1,0,3,2], [2,3,0,1]
    constexpr int ROW_HALF_MIRROR = 0x141;             // lane i of each half row <-> lane 7 - i
    if constexpr (G == 16) {
        v = max(v, __builtin_amdgcn_update_dpp(v, v, ROW_ROR + 8, 0xf, 0xf, false));
        v = max(v, __builtin_amdgcn_update_dpp(v, v, ROW_ROR + 4, 0xf, 0xf, false));
        v = max(v, __builtin_amdgcn_update_dpp(v, v, ROW_ROR + 2, 0xf, 0xf, false));
        v = max(v, __builtin_amdgcn_update_dpp(v, v, ROW_ROR + 1, 0xf, 0xf, false));
    } else {
        v = max(v, __builtin_amdgcn_update_dpp(v, v, QUAD_1032, 0xf, 0xf, false));
        v = max(v, __builtin_amdgcn_update_dpp(v, v, QUAD_2301, 0xf, 0xf, false)); // every lane: its quad's largest
        v = max(v, __builtin_amdgcn_update_dpp(v, v, ROW_HALF_MIRROR, 0xf, 0xf, false)); // ... and the other quad's
    }
    return v;
}

// Cooperative march of one ray by a group of G lanes (all lanes of the group call this with
// the same arguments; gl = lane index inside the group).  Collects up to S kept lattice indices in
// [k, k_hi), in ascending order, through emit(j, kk, cell).  Returns the number collected and
// leaves in k the index to resume at (>= k_hi: the ray is exhausted).
template <int OPT, int G, typename Emit>
__device__ __forceinline__ int32_t march_group(const MarchParams &p, const GridFast &gn, const GridFast &go,
                                               const float o[3], const float d[3], int32_t &k, int32_t k_hi, int32_t S,
                                               int gl, uint32_t ray_key, Emit emit)
{
    constexpr bool STRAT = (OPT & OPT_STRAT) != 0, SPARSE = (OPT & OPT_SPARSE) != 0;
    const int lane = threadIdx.x & (KN_WAVE - 1);
    const int gshift = lane & ~(G - 1);
    const uint32_t gmask = (G == 32) ? 0xffffffffu : ((1u << G) - 1u);
    const SkipJump sj(p, o, d, STRAT);
    int32_t n = 0;
    constexpr int SKIP_SHIFT = 2;
    static_assert((1 << SKIP_SHIFT) == KN_SKIP_BLOCK, "skip blocks are 4 voxels wide");
    constexpr int STEPS = 1; // lattice points per lane and iteration (2 halves the iterations but did not pay: the loop is bound by its ALU work)
    while (k < k_hi && n < S) {
        bool kept[STEPS];
        int32_t cell[STEPS], reach[STEPS], kk[STEPS];
#pragma unroll
        for (int c = 0; c < STEPS; ++c) {
            kk[c] = k + c * G + gl;
            kept[c] = false;
            cell[c] = -1;
            reach[c] = 0; // all lattice indices in [kk, reach) are known not to be kept
        }
        float x[STEPS], y[STEPS], z[STEPS];
        int32_t vox[STEPS], dist[STEPS], ix[STEPS], iy[STEPS], iz[STEPS];
        uint32_t word[STEPS];
        // The occupancy word is requested together with the skip-field byte (both addresses follow from the voxel
        // coordinates of the point), for both points of the lane: one memory round trip per iteration.
#pragma unroll
        for (int c = 0; c < STEPS; ++c) {
            vox[c] = 0;
            word[c] = 0xffffffffu;
            dist[c] = 0;
            if (kk[c] < k_hi) {
                kn_lattice_point<STRAT>(o[0], o[1], o[2], d[0], d[1], d[2], p.t_near, p.step, kk[c], x[c], y[c], z[c], ray_key);
                if (p.has_occ) {
                    const bool in = grid_coords_fast(go, x[c], y[c], z[c], ix[c], iy[c], iz[c]);
                    vox[c] = in ? (ix[c] * go.res1 + iy[c]) * go.res2 + iz[c] : -1;
                    word[c] = in ? p.occ_bits[(uint32_t)vox[c] >> 5] : 0u;
                    if (sj.use) // -1: outside the grid, the point is dropped by the exact test below
                        dist[c] = in ? (int32_t)p.skip_dist[((ix[c] >> SKIP_SHIFT) * p.skip_res[1] + (iy[c] >> SKIP_SHIFT)) *
                                                                p.skip_res[2] + (iz[c] >> SKIP_SHIFT)]
                                     : -1;
                }
            }
        }
#pragma unroll
        for (int c = 0; c < STEPS; ++c) {
            if (kk[c] < k_hi) {
                if (dist[c] >= 2) {
                    reach[c] = kk[c] + 1 + sj.jump(dist[c]);
                } else {
                    if (vox[c] >= 0 && ((word[c] >> (vox[c] & 31)) & 1u)) { // Sec. 3.4: inside the AABB, occupied voxel
                        if (p.has_occ && p.net_shift[0] >= 0)
                            cell[c] = ((ix[c] >> p.net_shift[0]) * gn.res1 + (iy[c] >> p.net_shift[1])) * gn.res2 +
                                      (iz[c] >> p.net_shift[2]);
                        else
                            cell[c] = grid_index_fast(gn, x[c], y[c], z[c]);
                        if constexpr (SPARSE) cell[c] = kn_net_of_cell(p.cell_net, cell[c]); // the network, or none
                        kept[c] = cell[c] >= 0;
                    }
                    reach[c] = kept[c] ? kk[c] : kk[c] + 1;
                }
            }
        }
        // kept points in ascending order
        bool full = false;
#pragma unroll
        for (int c = 0; c < STEPS; ++c) {
            if (full) break; // (uniform inside the group)
            const uint32_t mask = (uint32_t)(__ballot(kept[c]) >> gshift) & gmask;
            const int rank = __popc(mask & ((1u << gl) - 1u));
            const int tot = __popc(mask);
            const int room = S - n;
            if (kept[c] && rank < room) emit(n + rank, kk[c], cell[c]);
            if (tot > room) {
                // the first kept sample that did not fit is where the next wave resumes
                const uint32_t over = (uint32_t)(__ballot(kept[c] && rank == room) >> gshift) & gmask;
                k = k + c * G + (__ffs(over) - 1);
                n = S;
                full = true;
            } else {
                n += tot;
            }
        }
        if (full) break;
        // frontier: every index of these chunks was tested or skipped; the farthest jump that starts inside
        // them extends the known-empty range beyond
        k = max(k + STEPS * G, group_max<G>(max(reach[0], reach[STEPS - 1])));
    }
    return n;
}

// ---------------------------------------------------------------------------------------------
// stage kernel behind kn_march: MARCH_G lanes per ray, explicit output arrays
template <int OPT>
__global__ void __launch_bounds__(256)
    k_march_stage(MarchParams p, const float *__restrict__ rays_o, const float *__restrict__ rays_d, int64_t R,
                  const int32_t *__restrict__ k_begin, int32_t S, int32_t *__restrict__ out_k, int32_t *__restrict__ out_count,
                  int32_t *__restrict__ out_k_next)
{
    const int64_t r = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / MARCH_G;
    const int gl = threadIdx.x & (MARCH_G - 1);
    if (r >= R) return;
    const float o[3] = {rays_o[3 * r], rays_o[3 * r + 1], rays_o[3 * r + 2]};
    const float d[3] = {rays_d[3 * r], rays_d[3 * r + 1], rays_d[3 * r + 2]};
    const GridFast gn = make_fast(p.net), go = make_fast(p.occ);
    int32_t k_lo, k_hi;
    clip_ray(p.content, o, d, p.t_near, p.step, p.K, k_lo, k_hi);
    int32_t k = max(k_begin ? max(k_begin[r], 0) : 0, k_lo);
    int32_t *row = out_k + r * S;
    const uint32_t ray_key = kn_mix32(p.seed_key + (uint32_t)r);
    const int32_t n = march_group<OPT, MARCH_G>(p, gn, go, o, d, k, k_hi, S, gl, ray_key, [&](int j, int32_t kk, int32_t) { row[j] = kk; });
    for (int32_t j = n + gl; j < S; j += MARCH_G) row[j] = -1;
    if (gl == 0) {
        out_count[r] = n;
        if (out_k_next) out_k_next[r] = (k >= k_hi) ? p.K : k;
    }
}

// ---------------------------------------------------------------------------------------------
// render state
struct RayState {
    float *T;          // R
    float *C;          // R*3
    int32_t *k_next;   // R
    int32_t *k_end;    // R
};

constexpr int RAY_BLOCK = 256;  // threads per block of the two set-up kernels

// Sum over the blocks in front of this one of per-block counts written by the previous kernel
// (each thread takes a strided share; twelve loads of a thread are in flight together: one round trip for the 2,500
// blocks of an 800x800 frame, where batches of four were three).
__device__ __forceinline__ int32_t prefix_of_block_sums(const int32_t *__restrict__ blk_sum, int32_t *lds)
{
    constexpr int BATCH = 12;
    int32_t acc = 0;
    for (int b0 = 0; b0 < (int)blockIdx.x; b0 += RAY_BLOCK * BATCH) {
        int32_t v[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) v[u] = blk_sum[min(b0 + u * RAY_BLOCK + (int)threadIdx.x, (int)blockIdx.x)];
#pragma unroll
        for (int u = 0; u < BATCH; ++u)
            if (b0 + u * RAY_BLOCK + (int)threadIdx.x < (int)blockIdx.x) acc += v[u];
    }
    return kn_block_sum(acc, lds);
}

// clip every ray against the AABB and walk it to the first lattice point near content; rays that
// cannot produce a sample get the background right away.  Writes per-block counts of live rays.
template <int OPT>
__global__ void __launch_bounds__(RAY_BLOCK)
    k_render_init(MarchParams p, const float *__restrict__ rays_o, const float *__restrict__ rays_d, int64_t R, RayState s,
                  int32_t *__restrict__ alive, int32_t *__restrict__ blk_sum, float bg0, float bg1, float bg2,
                  float *__restrict__ rgb_out, int32_t *__restrict__ zero, int32_t n_zero, int32_t *__restrict__ hist,
                  int32_t n_hist, uint16_t *__restrict__ dir_table, int32_t dir_bf16)
{
    __shared__ int32_t lds[RAY_BLOCK / KN_WAVE];
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < n_zero) zero[r] = 0; // per-call counters
    if (r < n_hist) hist[r] = 0; // histogram of the sample grouping (kept zero by its consumer afterwards)
    int32_t lives = 0;
    if (r < R) {
        const float o[3] = {rays_o[3 * r], rays_o[3 * r + 1], rays_o[3 * r + 2]};
        const float d[3] = {rays_d[3 * r], rays_d[3 * r + 1], rays_d[3 * r + 2]};
        int32_t k_lo, k_hi;
        clip_ray(p.content, o, d, p.t_near, p.step, p.K, k_lo, k_hi);
        // walk through provably empty space up to the first lattice point that is near occupied blocks
        k_lo = skip_to_content<OPT>(p, make_fast(p.occ), o, d, k_lo, k_hi, kn_mix32(p.seed_key + (uint32_t)r));
        s.k_next[r] = k_lo;
        s.k_end[r] = k_hi;
        lives = k_lo < k_hi ? 1 : 0;
        alive[r] = lives;
        if (!lives) {
            rgb_out[3 * r] = bg0;
            rgb_out[3 * r + 1] = bg1;
            rgb_out[3 * r + 2] = bg2;
        } else if (dir_table) {
            // gamma(d) is the same for every sample of the ray: encoded once, in the grouped-MLP kernel's operand order
            kn_enc::u4 slots[4];
            if (dir_bf16) kn_enc::dir_slots<true>(d[0], d[1], d[2], slots);
            else kn_enc::dir_slots<false>(d[0], d[1], d[2], slots);
            kn_enc::u4 *dst = (kn_enc::u4 *)(dir_table + 32 * r);
#pragma unroll
            for (int g = 0; g < 4; ++g) dst[g] = slots[g];
        }
    }
    const int32_t total = kn_block_sum(lives, lds);
    if (threadIdx.x == 0) blk_sum[blockIdx.x] = total;
}

// Device-side description of a wave, written by the kernel that ends the previous one, so that the host can
// enqueue a wave before it knows how many rays are left: ctl[0] = rows of the live list, ctl[1] = S (samples
// per ray of this wave, = slots per row), ctl[2] = the schedule value S was derived from.
struct WaveSchedule {
    int32_t first, growth, K;
    int64_t budget; // slots shared by the live rays of a wave
};
__device__ __forceinline__ void set_wave(int32_t *ctl, int32_t n_rows, int32_t s_sched, const WaveSchedule &sched)
{
    int64_t S = s_sched;
    if (n_rows > 0 && S > sched.budget / n_rows) S = sched.budget / n_rows;
    if (S > sched.K) S = sched.K;
    if (S < 1) S = 1;
    ctl[0] = n_rows;
    ctl[1] = (int32_t)S;
    ctl[2] = s_sched;
}

// {value, then sequence number} into the host-visible mailbox; the host polls the sequence number
__device__ __forceinline__ void post_mailbox(unsigned long long *mailbox, unsigned long long seq, unsigned long long value)
{
    if (!mailbox) return;
    __hip_atomic_store(&mailbox[1], value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(&mailbox[0], seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// first live list: ray ids of the rays that survived k_render_init, in ascending order (same blocks
// as k_render_init; position = live rays in earlier blocks + rank inside the block)
__global__ void __launch_bounds__(RAY_BLOCK)
    k_first_live(const int32_t *__restrict__ alive, const int32_t *__restrict__ blk_sum, int64_t R,
                 int32_t *__restrict__ live_out, int32_t *__restrict__ alive_out, int32_t *__restrict__ n_live,
                 int32_t *__restrict__ ctl, WaveSchedule sched, unsigned long long *mailbox, unsigned long long seq)
{
    __shared__ int32_t lds[RAY_BLOCK / KN_WAVE];
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int32_t a = r < R ? alive[r] : 0; // (requested in front of the block sums: one round trip for both)
    const int32_t before = prefix_of_block_sums(blk_sum, lds);
    int32_t total;
    const int32_t pos = before + kn_block_exclusive_scan(a, lds, total);
    if (a) {
        live_out[pos] = (int32_t)r;
        alive_out[pos] = 1;
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        *n_live = before + total;
        set_wave(ctl, before + total, sched.first, sched);
        post_mailbox(mailbox, seq, (unsigned long long)(before + total));
    }
}

// G lanes per live ray: collect up to S kept samples into row i of the wave's row buffers.
// The workgroup also counts its samples per network in LDS (dynamic LDS: n_bins counters, or a hash table of
// 2 * hash_slots ints where a counter per network does not fit) and adds what it counted to the global histogram
// `hist` that the grouping of this wave starts from.
//
// From the second wave on (`blk_off` given) the kernel also compacts the live list while it reads it: it runs over
// the rows of the previous wave's list (`old_ctl`), the survivors among each group of 16 rows get the new row
// numbers blk_off[group] + rank (ascending, so the order of the list is kept), and the new list is written to
// live_out / alive_out.  blk_off comes from k_sum_partials (prefix sums of the survivor counts that the blend of
// the same 16-row groups left).
// HASH: the per-network counters are a hash table (large grids), else one counter per network.
// G: lanes per ray.  The kernel is bound by the latency of an iteration.  8 in the first wave, whose many rays stop
// after a few dozen samples: a wavefront keeps eight rays in flight, and a ray needs well under twice the iterations it
// would with 16 lanes (most iterations find few points to keep or none).  16 in later waves (few rays, long rows).
template <bool HASH, int OPT, int G>
__global__ void __launch_bounds__(256)
    k_march_wave(MarchParams p, const float *__restrict__ rays_o, const float *__restrict__ rays_d,
                 const int32_t *__restrict__ live, const int32_t *__restrict__ alive, const int32_t *__restrict__ ctl,
                 int32_t kbits, RayState s, int32_t *__restrict__ row_keys, uint32_t *__restrict__ row_rec,
                 int32_t *__restrict__ cnt, int32_t *__restrict__ hist, int32_t n_bins, int32_t hash_slots,
                 const int32_t *__restrict__ old_ctl, const int32_t *__restrict__ blk_off, const int32_t *__restrict__ grp_list,
                 int32_t *__restrict__ live_out, int32_t *__restrict__ alive_out)
{
    // per-network sample counters of the workgroup: one per network (hash_slots = 0: small grids), else a hash
    // table keyed by network (keys [hash_slots], then counts [hash_slots]; a power of two)
    extern __shared__ int32_t bins[];
    const int32_t n_lds = HASH ? 2 * hash_slots : n_bins;
    const int32_t n_in = blk_off ? old_ctl[0] : ctl[0]; // rows of the list that is read
    const int32_t S = ctl[1];
    constexpr int32_t T = 256, RAYS = T / G; // rays per workgroup
    constexpr int32_t GROUPS = RAYS / LIST_GROUP; // compaction groups per workgroup
    static_assert(RAYS % LIST_GROUP == 0, "a workgroup takes whole groups of rows");
    const int gl = threadIdx.x & (G - 1), lane = threadIdx.x & (KN_WAVE - 1);
    // (uniform exits: the grid is sized for an upper bound of the rows / of the groups with survivors)
    const int32_t n_groups = blk_off ? ctl[3] : 0;
    if (blk_off ? (int64_t)blockIdx.x * GROUPS >= n_groups : (int64_t)blockIdx.x * RAYS >= n_in) return;
    // Which ray this lane group marches, and its data, are requested before the counters are cleared: the dependent
    // loads (list entry -> ray number -> ray, resume point) are then in flight during the clearing and its barrier.
    int32_t i_in; // this ray's row in the list that is read
    bool lives;
    int32_t i;    // its row in the wave's buffers
    if (!blk_off) {
        i_in = (int32_t)(((int64_t)blockIdx.x * T + threadIdx.x) / G);
        lives = i_in < n_in && alive[i_in] != 0;
        i = i_in;
    } else {
        // The list is compacted in groups of LIST_GROUP = 16 rows (blk_off[g]: new row of group g's first survivor), and
        // the kernel runs over the groups that have survivors (grp_list, ctl[3] of them), so that the workgroups with
        // work are the first of the grid.  The 16 lanes of a DPP row fetch the flags of the group their row's ray belongs
        // to (8 lanes per ray: the two rays of a row are neighbours inside one group).
        const int32_t ray = threadIdx.x / G;                                  // ray of the workgroup
        const int64_t slot = (int64_t)blockIdx.x * GROUPS + ray / LIST_GROUP; // entry of the group list
        const int32_t g16 = slot < n_groups ? grp_list[slot] : -1;
        i_in = g16 >= 0 ? LIST_GROUP * g16 + (ray & (LIST_GROUP - 1)) : n_in;
        lives = i_in < n_in && alive[i_in] != 0;
        const int32_t q = LIST_GROUP * max(g16, 0) + (lane & (LIST_GROUP - 1));
        const bool f = g16 >= 0 && q < n_in && alive[q] != 0;
        const uint32_t flags = (uint32_t)(__ballot(f) >> (lane & ~(LIST_GROUP - 1))) & ((1u << LIST_GROUP) - 1u);
        i = lives ? blk_off[g16] + __popc(flags & ((1u << (i_in & (LIST_GROUP - 1))) - 1u)) : 0;
    }
    // (every lane loads: a retired or absent row reads the data of a valid list entry and drops it)
    const int32_t r = live[min(i_in, n_in - 1)];
    const float o[3] = {rays_o[3 * (int64_t)r], rays_o[3 * (int64_t)r + 1], rays_o[3 * (int64_t)r + 2]};
    const float d[3] = {rays_d[3 * (int64_t)r], rays_d[3 * (int64_t)r + 1], rays_d[3 * (int64_t)r + 2]};
    int32_t k = s.k_next[r];
    const int32_t k_hi = s.k_end[r];
    for (int32_t b = threadIdx.x; b < n_lds; b += T) bins[b] = (HASH && b < hash_slots) ? -1 : 0;
    __syncthreads();
    // one more sample of network `cell`
    auto count = [&](int32_t cell) {
        if constexpr (!HASH) {
            atomicAdd(&bins[cell], 1);
            return;
        }
        uint32_t h = ((uint32_t)cell * 2654435761u) >> (__builtin_clz((uint32_t)hash_slots) + 1);
        for (int probe = 0; probe < 8; ++probe) {
            int32_t old = bins[h];
            if (old == -1) old = atomicCAS(&bins[h], -1, cell);
            if (old == -1 || old == cell) {
                atomicAdd(&bins[hash_slots + h], 1);
                return;
            }
            h = (h + 1u) & (uint32_t)(hash_slots - 1);
        }
        atomicAdd(&hist[cell], 1); // no slot nearby: straight to the global histogram
    };
    if (!lives) {
        // without compaction retired rows stay in the list: they get no samples
        if (!blk_off && i_in < n_in && gl == 0) cnt[i_in] = 0;
    } else {
        if (blk_off && gl == 0) {
            live_out[i] = r;
            alive_out[i] = 1;
        }
        const GridFast gn = make_fast(p.net), go = make_fast(p.occ);
        int32_t *kr = row_keys + (int64_t)i * S;
        uint32_t *rr = row_rec + (int64_t)i * S;
        const uint32_t ray_key = kn_mix32(p.seed_key + (uint32_t)r);
        const int32_t n = march_group<OPT, G>(p, gn, go, o, d, k, k_hi, S, gl, ray_key, [&](int j, int32_t kk, int32_t cell) {
            kr[j] = cell;
            rr[j] = ((uint32_t)r << kbits) | (uint32_t)kk;
            count(cell);
        });
        if (gl == 0) {
            s.k_next[r] = k;
            cnt[i] = n;
        }
    }
    // the few bins this workgroup met go to the global histogram
    __syncthreads();
    const int32_t n_slots = HASH ? hash_slots : n_bins;
    for (int32_t b = threadIdx.x; b < n_slots; b += T) {
        const int32_t c = bins[(HASH ? hash_slots : 0) + b];
        if (c) atomicAdd(&hist[HASH ? bins[b] : b], c);
    }
}

// Eq. 2-4 over this wave's samples, early termination, retiring of finished rays.  A wavefront owns 32 consecutive
// rows (the kernel waits for its loads most of the time: with 64 rows per wavefront, half as many wavefronts, it
// takes 1.4 us longer; with 16 rows 0.4).  Its lanes fetch the rows' next BLEND_CHUNK samples together (BLEND_CHUNK lanes per row and request,
// consecutive addresses) and turn densities into alphas; the values go through LDS to the lane that owns the row, which runs
// the blend as the sequential recurrence of the definition: one lane per ray, the same operation order for every
// wave cut.  (Blending with 16 lanes per ray, all of them stepping through the recurrence on broadcast values, cost
// 16 times the instructions.)
// (16 samples per request: 70 KiB of LDS per workgroup, two wavefronts per SIMD, 3 us slower per frame; 4: too few loads in flight)
constexpr int BLEND_CHUNK = 8;
constexpr int BLEND_WAVE_ROWS = 32;                         // rows per wavefront: its first lanes own one each
constexpr int BLEND_ROWS = (256 / KN_WAVE) * BLEND_WAVE_ROWS; // rows per workgroup
__global__ void __launch_bounds__(256)
    k_composite_wave(const int32_t *__restrict__ live, const int32_t *__restrict__ ctl, int32_t rows_cap,
                     const int32_t *__restrict__ cnt, const float *__restrict__ out4, float step, float eps, float bg0,
                     float bg1, float bg2, RayState s, float *__restrict__ rgb_out, int32_t *__restrict__ alive,
                     int32_t *__restrict__ partials /*2 * gridDim.x: evaluated, blended*/,
                     int32_t *__restrict__ surv16 /*survivors per group of 16 rows*/, int32_t *__restrict__ zero,
                     int32_t n_zero, int32_t first_wave)
{
    // counters of the grouping that the next wave expects to be zero
    for (int64_t z = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; z < n_zero; z += (int64_t)gridDim.x * blockDim.x) zero[z] = 0;
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ f4 stage[256 / KN_WAVE][BLEND_WAVE_ROWS][BLEND_CHUNK + 1]; // + 1: the owner lanes' reads spread over the banks
    const int32_t n_live = ctl[0], S = ctl[1];
    const int wave = threadIdx.x / KN_WAVE, lane = threadIdx.x & (KN_WAVE - 1);
    const int32_t row0 = (int32_t)blockIdx.x * BLEND_ROWS + wave * BLEND_WAVE_ROWS; // first row of this wavefront
    const bool owner = lane < BLEND_WAVE_ROWS;
    const int32_t i = row0 + lane;
    // the grid covers rows_cap >= n_live rows; the flags of the rows beyond the list are cleared so that the next
    // wave's compaction can run over the same upper bound
    if (owner && i >= n_live && i < rows_cap) alive[i] = 0;
    // (flag, ray number and sample count of the row are requested together, from a valid row whatever the lane: taken one
    // after the other, each behind the test of the one before, they were three round trips in front of the first samples)
    const int32_t i_safe = max(min(i, n_live - 1), 0);
    const int32_t alive_i = alive[i_safe], live_i = live[i_safe], cnt_i = cnt[i_safe];
    const bool mine = owner && i < n_live && alive_i != 0;
    const int32_t r = mine ? live_i : 0;
    const int32_t n = mine ? cnt_i : 0;
    float T = 1.0f, c0 = 0.0f, c1 = 0.0f, c2 = 0.0f; // the state of a ray before its first wave
    if (mine && !first_wave) {
        T = s.T[r];
        c0 = s.C[3 * (int64_t)r];
        c1 = s.C[3 * (int64_t)r + 1];
        c2 = s.C[3 * (int64_t)r + 2];
    }
    bool dead = false;
    int32_t blended = 0;
    constexpr int LOADS = BLEND_WAVE_ROWS / (KN_WAVE / BLEND_CHUNK); // requests per lane and chunk
    const int sub = lane / BLEND_CHUNK, jl = lane % BLEND_CHUNK; // loader role: rows sub, sub + 64 / BLEND_CHUNK, ...; sample jl of the chunk
    for (int32_t j0 = 0; __ballot(mine && !dead && j0 < n) != 0ull; j0 += BLEND_CHUNK) {
        // fetch: KN_WAVE / BLEND_CHUNK rows per request, all requests issued before the first use
        f4 v[LOADS];
#pragma unroll
        for (int q = 0; q < LOADS; ++q) {
            const int rl = q * (KN_WAVE / BLEND_CHUNK) + sub;        // row of the wavefront this lane loads for
            const int32_t n_l = __shfl(n, rl, KN_WAVE);
            const int32_t gone = __shfl((int32_t)dead, rl, KN_WAVE);
            const bool need = j0 + jl < n_l && !gone;
            const int64_t at = (int64_t)min(row0 + rl, n_live - 1) * S + min(j0 + jl, S - 1); // always a slot of the wave
            // (only what the blend will use is requested: the kernel moves data at the rate of a device copy, and the
            // samples behind a ray's termination point are a third of the wave's)
            v[q] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
            if (need) v[q] = ((const f4 *)out4)[at];
        }
        __builtin_amdgcn_wave_barrier(); // the owners have finished reading the previous chunk
#pragma unroll
        for (int q = 0; q < LOADS; ++q) {
            v[q][3] = 1.0f - expf(-v[q][3] * step); // alpha (Eq. 4)
            stage[wave][q * (KN_WAVE / BLEND_CHUNK) + sub][jl] = v[q];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // blend: lane = row
        const int m = min(BLEND_CHUNK, n - j0);
        for (int u = 0; u < BLEND_CHUNK; ++u) {
            if (__ballot(mine && !dead && u < m) == 0ull) break;
            if (mine && !dead && u < m) {
                const f4 q = stage[wave][lane][u];
                const float wgt = T * q[3];
                c0 = fmaf(wgt, q[0], c0);
                c1 = fmaf(wgt, q[1], c1);
                c2 = fmaf(wgt, q[2], c2);
                T *= (1.0f - q[3]);
                ++blended;
                if (eps > 0.0f && T < eps) dead = true;
            }
        }
    }
    bool lives = false;
    if (mine) {
        const bool exhausted = s.k_next[r] >= s.k_end[r];
        lives = !dead && !exhausted;
        if (lives) {
            s.T[r] = T;
            s.C[3 * (int64_t)r] = c0;
            s.C[3 * (int64_t)r + 1] = c1;
            s.C[3 * (int64_t)r + 2] = c2;
        } else {
            rgb_out[3 * (int64_t)r] = fmaf(T, bg0, c0);
            rgb_out[3 * (int64_t)r + 1] = fmaf(T, bg1, c1);
            rgb_out[3 * (int64_t)r + 2] = fmaf(T, bg2, c2);
            alive[i] = 0;
        }
    }
    // survivors per group of 16 rows (the next wave's march compacts the list in those groups)
    {
        const unsigned long long sv = __ballot(lives);
        if (lane < BLEND_WAVE_ROWS / MARCH_G) {
            const int32_t grp = row0 / MARCH_G + lane;
            if ((int64_t)grp * MARCH_G < rows_cap) surv16[grp] = __builtin_popcountll((sv >> (MARCH_G * lane)) & ((1ull << MARCH_G) - 1ull));
        }
    }
    // block-level sums -> one plain store per block and counter (same-address atomics from tens of
    // thousands of wavefronts would serialise); k_sum_partials adds them up afterwards
    int32_t evaluated = n;
    __shared__ int32_t red[2][256 / KN_WAVE];
    blended = __builtin_amdgcn_readlane(kn_wave_inclusive_scan(blended), KN_WAVE - 1); // (all lanes are back together here)
    evaluated = __builtin_amdgcn_readlane(kn_wave_inclusive_scan(evaluated), KN_WAVE - 1);
    if (lane == 0) {
        red[0][wave] = evaluated;
        red[1][wave] = blended;
    }
    __syncthreads();
    if (threadIdx.x < 2) {
        int32_t t = 0;
#pragma unroll
        for (int w = 0; w < 256 / KN_WAVE; ++w) t += red[threadIdx.x][w];
        partials[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] = t;
    }
}

// The same blend with MARCH_G lanes per live ray, for waves of few rays with many samples each (the rest of a ray):
// Eq. 2-4 over this wave's samples, early termination, retiring of finished rays.  The lanes fetch 16 consecutive samples and turn densities into alphas in parallel; the
// blend itself is the sequential recurrence of the definition (same operation order for every
// wave cut), run redundantly by all lanes of the group on values broadcast through LDS.
__global__ void __launch_bounds__(256)
    k_composite_group(const int32_t *__restrict__ live, const int32_t *__restrict__ ctl, int32_t rows_cap,
                     const int32_t *__restrict__ cnt, const float *__restrict__ out4, float step, float eps, float bg0,
                     float bg1, float bg2, RayState s, float *__restrict__ rgb_out, int32_t *__restrict__ alive,
                     int32_t *__restrict__ partials /*2 * gridDim.x: evaluated, blended*/,
                     int32_t *__restrict__ surv16 /*survivors per group of 16 rows = per workgroup*/,
                     int32_t *__restrict__ zero, int32_t n_zero, int32_t first_wave)
{
    // counters of the grouping that the next wave expects to be zero
    for (int64_t z = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; z < n_zero; z += (int64_t)gridDim.x * blockDim.x) zero[z] = 0;
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ f4 stage[256];
    const int32_t n_live = ctl[0], S = ctl[1];
    const int32_t i = (int32_t)(((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / MARCH_G);
    const int gl = threadIdx.x & (MARCH_G - 1);
    f4 *grp_stage = stage + (threadIdx.x & ~(MARCH_G - 1));
    int32_t blended = 0, evaluated = 0, survivors = 0;
    // the grid covers rows_cap >= n_live rows; the flags of the rows beyond the list are cleared so that the
    // compaction that follows can run over the same upper bound
    // (flag, ray number, sample count and the first samples of the row are requested together, from a valid row whatever
    // the lane: one round trip in front of the loop instead of three)
    const int32_t i_safe = max(min(i, n_live - 1), 0);
    const int32_t alive_i = alive[i_safe], live_i = live[i_safe], cnt_i = cnt[i_safe];
    const f4 first = ((const f4 *)out4)[(int64_t)i_safe * S + min(gl, S - 1)];
    if (i >= n_live && i < rows_cap && gl == 0) alive[i] = 0;
    if (i < n_live && alive_i) {
        const int32_t r = live_i;
        const int32_t n = cnt_i;
        const f4 *smp = (const f4 *)out4 + (int64_t)i * S; // row i of the wave's slots
        float T = 1.0f, c0 = 0.0f, c1 = 0.0f, c2 = 0.0f; // the state of a ray before its first wave
        if (!first_wave) {
            T = s.T[r];
            c0 = s.C[3 * (int64_t)r];
            c1 = s.C[3 * (int64_t)r + 1];
            c2 = s.C[3 * (int64_t)r + 2];
        }
        bool dead = false;
        f4 v_next = gl < n ? first : (f4){0.0f, 0.0f, 0.0f, 0.0f};
        for (int32_t j0 = 0; j0 < n && !dead; j0 += MARCH_G) {
            f4 v = v_next;
            // the following 16 samples are requested before these are blended (clamped address: always a valid slot of
            // the row buffer; the value is only used for j < n)
            const int32_t jn = j0 + MARCH_G + gl;
            v_next = smp[min(jn, S - 1)];
            if (jn >= n) v_next = (f4){0.0f, 0.0f, 0.0f, 0.0f};
            v[3] = 1.0f - expf(-v[3] * step); // alpha (Eq. 4)
            __builtin_amdgcn_wave_barrier();
            grp_stage[gl] = v;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int m = min(MARCH_G, n - j0);
            for (int u = 0; u < m; ++u) {
                const f4 q = grp_stage[u];
                const float wgt = T * q[3];
                c0 = fmaf(wgt, q[0], c0);
                c1 = fmaf(wgt, q[1], c1);
                c2 = fmaf(wgt, q[2], c2);
                T *= (1.0f - q[3]);
                ++blended;
                if (eps > 0.0f && T < eps) { dead = true; break; }
            }
        }
        const bool exhausted = s.k_next[r] >= s.k_end[r];
        const bool lives = !dead && !exhausted;
        if (gl == 0) {
            evaluated = n;
            if (lives) {
                s.T[r] = T;
                s.C[3 * (int64_t)r] = c0;
                s.C[3 * (int64_t)r + 1] = c1;
                s.C[3 * (int64_t)r + 2] = c2;
                survivors = 1;
            } else {
                rgb_out[3 * (int64_t)r] = fmaf(T, bg0, c0);
                rgb_out[3 * (int64_t)r + 1] = fmaf(T, bg1, c1);
                rgb_out[3 * (int64_t)r + 2] = fmaf(T, bg2, c2);
                alive[i] = 0;
            }
        } else {
            blended = 0;
        }
    }
    // block-level sums -> one plain store per block and counter (same-address atomics from tens of
    // thousands of wavefronts would serialise); k_sum_partials adds them up afterwards
    __shared__ int32_t red[3][256 / KN_WAVE];
    blended = __builtin_amdgcn_readlane(kn_wave_inclusive_scan(blended), KN_WAVE - 1); // (all lanes are back together here)
    evaluated = __builtin_amdgcn_readlane(kn_wave_inclusive_scan(evaluated), KN_WAVE - 1);
    survivors = __builtin_amdgcn_readlane(kn_wave_inclusive_scan(survivors), KN_WAVE - 1);
    if ((threadIdx.x & (KN_WAVE - 1)) == 0) {
        red[0][threadIdx.x / KN_WAVE] = evaluated;
        red[1][threadIdx.x / KN_WAVE] = blended;
        red[2][threadIdx.x / KN_WAVE] = survivors;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        int32_t v = 0;
#pragma unroll
        for (int w = 0; w < 256 / KN_WAVE; ++w) v += red[threadIdx.x][w];
        if (threadIdx.x == 2) surv16[blockIdx.x] = v;
        else partials[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] = v;
    }
}

// one block: counters[0] += evaluated, counters[1] += blended, counters[2] = survivors of this wave
// ... counters[3] += slots of this wave, counters[4] += 1 if the wave had rows; writes the next wave's control
// partials: evaluated and blended samples per workgroup of the blend (2 * n_cb); surv16: survivors per group of 16
// rows (n_blocks groups)
__global__ void __launch_bounds__(1024) k_sum_partials(const int32_t *__restrict__ partials, int32_t n_cb,
                                                        const int32_t *__restrict__ surv16, int32_t n_blocks,
                                                        unsigned long long *__restrict__ counters,
                                                        const int32_t *__restrict__ ctl, int32_t *__restrict__ ctl_next,
                                                        WaveSchedule sched, int32_t *__restrict__ blk_off,
                                                        int32_t *__restrict__ grp_list,
                                                        unsigned long long *mailbox, unsigned long long seq)
{
    // This kernel sits alone between the blend and the next wave's march: what counts is its latency.  Every value is
    // requested once, as early as possible, and each thread scans 16 contiguous entries (one 64-byte line) itself.
    constexpr int T = 1024, PER = 16;
    typedef int32_t i4 __attribute__((ext_vector_type(4)));
    __shared__ int32_t lds[T / KN_WAVE], lds_with[T / KN_WAVE];
    __shared__ unsigned long long red[2][T / KN_WAVE];
    const int tid = threadIdx.x;
    int32_t rows = 0, slots_per_row = 0, s_sched = 0;
    unsigned long long tot_eval = 0ull, tot_blend = 0ull, tot_slots = 0ull, tot_waves = 0ull;
    if (tid == 0) { // the scalars of the closing thread
        rows = ctl[0];
        slots_per_row = ctl[1];
        s_sched = ctl[2];
        tot_eval = counters[0];
        tot_blend = counters[1];
        tot_slots = counters[3];
        tot_waves = counters[4];
    }
    unsigned long long ev = 0ull, bl = 0ull;
    for (int32_t b = tid; b < n_cb; b += T) {
        ev += (unsigned long long)partials[b];
        bl += (unsigned long long)partials[(int64_t)n_cb + b];
    }
    // exclusive prefix sums of the survivors per 16-row group: the next wave's march compacts the list with them.
    // grp_list: the groups that have survivors, ascending; the next march runs over those only (ctl_next[3] of them),
    // so that its workgroups with work are the first of its grid and start at once, not spread among four times as
    // many that find their 16 rows retired.
    int32_t survivors = 0, live_groups = 0;
    for (int32_t b0 = 0; b0 < n_blocks; b0 += T * PER) {
        const int32_t e0 = b0 + PER * tid;
        const bool full = e0 + PER <= n_blocks;
        int32_t v[PER];
        if (full) {
#pragma unroll
            for (int u = 0; u < PER / 4; ++u) {
                const i4 q = *(const i4 *)(surv16 + e0 + 4 * u);
                v[4 * u] = q[0]; v[4 * u + 1] = q[1]; v[4 * u + 2] = q[2]; v[4 * u + 3] = q[3];
            }
        } else {
#pragma unroll
            for (int u = 0; u < PER; ++u) v[u] = e0 + u < n_blocks ? surv16[e0 + u] : 0;
        }
        int32_t sum = 0, with = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            sum += v[u];
            with += v[u] > 0 ? 1 : 0;
        }
        // both prefix sums with one pair of barriers
        const int32_t inc_sum = kn_wave_inclusive_scan(sum), inc_with = kn_wave_inclusive_scan(with);
        __syncthreads();
        if ((tid & (KN_WAVE - 1)) == KN_WAVE - 1) {
            lds[tid / KN_WAVE] = inc_sum;
            lds_with[tid / KN_WAVE] = inc_with;
        }
        __syncthreads();
        int32_t total = 0, total_with = 0, off = survivors + inc_sum - sum, at = live_groups + inc_with - with;
#pragma unroll
        for (int w = 0; w < T / KN_WAVE; ++w) {
            const int32_t a = lds[w], b = lds_with[w];
            total += a;
            total_with += b;
            if (w < tid / KN_WAVE) {
                off += a;
                at += b;
            }
        }
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int32_t c = v[u];
            if (c > 0) grp_list[at++] = e0 + u;
            v[u] = off;
            off += c;
        }
        live_groups += total_with;
        if (full) {
#pragma unroll
            for (int u = 0; u < PER / 4; ++u) *(i4 *)(blk_off + e0 + 4 * u) = (i4){v[4 * u], v[4 * u + 1], v[4 * u + 2], v[4 * u + 3]};
        } else {
#pragma unroll
            for (int u = 0; u < PER; ++u)
                if (e0 + u < n_blocks) blk_off[e0 + u] = v[u];
        }
        survivors += total;
    }
    // (a wave's samples fit 31 bits: the slots of a wave do)
    ev = (unsigned long long)(uint32_t)__builtin_amdgcn_readlane(kn_wave_inclusive_scan((int32_t)ev), KN_WAVE - 1);
    bl = (unsigned long long)(uint32_t)__builtin_amdgcn_readlane(kn_wave_inclusive_scan((int32_t)bl), KN_WAVE - 1);
    if ((tid & (KN_WAVE - 1)) == 0) {
        red[0][tid / KN_WAVE] = ev;
        red[1][tid / KN_WAVE] = bl;
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 0; w < T / KN_WAVE; ++w) {
            tot_eval += red[0][w];
            tot_blend += red[1][w];
        }
        tot_slots += (unsigned long long)rows * (unsigned long long)slots_per_row;
        tot_waves += rows > 0 ? 1ull : 0ull;
        counters[0] = tot_eval;
        counters[1] = tot_blend;
        counters[2] = (unsigned long long)survivors;
        counters[3] = tot_slots;
        counters[4] = tot_waves;
        // the next wave: the survivors (the live list is compacted in between), schedule value grown
        const int64_t grown = (int64_t)s_sched * sched.growth;
        set_wave(ctl_next, survivors, (int32_t)(grown < sched.K ? grown : sched.K), sched);
        ctl_next[3] = live_groups;
        // running totals ride along so that the host never has to read the counters back
        if (mailbox) {
            __hip_atomic_store(&mailbox[2], tot_eval, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(&mailbox[3], tot_blend, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(&mailbox[4], tot_slots, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(&mailbox[5], tot_waves, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        post_mailbox(mailbox, seq, (unsigned long long)survivors);
    }
}

// stage kernel behind kn_composite: explicit per-ray sample ranges
// (delta: a spacing per sample, or nullptr for the constant `step`)
__global__ void k_composite_stage(const float *__restrict__ sigma, const float *__restrict__ rgb,
                                  const float *__restrict__ delta,
                                  const int32_t *__restrict__ offsets, int64_t R, float step, float eps, float bg0,
                                  float bg1, float bg2, float *__restrict__ rgb_out, float *__restrict__ T_out,
                                  int32_t *__restrict__ n_used)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    float T = 1.0f, c0 = 0.0f, c1 = 0.0f, c2 = 0.0f;
    int32_t used = 0;
    for (int32_t j = offsets[r]; j < offsets[r + 1]; ++j) {
        const float alpha = 1.0f - expf(-sigma[j] * (delta ? delta[j] : step));
        const float wgt = T * alpha;
        c0 = fmaf(wgt, rgb[3 * (int64_t)j], c0);
        c1 = fmaf(wgt, rgb[3 * (int64_t)j + 1], c1);
        c2 = fmaf(wgt, rgb[3 * (int64_t)j + 2], c2);
        T *= (1.0f - alpha);
        ++used;
        if (eps > 0.0f && T < eps) break;
    }
    rgb_out[3 * r] = fmaf(T, bg0, c0);
    rgb_out[3 * r + 1] = fmaf(T, bg1, c1);
    rgb_out[3 * r + 2] = fmaf(T, bg2, c2);
    if (T_out) T_out[r] = T;
    if (n_used) n_used[r] = used;
}

MarchParams make_params(const kn_scene *sc, float t_near, float step, int32_t K, const uint32_t *seed = nullptr)
{
    MarchParams p;
    p.cell_net = sc->cell_net;
    p.seed_key = seed ? kn_mix32(*seed) : 0u;
    p.net = sc->net_grid;
    p.occ = sc->has_occ ? sc->occ_grid : sc->net_grid;
    p.content = sc->content_box;
    p.occ_bits = sc->occ_bits;
    p.has_occ = sc->has_occ ? 1 : 0;
    p.skip_dist = sc->has_occ ? sc->skip_dist : nullptr;
    p.skip_edge_min = INFINITY;
    float mag = 0.0f;
    for (int a = 0; a < 3; ++a) {
        p.skip_res[a] = sc->skip_res[a];
        const float edge = p.occ.cell[a] * (float)KN_SKIP_BLOCK;
        p.skip_inv[a] = 1.0f / edge;
        p.skip_edge_min = fminf(p.skip_edge_min, edge);
        mag = fmaxf(mag, fabsf(p.occ.bmin[a]) + p.occ.cell[a] * (float)p.occ.res[a]);
    }
    p.skip_margin = 1e-3f * p.skip_edge_min + 4e-6f * mag;
    for (int a = 0; a < 3; ++a) {
        int sft = -1;
        if (sc->has_occ)
            for (int q = 0; q < 16; ++q)
                if ((int64_t)p.net.res[a] << q == (int64_t)p.occ.res[a]) sft = q;
        p.net_shift[a] = sft;
    }
    if (p.net_shift[0] < 0 || p.net_shift[1] < 0 || p.net_shift[2] < 0) p.net_shift[0] = p.net_shift[1] = p.net_shift[2] = -1;
    p.t_near = t_near;
    p.step = step;
    p.K = K;
    return p;
}

// Wave schedule.  Most rays end (early termination or leaving the content) within their first few dozen
// kept samples, and a wave costs several kernel launches whatever its size: a generous first wave and one
// large step afterwards (the rest of the ray for the few survivors) measured fastest at 800x800.  Finer
// lattices need proportionally more samples to saturate a ray: unless set explicitly, the first wave takes
// max(48, K / 16) samples per ray (1920x1080 with K = 1024: 64 instead of 48 saves 11 %).  The slot
// budget (slots per ray of the frame, shared by the live rays of a wave) only sizes the workspace; when it
// covers K slots for every ray that reaches content, the second wave is known to finish the frame and the
// call returns without waiting for it.
constexpr int DEFAULT_FIRST_WAVE = 48;

bool finite_pos(float v) { return isfinite(v) && v > 0.0f; }

// kernel variants for a scene and a sampling mode
int march_options(const kn_scene *sc, const uint32_t *seed) { return (sc->cell_net ? OPT_SPARSE : 0) | (seed ? OPT_STRAT : 0); }
using MarchStageFn = decltype(&k_march_stage<0>);
using RenderInitFn = decltype(&k_render_init<0>);
MarchStageFn march_stage_kernel(int opt)
{
    static const MarchStageFn table[4] = {k_march_stage<0>, k_march_stage<1>, k_march_stage<2>, k_march_stage<3>};
    return table[opt & 3];
}
RenderInitFn render_init_kernel(int opt)
{
    return (opt & OPT_STRAT) ? k_render_init<OPT_STRAT> : k_render_init<0>; // the table of a sparse grid plays no role here
}
constexpr int MARCH_G_NARROW = 8, MARCH_G_WIDE = 16; // lanes per ray in waves of short rows / of long rows
using MarchWaveFn = decltype(&k_march_wave<false, 0, MARCH_G_WIDE>);
MarchWaveFn march_wave_kernel(bool hash, int opt, bool narrow)
{
    static const MarchWaveFn table[2][2][4] = {
        {{k_march_wave<false, 0, MARCH_G_WIDE>, k_march_wave<false, 1, MARCH_G_WIDE>, k_march_wave<false, 2, MARCH_G_WIDE>,
          k_march_wave<false, 3, MARCH_G_WIDE>},
         {k_march_wave<true, 0, MARCH_G_WIDE>, k_march_wave<true, 1, MARCH_G_WIDE>, k_march_wave<true, 2, MARCH_G_WIDE>,
          k_march_wave<true, 3, MARCH_G_WIDE>}},
        {{k_march_wave<false, 0, MARCH_G_NARROW>, k_march_wave<false, 1, MARCH_G_NARROW>, k_march_wave<false, 2, MARCH_G_NARROW>,
          k_march_wave<false, 3, MARCH_G_NARROW>},
         {k_march_wave<true, 0, MARCH_G_NARROW>, k_march_wave<true, 1, MARCH_G_NARROW>, k_march_wave<true, 2, MARCH_G_NARROW>,
          k_march_wave<true, 3, MARCH_G_NARROW>}}};
    return table[narrow ? 1 : 0][hash ? 1 : 0][opt & 3];
}

} // namespace

// A mailbox for a call on `stream`: the one the stream already has, else a free one, else the least recently used one
// whose last call has reported (the device writes a mailbox only up to the last post a call asked for, so once that
// sequence number is visible nothing of the old owner is in flight).  nullptr when none can be had: the call then
// waits for its stream instead of polling.
static KnMailbox *mailbox_for(kn_ctx *ctx, hipStream_t stream)
{
    std::lock_guard<std::mutex> lock(ctx->mutex);
    KnMailbox *pick = nullptr;
    for (auto &m : ctx->mailbox) {
        if (!m.host) return nullptr;
        if (m.taken && m.stream == stream) { pick = &m; break; }
    }
    if (!pick)
        for (auto &m : ctx->mailbox)
            if (!m.taken) { pick = &m; break; }
    if (!pick)
        for (auto &m : ctx->mailbox) {
            const bool idle = __atomic_load_n((const unsigned long long *)&m.host[0], __ATOMIC_ACQUIRE) == m.last_posted;
            if (idle && (!pick || m.last_use < pick->last_use)) pick = &m;
        }
    if (pick) {
        pick->taken = true;
        pick->stream = stream;
        pick->last_use = ++ctx->use_counter;
    }
    return pick;
}

// Wait for the mailbox to show `seq` (spinning on pinned memory is much cheaper than draining the
// stream); falls back to a stream synchronise + device read when there is no mailbox or it stays silent.
static int wait_count(const KnMailbox *mb, hipStream_t st, unsigned long long seq, const void *dev_value, size_t dev_bytes,
                      long long *out)
{
    if (mb) {
        const auto t0 = std::chrono::steady_clock::now();
        long long spins = 0;
        while (true) {
            if (__atomic_load_n((const unsigned long long *)&mb->host[0], __ATOMIC_ACQUIRE) == seq) {
                *out = (long long)__atomic_load_n((const unsigned long long *)&mb->host[1], __ATOMIC_RELAXED);
                return KN_OK;
            }
            if ((++spins & 0x3ff) == 0) {
                if (hipStreamQuery(st) == hipSuccess && // stream drained: the post is there or will never come
                    __atomic_load_n((const unsigned long long *)&mb->host[0], __ATOMIC_ACQUIRE) != seq)
                    break;
                if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(20)) break;
            }
        }
    }
    unsigned long long v64 = 0;
    int32_t v32 = 0;
    KN_HIP(hipMemcpyAsync(dev_bytes == 8 ? (void *)&v64 : (void *)&v32, dev_value, dev_bytes, hipMemcpyDeviceToHost, st));
    KN_HIP(hipStreamSynchronize(st));
    *out = dev_bytes == 8 ? (long long)v64 : (long long)v32;
    return KN_OK;
}

static int kbits_for(int32_t K)
{
    int b = 1;
    while ((1 << b) < K) ++b;
    return b;
}

// layout of the render workspace
struct RenderWs {
    int32_t *partials, *surv16, *blk_sum, *blk_off, *grp_list, *live_a, *live_b, *cnt, *alive_a, *alive_b, *n_live_dev, *row_keys, *ctl;
    uint32_t *row_rec;
    float *T, *C, *out4;
    int32_t *k_next, *k_end;
    unsigned long long *counters;
    uint16_t *dir_table; // 32 halfs per ray (16-bit scenes)
};

static void carve_render(KnCarver &ws, int64_t R, int64_t slots, RenderWs &w)
{
    w.partials = ws.carve<int32_t>(2 * kn_div_up(R, MARCH_G));
    w.surv16 = ws.carve<int32_t>(kn_div_up(R, MARCH_G));
    w.blk_sum = ws.carve<int32_t>(kn_div_up(R, RAY_BLOCK) + 1);
    w.blk_off = ws.carve<int32_t>(kn_div_up(R, LIST_GROUP));
    w.grp_list = ws.carve<int32_t>(kn_div_up(R, LIST_GROUP));
    w.live_a = ws.carve<int32_t>(R);
    w.live_b = ws.carve<int32_t>(R);
    w.cnt = ws.carve<int32_t>(R);
    w.alive_a = ws.carve<int32_t>(R);
    w.alive_b = ws.carve<int32_t>(R);
    w.n_live_dev = ws.carve<int32_t>(1);
    w.T = ws.carve<float>(R);
    w.C = ws.carve<float>(3 * R);
    w.k_next = ws.carve<int32_t>(R);
    w.k_end = ws.carve<int32_t>(R);
    w.counters = ws.carve<unsigned long long>(8);
    w.ctl = ws.carve<int32_t>(8); // two wave-control blocks of 4 ints, used alternately
    w.row_keys = ws.carve<int32_t>(slots);
    w.row_rec = ws.carve<uint32_t>(slots);
    w.out4 = ws.carve<float>(4 * slots);
    w.dir_table = ws.carve<uint16_t>(32 * R);
}

int64_t kn_render_ws_bytes(const kn_scene *sc, int64_t R, int32_t slots_per_ray)
{
    KnCarver c((void *)256, INT64_MAX / 2);
    RenderWs w;
    const int64_t slots = R * slots_per_ray;
    carve_render(c, R, slots, w);
    return c.used + kn_group_ws_bytes(slots, sc->N);
}

static int march_impl(const kn_scene *sc, void *stream, const float *rays_o, const float *rays_d, int64_t R, float t_near,
                      float step, int32_t K, const uint32_t *seed, const int32_t *k_begin, int32_t S, int32_t *out_k,
                      int32_t *out_count, int32_t *out_k_next)
{
    if (!sc || R < 0 || K < 0 || S < 1 || !isfinite(t_near) || !finite_pos(step)) return KN_E_INVALID_ARG;
    if (R > 0 && (!rays_o || !rays_d || !out_k || !out_count)) return KN_E_INVALID_ARG;
    if (R == 0) return KN_OK;
    const int64_t blocks = kn_div_up(R * MARCH_G, 256);
    if (blocks > 0x7fffffffLL) return KN_E_UNSUPPORTED;
    if (seed && R > 0xffffffffLL) return KN_E_UNSUPPORTED; // ray numbers are 32-bit
    hipLaunchKernelGGL(march_stage_kernel(march_options(sc, seed)), dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       make_params(sc, t_near, step, K, seed), rays_o, rays_d, R, k_begin, S, out_k, out_count, out_k_next);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

extern "C" int kn_march(const kn_scene *sc, void *stream, const float *rays_o, const float *rays_d, int64_t R, float t_near,
                        float step, int32_t K, const int32_t *k_begin, int32_t S, int32_t *out_k, int32_t *out_count,
                        int32_t *out_k_next)
{
    return march_impl(sc, stream, rays_o, rays_d, R, t_near, step, K, nullptr, k_begin, S, out_k, out_count, out_k_next);
}

extern "C" int kn_march_stratified(const kn_scene *sc, void *stream, const float *rays_o, const float *rays_d, int64_t R,
                                   float t_near, float step, int32_t K, uint32_t seed, const int32_t *k_begin, int32_t S,
                                   int32_t *out_k, int32_t *out_count, int32_t *out_k_next)
{
    return march_impl(sc, stream, rays_o, rays_d, R, t_near, step, K, &seed, k_begin, S, out_k, out_count, out_k_next);
}

static int composite_impl(void *stream, const float *sigma, const float *rgb, const float *delta, const int32_t *offsets,
                          int64_t R, float step, float term_eps, const float bg[3], float *rgb_out, float *T_out,
                          int32_t *n_used)
{
    if (R < 0 || !bg || !finite_pos(step) || !(term_eps >= 0.0f && term_eps < 1.0f)) return KN_E_INVALID_ARG;
    if (R > 0 && (!offsets || !rgb_out)) return KN_E_INVALID_ARG; // sigma / rgb may be NULL when no ray has samples
    if (R == 0) return KN_OK;
    if (kn_div_up(R, 256) > 0x7fffffffLL) return KN_E_UNSUPPORTED;
    hipLaunchKernelGGL(k_composite_stage, dim3((unsigned)kn_div_up(R, 256)), dim3(256), 0, (hipStream_t)stream, sigma, rgb,
                       delta, offsets, R, step, term_eps, bg[0], bg[1], bg[2], rgb_out, T_out, n_used);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

extern "C" int kn_composite(void *stream, const float *sigma, const float *rgb, const int32_t *offsets, int64_t R,
                            float step, float term_eps, const float bg[3], float *rgb_out, float *T_out, int32_t *n_used)
{
    return composite_impl(stream, sigma, rgb, nullptr, offsets, R, step, term_eps, bg, rgb_out, T_out, n_used);
}

extern "C" int kn_composite_deltas(void *stream, const float *sigma, const float *rgb, const float *delta,
                                   const int32_t *offsets, int64_t R, float term_eps, const float bg[3], float *rgb_out,
                                   float *T_out, int32_t *n_used)
{
    // (delta may be NULL only when no ray has samples, like sigma and rgb; the kernel then never reads it)
    return composite_impl(stream, sigma, rgb, delta, offsets, R, 1.0f, term_eps, bg, rgb_out, T_out, n_used);
}

static int render_impl(kn_ctx *ctx, const kn_scene *sc, void *stream, const float *rays_o, const float *rays_d, int64_t R, float t_near,
                       float step, int32_t K, float term_eps, const float bg[3], const uint32_t *seed, float *rgb_out,
                       kn_render_stats *stats, void *workspace, int64_t workspace_bytes)
{
    if (!ctx || !sc || R < 0 || K < 0 || !bg || !isfinite(t_near) || !finite_pos(step) || !(term_eps >= 0.0f && term_eps < 1.0f))
        return KN_E_INVALID_ARG;
    if (R > 0 && (!rays_o || !rays_d || !rgb_out)) return KN_E_INVALID_ARG;
    if (stats) {
        stats->rays = R;
        stats->waves = stats->samples_evaluated = stats->samples_blended = stats->slots = 0;
    }
    if (R == 0) return KN_OK;
    const KnKnobs knobs = kn_knobs(ctx); // the schedule this call runs with, whatever is set meanwhile
    const int kbits = kbits_for(K > 1 ? K : 2);
    if (R > (1ll << (32 - kbits)) || R > 0x7fffffffLL / knobs.slots_per_ray || R > (1ll << 26))
        return KN_E_UNSUPPORTED; // slot numbers, row * lanes and byte offsets into the table of encoded directions are 32-bit
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < kn_render_ws_bytes(sc, R, knobs.slots_per_ray))
        return KN_E_WORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    KnCarver ws(workspace, workspace_bytes);
    RenderWs w;
    const int64_t budget = R * knobs.slots_per_ray;
    carve_render(ws, R, budget, w);
    if (!ws.ok()) return KN_E_WORKSPACE;
    KnGroupWs gw;
    kn_group_carve(ws, budget, sc->N, &gw);
    if (!ws.ok()) return KN_E_WORKSPACE;

    const MarchParams p = make_params(sc, t_near, step, K, seed);
    const int opt = march_options(sc, seed);
    RayState rs{w.T, w.C, w.k_next, w.k_end};
    const unsigned rblocks = (unsigned)kn_div_up(R, RAY_BLOCK);
    const int64_t n_hist = 2 * (int64_t)sc->N; // histogram and fill cursors of the sample grouping
    const bool fused_hist = kn_group_fused(knobs, sc->N);
    // the marching kernel counts the samples per network: a counter per network in LDS on small grids, a hash table
    // of the networks a workgroup meets on large ones
    const int32_t march_hash = fused_hist ? 0 : knobs.group_hash_slots;
    KnStageTimer tm(ctx, st);
    tm.begin();
    KnMailbox *mb = mailbox_for(ctx, st);
    unsigned long long *mb_dev = mb ? mb->dev : nullptr;
    unsigned long long seq_local = 0; // sequence numbers without a mailbox (nobody reads them)
    // (a mailbox's counters are this call's alone until its last post has landed: see mailbox_for)
    auto next_seq = [&]() -> unsigned long long {
        if (!mb) return ++seq_local;
        mb->last_posted = ++mb->seq;
        return mb->seq;
    };
    int first_samples = knobs.first_wave_samples > 0 ? knobs.first_wave_samples : (K / 16 > DEFAULT_FIRST_WAVE ? K / 16 : DEFAULT_FIRST_WAVE);
    if (first_samples > knobs.slots_per_ray) first_samples = knobs.slots_per_ray;
    const WaveSchedule sched{first_samples, knobs.wave_growth, K > 0 ? K : 1, budget};
    hipLaunchKernelGGL(render_init_kernel(opt), dim3(rblocks), dim3(RAY_BLOCK), 0, st, p, rays_o, rays_d, R, rs, w.alive_b, w.blk_sum,
                       bg[0], bg[1], bg[2], rgb_out, (int32_t *)w.counters, 16, gw.hist, R >= n_hist ? (int32_t)n_hist : 0,
                       sc->desc.wdtype == KN_F32 ? (uint16_t *)nullptr : w.dir_table, sc->desc.wdtype == KN_BF16 ? 1 : 0);
    KN_CHECK_LAUNCH();
    if (R < n_hist) KN_TRY(kn_fill_i32(st, gw.hist, n_hist, 0));
    if (R < 16) KN_TRY(kn_fill_i32(st, (int32_t *)w.counters, 16, 0));
    unsigned long long seq = next_seq();
    hipLaunchKernelGGL(k_first_live, dim3(rblocks), dim3(RAY_BLOCK), 0, st, w.alive_b, w.blk_sum, R, w.live_a, w.alive_a,
                       w.n_live_dev, w.ctl, sched, mb_dev, seq);
    KN_CHECK_LAUNCH();
    tm.mark(KN_ST_SETUP);

    KnSampleSrc src{};
    src.points = nullptr;
    src.dirs = nullptr;
    src.rec = w.row_rec;
    src.rays_o = rays_o;
    src.rays_d = rays_d;
    src.t_near = t_near;
    src.step = step;
    src.kbits = kbits;
    src.out4 = w.out4;
    src.strat = seed ? 1 : 0;
    src.seed_key = p.seed_key;
    src.dir_table = w.dir_table;

    const int tile_len = kn_mlp_tile_len(sc);
    int32_t *live = w.live_a, *live_next = w.live_b, *alive = w.alive_a, *alive_next = w.alive_b;
    int wave_no = 0; // waves enqueued so far; wave i reads control block i % 2, its last kernel writes the other one
    // The shape of a wave (rows, samples per ray) lives in device memory, so a wave can be enqueued before the
    // host knows how many rays the previous one left: `rows_cap` is the host's upper bound, which sizes the grids.
    // rows_in: upper bound of the rows of the list the march reads.  From the second wave on that is the previous
    // wave's list, which the kernel compacts on the way (see k_march_wave); the new list is then the current one.
    int64_t s_bound = first_samples; // host-side upper bound of the samples per ray of the wave being enqueued
    auto march = [&](int64_t rows_in, bool compacting) -> int {
        const int32_t *ctl = w.ctl + 4 * (wave_no & 1), *old_ctl = w.ctl + 4 * ((wave_no + 1) & 1);
        const bool narrow = s_bound <= 64; // short rows (the first wave)
        const int lanes = narrow ? MARCH_G_NARROW : MARCH_G_WIDE;
        hipLaunchKernelGGL(march_wave_kernel(march_hash != 0, opt, narrow), dim3((unsigned)kn_div_up(rows_in * lanes, 256)), dim3(256),
                           sizeof(int32_t) * (size_t)(march_hash ? 2 * march_hash : sc->N), st, p, rays_o, rays_d, live, alive,
                           ctl, kbits, rs, w.row_keys, w.row_rec, w.cnt, gw.hist, sc->N, march_hash, old_ctl,
                           compacting ? w.blk_off : (const int32_t *)nullptr, w.grp_list, live_next, alive_next);
        KN_CHECK_LAUNCH();
        if (compacting) {
            int32_t *t = live; live = live_next; live_next = t;
            t = alive; alive = alive_next; alive_next = t;
        }
        tm.mark(KN_ST_MARCH);
        return KN_OK;
    };
    // post: the wave's survivor count and the running totals go to the mailbox (only where the host is going to look:
    // the writes to host memory are part of the kernel that closes the wave)
    // closing: false when the wave is known to be the last and nobody is going to read its sums (they feed the next
    // wave's control block and list compaction, and the counters): the kernel that adds them up is then left out
    auto rest_of_wave = [&](int64_t rows_cap, bool post, bool closing) -> int {
        int32_t *ctl = w.ctl + 4 * (wave_no & 1), *ctl_next = w.ctl + 4 * ((wave_no + 1) & 1);
        KnBucketOut bo;
        KN_TRY(kn_group_run(st, knobs, w.row_keys, w.cnt, ctl, rows_cap, sc->N, tile_len, gw, &bo));
        tm.mark(KN_ST_BUCKET);
        hipEvent_t e0 = nullptr, e1 = nullptr;
        (void)tm.kernel_events(KN_ST_MLP, &e0, &e1);
        KN_TRY(kn_mlp_launch(sc, st, src, bo, budget, nullptr, nullptr, e0, e1));
        tm.mark(KN_ST_MLP);
        // many rays with few samples each: one lane per ray; few rays with many samples: 16 lanes per ray
        const bool lane_per_ray = s_bound <= 64;
        const int32_t groups = (int32_t)kn_div_up(rows_cap, MARCH_G);
        const int32_t cblocks = lane_per_ray ? (int32_t)kn_div_up(rows_cap, BLEND_ROWS) : groups;
        if (lane_per_ray)
            hipLaunchKernelGGL(k_composite_wave, dim3((unsigned)cblocks), dim3(256), 0, st, live, ctl, (int32_t)rows_cap, w.cnt,
                               w.out4, step, term_eps, bg[0], bg[1], bg[2], rs, rgb_out, alive, w.partials, w.surv16, gw.hist,
                               fused_hist ? (int32_t)n_hist : 0, wave_no == 0 ? 1 : 0);
        else
            hipLaunchKernelGGL(k_composite_group, dim3((unsigned)cblocks), dim3(256), 0, st, live, ctl, (int32_t)rows_cap, w.cnt,
                               w.out4, step, term_eps, bg[0], bg[1], bg[2], rs, rgb_out, alive, w.partials, w.surv16, gw.hist,
                               fused_hist ? (int32_t)n_hist : 0, wave_no == 0 ? 1 : 0);
        KN_CHECK_LAUNCH();
        if (closing) {
            if (post) seq = next_seq();
            hipLaunchKernelGGL(k_sum_partials, dim3(1), dim3(1024), 0, st, w.partials, cblocks, w.surv16, groups, w.counters, ctl,
                               ctl_next, sched, w.blk_off, w.grp_list, post ? mb_dev : (unsigned long long *)nullptr, seq);
            KN_CHECK_LAUNCH();
        }
        tm.mark(KN_ST_BLEND);
        tm.add(1, 0, 0, 0);
        ++wave_no;
        s_bound = s_bound * knobs.wave_growth < (int64_t)K ? s_bound * knobs.wave_growth : (int64_t)K;
        return KN_OK;
    };
    // first wave: its march is enqueued for all R rays while the host is still waiting for the number of live rays
    tm.begin();
    KN_TRY(march(R, false));
    long long first = 0;
    KN_TRY(wait_count(mb, st, seq, w.n_live_dev, sizeof(int32_t), &first));
    if (first < 0 || first > R) return KN_E_HIP;
    long long n_alive = first;
    if (first > 0) {
        // Further waves.  The second one is enqueued right behind the first (its shape is computed on the device);
        // after that the host looks at the survivor count before it enqueues more.
        bool speculative = (int64_t)first_samples < (int64_t)K;
        // With K slots for each of the `first` rays the second wave takes every ray to its end: nothing to wait for
        // (unless the caller wants the counters of this frame).
        const bool second_wave_ends_it = speculative && first * (long long)K <= budget &&
                                         (int64_t)first_samples * knobs.wave_growth >= (int64_t)K;
        const bool want_counts = tm.counts || stats != nullptr;
        // a wave's count is read by the host unless the next wave is enqueued blindly (the first wave's, when a second
        // follows) or nothing follows for sure (the second wave's, when it ends every ray)
        const bool blind_second = speculative;
        auto host_reads = [&](int wave_index) {
            if (want_counts) return true;
            if (wave_index == 0) return !blind_second;
            if (wave_index == 1 && blind_second) return !second_wave_ends_it;
            return true;
        };
        KN_TRY(rest_of_wave(first, host_reads(0), true));
        int64_t list_cap = first; // upper bound of the length of the current live list
        while (true) {
            if (wave_no == 2 && second_wave_ends_it && !want_counts) break;
            int64_t next_cap = list_cap; // survivors <= rows of the list they come from
            if (!speculative) {
                KN_TRY(wait_count(mb, st, seq, w.counters + 2, sizeof(unsigned long long), &n_alive));
                if (n_alive < 0 || n_alive > list_cap) return KN_E_HIP; // cannot happen; guards the loop
                if (n_alive == 0) break;
                next_cap = n_alive;
            }
            speculative = false;
            tm.begin();
            KN_TRY(march(list_cap, true)); // reads (and compacts) the old list
            list_cap = next_cap;
            // (the second wave, enqueued blindly, when it ends every ray and the frame's counters are not wanted: see the
            // loop's first line)
            const bool last_for_sure = wave_no == 1 && second_wave_ends_it && !want_counts;
            KN_TRY(rest_of_wave(list_cap, host_reads(wave_no), !last_for_sure));
        }
    }
    if (tm.counts || stats) {
        unsigned long long c[5] = {0ull, 0ull, 0ull, 0ull, 0ull}; // evaluated, blended, survivors, slots, waves
        if (wave_no > 0 && mb &&
            __atomic_load_n((const unsigned long long *)&mb->host[0], __ATOMIC_ACQUIRE) == seq) {
            c[0] = __atomic_load_n((const unsigned long long *)&mb->host[2], __ATOMIC_RELAXED);
            c[1] = __atomic_load_n((const unsigned long long *)&mb->host[3], __ATOMIC_RELAXED);
            c[3] = __atomic_load_n((const unsigned long long *)&mb->host[4], __ATOMIC_RELAXED);
            c[4] = __atomic_load_n((const unsigned long long *)&mb->host[5], __ATOMIC_RELAXED);
        } else if (wave_no > 0) {
            KN_HIP(hipMemcpyAsync(c, w.counters, sizeof(c), hipMemcpyDeviceToHost, st));
            KN_HIP(hipStreamSynchronize(st));
        }
        tm.add(0, (int64_t)c[0], (int64_t)c[0], 1);
        if (stats) {
            stats->waves = (int64_t)c[4];
            stats->samples_evaluated = (int64_t)c[0];
            stats->samples_blended = (int64_t)c[1];
            stats->slots = (int64_t)c[3];
        }
    }
    return KN_OK;
}

extern "C" int kn_render(kn_ctx *ctx, const kn_scene *sc, void *stream, const float *rays_o, const float *rays_d, int64_t R, float t_near,
                         float step, int32_t K, float term_eps, const float bg[3], float *rgb_out, kn_render_stats *stats,
                         void *workspace, int64_t workspace_bytes)
{
    return render_impl(ctx, sc, stream, rays_o, rays_d, R, t_near, step, K, term_eps, bg, nullptr, rgb_out, stats, workspace,
                       workspace_bytes);
}

extern "C" int kn_render_stratified(kn_ctx *ctx, const kn_scene *sc, void *stream, const float *rays_o, const float *rays_d, int64_t R,
                                    float t_near, float step, int32_t K, float term_eps, const float bg[3], uint32_t seed,
                                    float *rgb_out, kn_render_stats *stats, void *workspace, int64_t workspace_bytes)
{
    return render_impl(ctx, sc, stream, rays_o, rays_d, R, t_near, step, K, term_eps, bg, &seed, rgb_out, stats, workspace,
                       workspace_bytes);
}
