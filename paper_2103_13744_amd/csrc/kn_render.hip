// Ray marching with empty-space skipping, alpha blending with early ray termination, and the
// wave loop that ties them to bucketing and the grouped MLP (Sec. 3.1 Eq. 1-4, Sec. 3.4).
//
// A wave gives every live ray up to S sample slots.  Slot j of live ray i is entry j*n_live + i of
// the wave's arrays, so that marching, the networks' output scatter and blending all touch
// consecutive addresses for consecutive rays.  Unused slots carry the key N ("no network").
#include "kn_common.h"

#include <math.h>

int kn_cell_keys(const kn_scene *sc, hipStream_t st, const float *points, int64_t M, int32_t *ids, int32_t *keys);

namespace {

struct MarchParams {
    KnGrid net, occ;
    const uint32_t *occ_bits;
    int32_t has_occ;
    float t_near, step;
    int32_t K;
};

// One axis of Eq. 6 without the division when the result cannot depend on it: u' = rel * (1/cell)
// differs from the correctly rounded quotient by a few ulp; only when u' sits that close to an
// integer is the division itself evaluated.  Returns floor(quotient) as a float.
__device__ __forceinline__ float axis_floor(float rel, float cell, float inv_cell)
{
    const float u = rel * inv_cell;
    const float f = floorf(u);
    const float frac = u - f;
    const float guard = fabsf(u) * 4.8e-7f + 1e-30f;
    if (frac > guard && (1.0f - frac) > guard) return f; // also false for NaN / inf
    return floorf(rel / cell);
}

struct GridFast {
    float bmin[3], cell[3], inv[3], resf[3];
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
    }
    f.res1 = g.res[1];
    f.res2 = g.res[2];
    return f;
}

__device__ __forceinline__ int32_t grid_index_fast(const GridFast &g, float x, float y, float z)
{
    const float fx = axis_floor(x - g.bmin[0], g.cell[0], g.inv[0]);
    const float fy = axis_floor(y - g.bmin[1], g.cell[1], g.inv[1]);
    const float fz = axis_floor(z - g.bmin[2], g.cell[2], g.inv[2]);
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
    if (!(tmin <= tmax)) { // empty or NaN: keep NaN conservative (full range), empty -> nothing
        if (tmin > tmax) { a = 0.0f; b = 0.0f; } else { a = 0.0f; b = (float)K; }
    }
    k_lo = (int32_t)a;
    k_hi = (int32_t)b;
}

__device__ __forceinline__ bool sample_kept(const MarchParams &p, const GridFast &gn, const GridFast &go, float x, float y,
                                            float z, int32_t &cell)
{
    cell = grid_index_fast(gn, x, y, z);
    if (cell < 0) return false;
    if (!p.has_occ) return true;
    const int32_t v = grid_index_fast(go, x, y, z);
    if (v < 0) return false;
    return (p.occ_bits[(uint32_t)v >> 5] >> (v & 31)) & 1u;
}

// ---------------------------------------------------------------------------------------------
// stage kernel behind kn_march: one thread per ray, explicit output arrays
__global__ void k_march_stage(MarchParams p, const float *__restrict__ rays_o, const float *__restrict__ rays_d, int64_t R,
                              const int32_t *__restrict__ k_begin, int32_t S, int32_t *__restrict__ out_k,
                              int32_t *__restrict__ out_count, int32_t *__restrict__ out_k_next)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    const float o[3] = {rays_o[3 * r], rays_o[3 * r + 1], rays_o[3 * r + 2]};
    const float d[3] = {rays_d[3 * r], rays_d[3 * r + 1], rays_d[3 * r + 2]};
    const GridFast gn = make_fast(p.net), go = make_fast(p.occ);
    int32_t k_lo, k_hi;
    clip_ray(p.net, o, d, p.t_near, p.step, p.K, k_lo, k_hi);
    int32_t k = k_begin ? max(k_begin[r], 0) : 0;
    k = max(k, k_lo);
    int32_t n = 0;
    for (; k < k_hi && n < S; ++k) {
        float x, y, z;
        kn_lattice_point(o[0], o[1], o[2], d[0], d[1], d[2], p.t_near, p.step, k, x, y, z);
        int32_t cell;
        if (sample_kept(p, gn, go, x, y, z, cell)) out_k[r * S + n++] = k;
    }
    // ran out of candidate indices: the ray is exhausted
    const int32_t k_next = (k >= k_hi) ? p.K : k;
    for (int32_t j = n; j < S; ++j) out_k[r * S + j] = -1;
    out_count[r] = n;
    if (out_k_next) out_k_next[r] = k_next;
}

// ---------------------------------------------------------------------------------------------
// render state
struct RayState {
    float *T;          // R
    float *C;          // R*3
    int32_t *k_next;   // R
    int32_t *k_end;    // R
};

__global__ void k_render_init(MarchParams p, const float *__restrict__ rays_o, const float *__restrict__ rays_d, int64_t R,
                              RayState s, int32_t *__restrict__ live)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    const float o[3] = {rays_o[3 * r], rays_o[3 * r + 1], rays_o[3 * r + 2]};
    const float d[3] = {rays_d[3 * r], rays_d[3 * r + 1], rays_d[3 * r + 2]};
    int32_t k_lo, k_hi;
    clip_ray(p.net, o, d, p.t_near, p.step, p.K, k_lo, k_hi);
    s.T[r] = 1.0f;
    s.C[3 * r] = s.C[3 * r + 1] = s.C[3 * r + 2] = 0.0f;
    s.k_next[r] = k_lo;
    s.k_end[r] = k_hi;
    live[r] = (int32_t)r;
}

// one thread per live ray: collect up to S kept samples, write key + record per slot
__global__ void k_march_wave(MarchParams p, const float *__restrict__ rays_o, const float *__restrict__ rays_d,
                             const int32_t *__restrict__ live, int32_t n_live, int32_t S, int32_t kbits, int32_t N,
                             RayState s, int32_t *__restrict__ keys, uint32_t *__restrict__ rec, int32_t *__restrict__ cnt)
{
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_live) return;
    const int32_t r = live[i];
    const float o[3] = {rays_o[3 * (int64_t)r], rays_o[3 * (int64_t)r + 1], rays_o[3 * (int64_t)r + 2]};
    const float d[3] = {rays_d[3 * (int64_t)r], rays_d[3 * (int64_t)r + 1], rays_d[3 * (int64_t)r + 2]};
    const GridFast gn = make_fast(p.net), go = make_fast(p.occ);
    int32_t k = s.k_next[r];
    const int32_t k_hi = s.k_end[r];
    int32_t n = 0;
    for (; k < k_hi && n < S; ++k) {
        float x, y, z;
        kn_lattice_point(o[0], o[1], o[2], d[0], d[1], d[2], p.t_near, p.step, k, x, y, z);
        int32_t cell;
        if (sample_kept(p, gn, go, x, y, z, cell)) {
            const int64_t slot = (int64_t)n * n_live + i;
            keys[slot] = cell;
            rec[slot] = ((uint32_t)r << kbits) | (uint32_t)k;
            ++n;
        }
    }
    s.k_next[r] = k;
    cnt[i] = n;
    for (int32_t j = n; j < S; ++j) keys[(int64_t)j * n_live + i] = N;
}

// one thread per live ray: Eq. 2-4 over this wave's samples, early termination, retire finished rays
__global__ void k_composite_wave(const int32_t *__restrict__ live, int32_t n_live, const int32_t *__restrict__ cnt,
                                 const float *__restrict__ sigma, const float *__restrict__ rgb, float step, float eps,
                                 float bg0, float bg1, float bg2, RayState s, float *__restrict__ rgb_out,
                                 int32_t *__restrict__ alive, unsigned long long *__restrict__ counters)
{
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    int32_t blended = 0, evaluated = 0;
    if (i < n_live) {
        const int32_t r = live[i];
        const int32_t n = cnt[i];
        float T = s.T[r];
        float c0 = s.C[3 * (int64_t)r], c1 = s.C[3 * (int64_t)r + 1], c2 = s.C[3 * (int64_t)r + 2];
        bool dead = false;
        for (int32_t j = 0; j < n; ++j) {
            const int64_t slot = (int64_t)j * n_live + i;
            const float sg = sigma[slot];
            const float alpha = 1.0f - expf(-sg * step);
            const float wgt = T * alpha;
            c0 = fmaf(wgt, rgb[3 * slot], c0);
            c1 = fmaf(wgt, rgb[3 * slot + 1], c1);
            c2 = fmaf(wgt, rgb[3 * slot + 2], c2);
            T *= (1.0f - alpha);
            ++blended;
            if (eps > 0.0f && T < eps) { dead = true; break; }
        }
        evaluated = n;
        const bool exhausted = s.k_next[r] >= s.k_end[r];
        const bool lives = !dead && !exhausted;
        if (lives) {
            s.T[r] = T;
            s.C[3 * (int64_t)r] = c0;
            s.C[3 * (int64_t)r + 1] = c1;
            s.C[3 * (int64_t)r + 2] = c2;
        } else {
            rgb_out[3 * (int64_t)r] = fmaf(T, bg0, c0);
            rgb_out[3 * (int64_t)r + 1] = fmaf(T, bg1, c1);
            rgb_out[3 * (int64_t)r + 2] = fmaf(T, bg2, c2);
        }
        alive[i] = lives ? 1 : 0;
    }
    // wave-level sums -> two atomics per wavefront
#pragma unroll
    for (int d = KN_WAVE / 2; d > 0; d >>= 1) {
        blended += __shfl_down(blended, d, KN_WAVE);
        evaluated += __shfl_down(evaluated, d, KN_WAVE);
    }
    if ((threadIdx.x & (KN_WAVE - 1)) == 0 && (blended | evaluated)) {
        atomicAdd(&counters[0], (unsigned long long)evaluated);
        atomicAdd(&counters[1], (unsigned long long)blended);
    }
}

__global__ void k_compact_live(const int32_t *__restrict__ live_in, const int32_t *__restrict__ alive,
                               const int32_t *__restrict__ pos, int32_t n_live, int32_t *__restrict__ live_out)
{
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_live && alive[i]) live_out[pos[i]] = live_in[i];
}

// stage kernel behind kn_composite: explicit per-ray sample ranges
__global__ void k_composite_stage(const float *__restrict__ sigma, const float *__restrict__ rgb,
                                  const int32_t *__restrict__ offsets, int64_t R, float step, float eps, float bg0,
                                  float bg1, float bg2, float *__restrict__ rgb_out, float *__restrict__ T_out,
                                  int32_t *__restrict__ n_used)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    float T = 1.0f, c0 = 0.0f, c1 = 0.0f, c2 = 0.0f;
    int32_t used = 0;
    for (int32_t j = offsets[r]; j < offsets[r + 1]; ++j) {
        const float alpha = 1.0f - expf(-sigma[j] * step);
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

MarchParams make_params(const kn_scene *sc, float t_near, float step, int32_t K)
{
    MarchParams p;
    p.net = sc->net_grid;
    p.occ = sc->has_occ ? sc->occ_grid : sc->net_grid;
    p.occ_bits = sc->occ_bits;
    p.has_occ = sc->has_occ ? 1 : 0;
    p.t_near = t_near;
    p.step = step;
    p.K = K;
    return p;
}

int g_first_wave_samples = 8;
int g_slots_per_ray = 8;

bool finite_pos(float v) { return isfinite(v) && v > 0.0f; }

} // namespace

extern "C" int kn_set_render_params(int32_t first_wave_samples, int32_t slots_per_ray)
{
    g_first_wave_samples = first_wave_samples > 0 ? first_wave_samples : 8;
    g_slots_per_ray = slots_per_ray > 0 ? slots_per_ray : 8;
    if (g_slots_per_ray < g_first_wave_samples) g_slots_per_ray = g_first_wave_samples;
    return KN_OK;
}

static int kbits_for(int32_t K)
{
    int b = 1;
    while ((1 << b) < K) ++b;
    return b;
}

// layout of the render workspace; returns total bytes (pointers valid only if ws.ok())
struct RenderWs {
    int32_t *live_a, *live_b, *cnt, *alive, *pos, *scan_tmp, *n_live_dev, *keys;
    uint32_t *rec;
    float *T, *C, *sigma, *rgb;
    int32_t *k_next, *k_end;
    unsigned long long *counters;
};

static void carve_render(KnCarver &ws, int64_t R, int64_t slots, RenderWs &w)
{
    w.live_a = ws.carve<int32_t>(R);
    w.live_b = ws.carve<int32_t>(R);
    w.cnt = ws.carve<int32_t>(R);
    w.alive = ws.carve<int32_t>(R);
    w.pos = ws.carve<int32_t>(R);
    w.scan_tmp = ws.carve<int32_t>(kn_scan_tmp_len(R));
    w.n_live_dev = ws.carve<int32_t>(1);
    w.T = ws.carve<float>(R);
    w.C = ws.carve<float>(3 * R);
    w.k_next = ws.carve<int32_t>(R);
    w.k_end = ws.carve<int32_t>(R);
    w.counters = ws.carve<unsigned long long>(2);
    w.keys = ws.carve<int32_t>(slots);
    w.rec = ws.carve<uint32_t>(slots);
    w.sigma = ws.carve<float>(slots);
    w.rgb = ws.carve<float>(3 * slots);
}

int64_t kn_render_ws_bytes(const kn_scene *sc, int64_t R)
{
    KnCarver c((void *)256, INT64_MAX / 2);
    RenderWs w;
    const int64_t slots = R * g_slots_per_ray;
    carve_render(c, R, slots, w);
    return c.used + kn_bucket_ws_bytes(slots, sc->N);
}

extern "C" int kn_march(const kn_scene *sc, void *stream, const float *rays_o, const float *rays_d, int64_t R, float t_near,
                        float step, int32_t K, const int32_t *k_begin, int32_t S, int32_t *out_k, int32_t *out_count,
                        int32_t *out_k_next)
{
    if (!sc || R < 0 || K < 0 || S < 1 || !isfinite(t_near) || !finite_pos(step)) return KN_E_INVALID_ARG;
    if (R > 0 && (!rays_o || !rays_d || !out_k || !out_count)) return KN_E_INVALID_ARG;
    if (R == 0) return KN_OK;
    if (kn_div_up(R, 256) > 0x7fffffffLL) return KN_E_UNSUPPORTED;
    hipLaunchKernelGGL(k_march_stage, dim3((unsigned)kn_div_up(R, 256)), dim3(256), 0, (hipStream_t)stream,
                       make_params(sc, t_near, step, K), rays_o, rays_d, R, k_begin, S, out_k, out_count, out_k_next);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

extern "C" int kn_composite(void *stream, const float *sigma, const float *rgb, const int32_t *offsets, int64_t R,
                            float step, float term_eps, const float bg[3], float *rgb_out, float *T_out, int32_t *n_used)
{
    if (R < 0 || !bg || !finite_pos(step) || !(term_eps >= 0.0f && term_eps < 1.0f)) return KN_E_INVALID_ARG;
    if (R > 0 && (!offsets || !rgb_out)) return KN_E_INVALID_ARG; // sigma / rgb may be NULL when no ray has samples
    if (R == 0) return KN_OK;
    if (kn_div_up(R, 256) > 0x7fffffffLL) return KN_E_UNSUPPORTED;
    hipLaunchKernelGGL(k_composite_stage, dim3((unsigned)kn_div_up(R, 256)), dim3(256), 0, (hipStream_t)stream, sigma, rgb,
                       offsets, R, step, term_eps, bg[0], bg[1], bg[2], rgb_out, T_out, n_used);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

extern "C" int kn_render(const kn_scene *sc, void *stream, const float *rays_o, const float *rays_d, int64_t R, float t_near,
                         float step, int32_t K, float term_eps, const float bg[3], float *rgb_out, kn_render_stats *stats,
                         void *workspace, int64_t workspace_bytes)
{
    if (!sc || R < 0 || K < 0 || !bg || !isfinite(t_near) || !finite_pos(step) || !(term_eps >= 0.0f && term_eps < 1.0f))
        return KN_E_INVALID_ARG;
    if (R > 0 && (!rays_o || !rays_d || !rgb_out)) return KN_E_INVALID_ARG;
    if (stats) {
        stats->rays = R;
        stats->waves = stats->samples_evaluated = stats->samples_blended = stats->slots = 0;
    }
    if (R == 0) return KN_OK;
    const int kbits = kbits_for(K > 1 ? K : 2);
    if (R > (1ll << (32 - kbits)) || R > 0x7fffffffLL / g_slots_per_ray) return KN_E_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < kn_render_ws_bytes(sc, R)) return KN_E_WORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    KnCarver ws(workspace, workspace_bytes);
    RenderWs w;
    const int64_t budget = R * g_slots_per_ray;
    carve_render(ws, R, budget, w);
    if (!ws.ok()) return KN_E_WORKSPACE;
    const int64_t bucket_base = ws.used;

    const MarchParams p = make_params(sc, t_near, step, K);
    RayState rs{w.T, w.C, w.k_next, w.k_end};
    const unsigned rblocks = (unsigned)kn_div_up(R, 256);
    hipLaunchKernelGGL(k_render_init, dim3(rblocks), dim3(256), 0, st, p, rays_o, rays_d, R, rs, w.live_a);
    KN_CHECK_LAUNCH();
    KN_TRY(kn_fill_i32(st, (int32_t *)w.counters, 4, 0));

    KnSampleSrc src{};
    src.points = nullptr;
    src.dirs = nullptr;
    src.rec = w.rec;
    src.rays_o = rays_o;
    src.rays_d = rays_d;
    src.t_near = t_near;
    src.step = step;
    src.kbits = kbits;

    const int tile_len = kn_mlp_tile_len(sc);
    int32_t *live = w.live_a, *live_next = w.live_b;
    int64_t n_live = R, waves = 0, slots_total = 0;
    while (n_live > 0) {
        int64_t S = budget / n_live;
        if (S < g_first_wave_samples) S = g_first_wave_samples;
        if (S > K) S = K;
        if (S < 1) S = 1;
        const int64_t Mw = n_live * S;
        const unsigned lblocks = (unsigned)kn_div_up(n_live, 256);
        KnStageTimer tm(st);
        tm.mark();
        hipLaunchKernelGGL(k_march_wave, dim3(lblocks), dim3(256), 0, st, p, rays_o, rays_d, live, (int32_t)n_live, (int32_t)S,
                           kbits, sc->N, rs, w.keys, w.rec, w.cnt);
        KN_CHECK_LAUNCH();
        tm.mark();
        KnCarver bws((char *)workspace + bucket_base, workspace_bytes - bucket_base);
        KnBucketOut bo;
        KN_TRY(kn_bucket_run(st, w.keys, Mw, sc->N, tile_len, nullptr, nullptr, nullptr, bws, &bo));
        tm.mark();
        KN_TRY(kn_mlp_launch(sc, st, src, bo, Mw, w.sigma, w.rgb));
        tm.mark();
        hipLaunchKernelGGL(k_composite_wave, dim3(lblocks), dim3(256), 0, st, live, (int32_t)n_live, w.cnt, w.sigma, w.rgb, step,
                           term_eps, bg[0], bg[1], bg[2], rs, rgb_out, w.alive, w.counters);
        KN_CHECK_LAUNCH();
        KN_TRY(kn_exclusive_scan_i32(st, w.alive, w.pos, n_live, w.scan_tmp, w.n_live_dev));
        hipLaunchKernelGGL(k_compact_live, dim3(lblocks), dim3(256), 0, st, live, w.alive, w.pos, (int32_t)n_live, live_next);
        KN_CHECK_LAUNCH();
        tm.mark();
        int32_t next = 0;
        KN_HIP(hipMemcpyAsync(&next, w.n_live_dev, sizeof(int32_t), hipMemcpyDeviceToHost, st));
        KN_HIP(hipStreamSynchronize(st));
        if (tm.on) {
            g_kn_profile.ms_march += tm.elapsed(0);
            g_kn_profile.ms_bucket += tm.elapsed(1);
            g_kn_profile.ms_mlp += tm.elapsed(2);
            g_kn_profile.ms_blend += tm.elapsed(3);
            g_kn_profile.mlp_launches += 1;
            g_kn_profile.bucket_keys += Mw;
        }
        if (next < 0 || next > n_live) return KN_E_HIP; // cannot happen; guards the loop
        ++waves;
        slots_total += Mw;
        n_live = next;
        int32_t *t = live; live = live_next; live_next = t;
    }
    if (g_kn_profile_on || stats) {
        unsigned long long c[2];
        KN_HIP(hipMemcpyAsync(c, w.counters, sizeof(c), hipMemcpyDeviceToHost, st));
        KN_HIP(hipStreamSynchronize(st));
        if (g_kn_profile_on) {
            g_kn_profile.mlp_samples += (int64_t)c[0];
            g_kn_profile.calls += 1;
        }
        if (stats) {
            stats->waves = waves;
            stats->samples_evaluated = (int64_t)c[0];
            stats->samples_blended = (int64_t)c[1];
            stats->slots = slots_total;
        }
    }
    return KN_OK;
}
