/*
 * kn_oracle.c -- CPU oracle for the KiloNeRF rendering path (TEST INFRASTRUCTURE).
 *
 * Written from the paper's definitions, one function per step, no blocking, fusion or
 * reordering.  Only tests, the smoke check and the benchmark's cpu_baseline leg use it.
 * Build: gcc -O2 -ffp-contract=off -fPIC -shared (add -fopenmp for the threaded build;
 * the loops over independent rays / points are the only parallel ones).
 *
 * Readings of the paper taken here (each is also pinned by a CPU test):
 *  - Eq. 4 is printed without the minus sign; alpha = 1 - exp(-sigma*delta) is used, the
 *    only reading under which constant density gives transmittance exp(-sigma*distance).
 *  - delta is the constant lattice spacing `step` for every sample (Sec. 3.4: K fixes the
 *    distance between sampled points); skipped samples do not stretch it.
 *  - Lattice points sit at the middle of each step: t_k = t_near + (k + 1/2) * step.
 *  - The 3-D cell index of Eq. 6 is linearised x slowest, z fastest; cells are half open,
 *    so a point on the upper face of the AABB is outside.
 *  - The network receives the global position x (Eq. 7), not a cell-local one.
 *  - Encoding gamma_L(p) = [p, sin(2^k p), cos(2^k p) for k = 0..L-1] without a factor
 *    of pi (3 + 6L values; 63 for L = 10 and 27 for L = 4).
 *  - Layers: e_x -> H ReLU -> H ReLU -> (1 + H): output 0 is the density, passed through
 *    ReLU; outputs 1..H are the feature vector, no activation; [feature, gamma(d)] -> H
 *    ReLU -> 3 sigmoid (Sec. 3.2, "Network Architecture").
 *  - Early termination (Sec. 3.4): after sample i has been blended, stop if T < eps
 *    (strictly); eps = 0 turns it off.  The background colour is added with weight T.
 *  - Occupancy extraction (Sec. 3.4): the 3x3x3 subgrid of a voxel sits at its sub-cell centres
 *    (offsets 1/6, 1/2, 5/6 of the voxel per axis); "above" tau is strict; the sampled density
 *    field is the network grid itself.
 *  - Sparse network grid (Sec. 5 names data structures that instantiate networks only near surfaces):
 *    a table maps each cell of the regular grid to the index of its network or to "none"; a cell
 *    without a network has density 0 everywhere, its lattice points are skipped like empty space,
 *    and a point in it gets the id -1.
 *  - Stratified sampling (Sec. 3.4 "Sampling", after NeRF): lattice point k of a ray is drawn uniformly from
 *    its own interval, t_k = t_near + (k + u) * step with u in [0, 1) from a counter-based
 *    generator keyed by (seed, ray index, k); delta of sample k is the distance to the next
 *    lattice point, t_(k+1) - t_k, whether or not that point is skipped.
 */
#include "kn_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define KNO_MAX_H   256
#define KNO_MAX_ENC 128

int kno_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int64_t kno_params_per_net(int32_t H, int32_t L_pos, int32_t L_dir)
{
    int64_t ex = 3 + 6 * (int64_t)L_pos, ed = 3 + 6 * (int64_t)L_dir;
    return (ex * H + H) + ((int64_t)H * H + H) + ((int64_t)H * (H + 1) + (H + 1)) +
           ((H + ed) * H + H) + ((int64_t)H * 3 + 3);
}

void kno_posenc(const float p[3], int32_t L, double *out)
{
    for (int a = 0; a < 3; ++a) out[a] = (double)p[a];
    for (int k = 0; k < L; ++k) {
        double f = ldexp(1.0, k); /* 2^k */
        for (int a = 0; a < 3; ++a) {
            out[3 + 6 * k + a] = sin(f * (double)p[a]);
            out[3 + 6 * k + 3 + a] = cos(f * (double)p[a]);
        }
    }
}

int32_t kno_grid_index(const float bmin[3], const float bmax[3], const int32_t res[3],
                       const float x[3])
{
    int32_t idx[3];
    for (int a = 0; a < 3; ++a) {
        /* Eq. 6 evaluated literally in fp32: cell size first, then the quotient. */
        float extent = bmax[a] - bmin[a];
        float cell = extent / (float)res[a];
        float rel = x[a] - bmin[a];
        float u = rel / cell;
        float fl = floorf(u);
        if (!(fl >= 0.0f) || !(fl < (float)res[a])) return -1; /* also rejects NaN */
        idx[a] = (int32_t)fl;
    }
    return (idx[0] * res[1] + idx[1]) * res[2] + idx[2];
}

/* Network of a point: Eq. 6 gives the cell; a sparse scene then looks the cell up in its table
 * (entries outside [0, n_nets) mean "no network here").  -1 = outside the AABB or no network. */
static int32_t network_of(const kno_scene *s, const float x[3])
{
    int32_t cell = kno_grid_index(s->aabb_min, s->aabb_max, s->res, x);
    if (cell < 0 || !s->cell_net) return cell;
    int32_t n = s->cell_net[cell];
    return (n >= 0 && n < s->n_nets) ? n : -1;
}

int kno_cell_ids(const kno_scene *s, const float *points, int64_t M, int32_t *ids)
{
    if (!s || (M > 0 && (!points || !ids))) return -1;
    for (int64_t m = 0; m < M; ++m) ids[m] = network_of(s, points + 3 * m);
    return 0;
}

int kno_bucket(const int32_t *ids, int64_t M, int32_t N, int32_t *counts, int32_t *offsets,
               int32_t *perm)
{
    if (N < 0 || M < 0 || !counts || !offsets || (M > 0 && (!ids || !perm))) return -1;
    for (int32_t n = 0; n <= N; ++n) counts[n] = 0;
    for (int64_t m = 0; m < M; ++m) {
        int32_t b = ids[m] < 0 ? N : ids[m];
        if (b > N) return -1;
        counts[b] += 1;
    }
    offsets[0] = 0;
    for (int32_t n = 0; n <= N; ++n) offsets[n + 1] = offsets[n] + counts[n];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N + 1));
    if (!cursor) return -2;
    for (int32_t n = 0; n <= N; ++n) cursor[n] = offsets[n];
    for (int64_t m = 0; m < M; ++m) { /* ascending m => stable */
        int32_t b = ids[m] < 0 ? N : ids[m];
        perm[cursor[b]++] = (int32_t)m;
    }
    free(cursor);
    return 0;
}

/* y[o] = b[o] + sum_i in[i] * W[i][o], W stored row = input, column = output. */
static void affine(const float *W, const float *b, const double *in, int n_in, int n_out,
                   double *out)
{
    for (int o = 0; o < n_out; ++o) {
        double acc = (double)b[o];
        for (int i = 0; i < n_in; ++i) acc += in[i] * (double)W[(size_t)i * n_out + o];
        out[o] = acc;
    }
}

static double relu(double v) { return v > 0.0 ? v : 0.0; }

int kno_mlp(const kno_scene *s, int32_t n, const float x[3], const float d[3], double *sigma,
            double *rgb)
{
    const int H = s->hidden;
    const int ex = 3 + 6 * s->L_pos, ed = 3 + 6 * s->L_dir;
    if (H < 1 || H > KNO_MAX_H || ex > KNO_MAX_ENC || ed > KNO_MAX_ENC) return -1;
    const int64_t P = kno_params_per_net(H, s->L_pos, s->L_dir);
    const float *w = s->weights + (size_t)n * (size_t)P;
    const float *W1 = w;                 const float *b1 = W1 + (size_t)ex * H;
    const float *W2 = b1 + H;            const float *b2 = W2 + (size_t)H * H;
    const float *W3 = b2 + H;            const float *b3 = W3 + (size_t)H * (H + 1);
    const float *W4 = b3 + (H + 1);      const float *b4 = W4 + (size_t)(H + ed) * H;
    const float *W5 = b4 + H;            const float *b5 = W5 + (size_t)H * 3;

    double gx[KNO_MAX_ENC], in4[KNO_MAX_H + KNO_MAX_ENC];
    double h1[KNO_MAX_H], h2[KNO_MAX_H], o3[KNO_MAX_H + 1], h4[KNO_MAX_H], o5[3];

    kno_posenc(x, s->L_pos, gx);
    affine(W1, b1, gx, ex, H, h1);
    for (int i = 0; i < H; ++i) h1[i] = relu(h1[i]);
    affine(W2, b2, h1, H, H, h2);
    for (int i = 0; i < H; ++i) h2[i] = relu(h2[i]);
    affine(W3, b3, h2, H, H + 1, o3);
    *sigma = relu(o3[0]);
    for (int i = 0; i < H; ++i) in4[i] = o3[1 + i]; /* feature vector: no activation */
    kno_posenc(d, s->L_dir, in4 + H);
    affine(W4, b4, in4, H + ed, H, h4);
    for (int i = 0; i < H; ++i) h4[i] = relu(h4[i]);
    affine(W5, b5, h4, H, 3, o5);
    for (int c = 0; c < 3; ++c) rgb[c] = 1.0 / (1.0 + exp(-o5[c]));
    return 0;
}

int kno_eval_points(const kno_scene *s, const float *points, const float *dirs, int64_t M,
                    double *sigma, double *rgb, int32_t *ids)
{
    if (!s || (M > 0 && (!points || !dirs || !sigma || !rgb))) return -1;
    int err = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 256)
#endif
    for (int64_t m = 0; m < M; ++m) {
        int32_t id = network_of(s, points + 3 * m);
        if (ids) ids[m] = id;
        if (id < 0) {
            sigma[m] = 0.0;
            rgb[3 * m] = rgb[3 * m + 1] = rgb[3 * m + 2] = 0.0;
        } else if (kno_mlp(s, id, points + 3 * m, dirs + 3 * m, sigma + m, rgb + 3 * m) != 0) {
            err = -1;
        }
    }
    return err;
}

/* 32-bit mixing function (the finalizer of MurmurHash3, a published bijection on 32-bit words). */
static uint32_t mix32(uint32_t v)
{
    v ^= v >> 16;
    v *= 0x85ebca6bu;
    v ^= v >> 13;
    v *= 0xc2b2ae35u;
    v ^= v >> 16;
    return v;
}

float kno_stratified_offset(uint32_t seed, uint32_t ray, int32_t k)
{
    uint32_t per_ray = mix32(mix32(seed) + ray);
    uint32_t word = mix32(per_ray ^ (uint32_t)k);
    return (float)(word >> 8) * (1.0f / 16777216.0f); /* 24 bits -> [0, 1), exact in fp32 */
}

/* Where inside its interval lattice point k sits: the middle, or the stratified draw. */
typedef struct {
    int on;
    uint32_t seed, ray;
} strat;

static float lattice_offset(const strat *j, int32_t k)
{
    return (j && j->on) ? kno_stratified_offset(j->seed, j->ray, k) : 0.5f;
}

/* Parameter of lattice point k on a ray: t_k = t_near + (k + offset) step as one fused
 * multiply-add in fp32 (never accumulated along the ray). */
static float lattice_t(float t_near, float step, int32_t k, const strat *j)
{
    return fmaf((float)k + lattice_offset(j, k), step, t_near);
}

/* Position of lattice point k: x = o + t_k d, one fused multiply-add per axis. */
static void lattice_point(const float o[3], const float d[3], float t_near, float step, int32_t k,
                          const strat *j, float x[3])
{
    float t = lattice_t(t_near, step, k, j);
    for (int a = 0; a < 3; ++a) x[a] = fmaf(t, d[a], o[a]);
}

/* delta of sample k: the constant spacing on the midpoint lattice; with stratified sampling the
 * distance to the next lattice point (NeRF's delta_i = t_(i+1) - t_i), also for k = K - 1. */
static double lattice_delta(float t_near, float step, int32_t k, const strat *j)
{
    if (!(j && j->on)) return (double)step;
    return (double)lattice_t(t_near, step, k + 1, j) - (double)lattice_t(t_near, step, k, j);
}

static int sample_is_kept(const kno_scene *s, const float x[3])
{
    if (network_of(s, x) < 0) return 0; /* outside the AABB, or a cell without a network */
    if (s->occ_res[0] == 0) return 1;                                      /* no occupancy grid */
    int32_t v = kno_grid_index(s->aabb_min, s->aabb_max, s->occ_res, x);
    return v >= 0 && s->occupancy[v] != 0;
}

static int32_t march_ray(const kno_scene *s, const float o[3], const float d[3], float t_near,
                         float step, int32_t K, const strat *j, int32_t *ks)
{
    int32_t n = 0;
    for (int32_t k = 0; k < K; ++k) {
        float x[3];
        lattice_point(o, d, t_near, step, k, j, x);
        if (sample_is_kept(s, x)) ks[n++] = k;
    }
    return n;
}

int32_t kno_march(const kno_scene *s, const float o[3], const float d[3], float t_near,
                  float step, int32_t K, int32_t *ks)
{
    return march_ray(s, o, d, t_near, step, K, NULL, ks);
}

int32_t kno_march_stratified(const kno_scene *s, const float o[3], const float d[3], float t_near,
                             float step, int32_t K, uint32_t seed, uint32_t ray, int32_t *ks)
{
    const strat j = {1, seed, ray};
    return march_ray(s, o, d, t_near, step, K, &j, ks);
}

/* Eq. 2-4 with a delta per sample (delta == NULL: the constant `step`). */
static int32_t composite(const double *sigma, const double *rgb, const double *delta, int32_t n,
                         double step, double eps, const double bg[3], double out[3], double *T_out,
                         double *margin_out)
{
    double T = 1.0, C[3] = {0.0, 0.0, 0.0}, margin = INFINITY;
    int32_t used = 0;
    for (int32_t i = 0; i < n; ++i) {
        double alpha = 1.0 - exp(-sigma[i] * (delta ? delta[i] : step)); /* Eq. 4 (sign restored) */
        for (int c = 0; c < 3; ++c) C[c] += T * alpha * rgb[3 * i + c]; /* Eq. 2 */
        T *= (1.0 - alpha);                                   /* Eq. 3 */
        ++used;
        if (eps > 0.0) {
            double mg = fabs(T - eps) / eps;
            if (mg < margin) margin = mg;
            if (T < eps) break;                               /* Sec. 3.4, ERT */
        }
    }
    for (int c = 0; c < 3; ++c) out[c] = C[c] + T * bg[c];
    if (T_out) *T_out = T;
    if (margin_out) *margin_out = margin;
    return used;
}

int32_t kno_composite(const double *sigma, const double *rgb, int32_t n, double step, double eps,
                      const double bg[3], double out[3], double *T_out, double *margin_out)
{
    return composite(sigma, rgb, NULL, n, step, eps, bg, out, T_out, margin_out);
}

int32_t kno_composite_deltas(const double *sigma, const double *rgb, const double *delta, int32_t n,
                             double eps, const double bg[3], double out[3], double *T_out,
                             double *margin_out)
{
    if (n > 0 && !delta) return -1;
    return composite(sigma, rgb, delta, n, 0.0, eps, bg, out, T_out, margin_out);
}

static int render_rays(const kno_scene *s, const float *rays_o, const float *rays_d, int64_t R,
                       float t_near, float step, int32_t K, float term_eps, const float bg[3],
                       const uint32_t *seed, const uint32_t *ray_ids, double *rgb_out, int32_t *n_eval,
                       double *T_final, double *margin)
{
    if (!s || K < 0 || (R > 0 && (!rays_o || !rays_d || !rgb_out)) || !bg) return -1;
    int err = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 16)
#endif
    for (int64_t r = 0; r < R; ++r) {
        const float *o = rays_o + 3 * r, *d = rays_d + 3 * r;
        const double eps = (double)term_eps;
        const strat j = {seed != NULL, seed ? *seed : 0u, ray_ids ? ray_ids[r] : (uint32_t)r};
        double T = 1.0, C[3] = {0.0, 0.0, 0.0}, mg_min = INFINITY;
        int32_t used = 0;
        for (int32_t k = 0; k < K; ++k) {
            float x[3];
            lattice_point(o, d, t_near, step, k, &j, x);
            if (!sample_is_kept(s, x)) continue;
            int32_t id = network_of(s, x);
            double sg, col[3];
            if (kno_mlp(s, id, x, d, &sg, col) != 0) { err = -1; break; }
            double alpha = 1.0 - exp(-sg * lattice_delta(t_near, step, k, &j));
            for (int c = 0; c < 3; ++c) C[c] += T * alpha * col[c];
            T *= (1.0 - alpha);
            ++used;
            if (eps > 0.0) {
                double mg = fabs(T - eps) / eps;
                if (mg < mg_min) mg_min = mg;
                if (T < eps) break;
            }
        }
        for (int c = 0; c < 3; ++c) rgb_out[3 * r + c] = C[c] + T * (double)bg[c];
        if (n_eval) n_eval[r] = used;
        if (T_final) T_final[r] = T;
        if (margin) margin[r] = mg_min;
    }
    return err;
}

int kno_render(const kno_scene *s, const float *rays_o, const float *rays_d, int64_t R,
               float t_near, float step, int32_t K, float term_eps, const float bg[3],
               double *rgb_out, int32_t *n_eval, double *T_final, double *margin)
{
    return render_rays(s, rays_o, rays_d, R, t_near, step, K, term_eps, bg, NULL, NULL, rgb_out, n_eval,
                       T_final, margin);
}

int kno_render_stratified(const kno_scene *s, const float *rays_o, const float *rays_d, int64_t R,
                          float t_near, float step, int32_t K, float term_eps, const float bg[3],
                          uint32_t seed, const uint32_t *ray_ids, double *rgb_out, int32_t *n_eval,
                          double *T_final, double *margin)
{
    return render_rays(s, rays_o, rays_d, R, t_near, step, K, term_eps, bg, &seed, ray_ids, rgb_out,
                       n_eval, T_final, margin);
}

/* Sec. 3.4: one voxel of the occupancy grid, 27 probes. */
static int extract_voxel(const kno_scene *s, const int32_t occ_res[3], float tau, int64_t voxel,
                         uint8_t *occ, double *max_sigma, double *margin)
{
    static const float sub[3] = {1.0f / 6.0f, 0.5f, 5.0f / 6.0f};
    const float dir[3] = {0.0f, 0.0f, 1.0f}; /* the density does not depend on the direction */
    int32_t v[3];
    v[2] = (int32_t)(voxel % occ_res[2]);
    v[1] = (int32_t)((voxel / occ_res[2]) % occ_res[1]);
    v[0] = (int32_t)(voxel / ((int64_t)occ_res[2] * occ_res[1]));
    float cell[3];
    for (int a = 0; a < 3; ++a) cell[a] = (s->aabb_max[a] - s->aabb_min[a]) / (float)occ_res[a];
    int any = 0;
    double top = 0.0, mg = INFINITY;
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j)
            for (int k = 0; k < 3; ++k) {
                const int sel[3] = {i, j, k};
                float x[3];
                for (int a = 0; a < 3; ++a) x[a] = fmaf((float)v[a] + sub[sel[a]], cell[a], s->aabb_min[a]);
                double sg = 0.0, rgb[3];
                int32_t id = network_of(s, x);
                if (id >= 0 && kno_mlp(s, id, x, dir, &sg, rgb) != 0) return -1;
                if (sg > (double)tau) any = 1;
                if (sg > top) top = sg;
                if (fabs(sg - (double)tau) < mg) mg = fabs(sg - (double)tau);
            }
    *occ = (uint8_t)any;
    if (max_sigma) *max_sigma = top;
    if (margin) *margin = mg;
    return 0;
}

int kno_extract_occupancy_at(const kno_scene *s, const int32_t occ_res[3], float tau,
                             const int64_t *voxels, int64_t n, uint8_t *occ, double *max_sigma,
                             double *margin)
{
    if (!s || !occ_res || occ_res[0] < 1 || occ_res[1] < 1 || occ_res[2] < 1 || n < 0 || (n > 0 && (!voxels || !occ)))
        return -1;
    const int64_t total = (int64_t)occ_res[0] * occ_res[1] * occ_res[2];
    int err = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 64)
#endif
    for (int64_t i = 0; i < n; ++i) {
        if (voxels[i] < 0 || voxels[i] >= total ||
            extract_voxel(s, occ_res, tau, voxels[i], occ + i, max_sigma ? max_sigma + i : NULL,
                          margin ? margin + i : NULL) != 0)
            err = -1;
    }
    return err;
}

int kno_extract_occupancy(const kno_scene *s, const int32_t occ_res[3], float tau, uint8_t *occ,
                          double *max_sigma, double *margin)
{
    if (!s || !occ_res || occ_res[0] < 1 || occ_res[1] < 1 || occ_res[2] < 1 || !occ) return -1;
    const int64_t total = (int64_t)occ_res[0] * occ_res[1] * occ_res[2];
    int err = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 64)
#endif
    for (int64_t vx = 0; vx < total; ++vx)
        if (extract_voxel(s, occ_res, tau, vx, occ + vx, max_sigma ? max_sigma + vx : NULL,
                          margin ? margin + vx : NULL) != 0)
            err = -1;
    return err;
}
