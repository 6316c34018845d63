/*
 * kn_oracle.h -- CPU oracle for the KiloNeRF rendering path (TEST INFRASTRUCTURE).
 *
 * A plain, slow, single-source C implementation of what the rendering path of
 * "KiloNeRF: Speeding up Neural Radiance Fields with Thousands of Tiny MLPs"
 * computes.  It exists only to check the HIP library: tests, the smoke check and
 * the cpu_baseline leg of the benchmark may call it; the product path never does.
 * It shares no code with the HIP path.
 *
 * Precision: everything that decides an integer (sample lattice position, cell
 * index, occupancy voxel) is taken in fp32 with one fixed operation sequence,
 * because the index is only well defined for one precision.  Everything else
 * (positional encoding, the affine layers, activations, compositing) runs in
 * fp64 on the fp32 inputs.  Two decisions rest on such fp64 values, early
 * termination (T < eps) and occupancy extraction (sigma > tau): there the oracle
 * also reports how close the value came to the threshold, so that a check can
 * tell a legitimate rounding difference from a mistake.
 *
 * All pointers are host pointers.  No function allocates memory that outlives
 * the call.  Return value 0 = ok, negative = invalid argument.
 */
#ifndef KN_ORACLE_H
#define KN_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t res[3];          /* network grid r = (rx, ry, rz)           (Sec. 3.2)   */
    float   aabb_min[3];     /* b_min                                    (Sec. 3.2)   */
    float   aabb_max[3];     /* b_max                                                 */
    int32_t hidden;          /* H: units per hidden layer (32 in the paper, Sec. 3.2) */
    int32_t L_pos, L_dir;    /* frequencies of the encoding of x and of d             */
    const float *weights;    /* N * kno_params_per_net(H, L_pos, L_dir) values        */
    int32_t occ_res[3];      /* occupancy grid resolution, all 0 = no grid            */
    const uint8_t *occupancy;/* occ_res[0]*occ_res[1]*occ_res[2] bytes, x slowest     */
    const int32_t *cell_net; /* NULL: one network per cell, network id = cell index.  Else a  */
                             /* sparse grid (Sec. 5): rx*ry*rz entries, cell -> network index */
                             /* in [0, n_nets); any other value = no network in that cell     */
    int32_t n_nets;          /* networks behind `weights` when cell_net is given              */
} kno_scene;

/* Number of parameters of one tiny MLP.  Layers (Sec. 3.2, "Network Architecture"):
 * L1 e_x->H, L2 H->H, L3 H->1+H (density, feature), L4 H+e_d->H, L5 H->3,
 * e_x = 3+6*L_pos, e_d = 3+6*L_dir; each layer has a bias. */
int64_t kno_params_per_net(int32_t hidden, int32_t L_pos, int32_t L_dir);

/* gamma_L(p) of a 3-vector: [p, then per k: sin(2^k p) (3), cos(2^k p) (3)].  out has 3+6L. */
void kno_posenc(const float p[3], int32_t L, double *out);

/* Spatial binning g(x) (Sec. 3.2, Eq. 6) for a grid of resolution res over the
 * scene AABB, fp32: per axis floor((x-bmin)/((bmax-bmin)/r)).  Returns the linear
 * index (ix*ry+iy)*rz+iz, or -1 if x falls outside [bmin,bmax) on any axis. */
int32_t kno_grid_index(const float bmin[3], const float bmax[3], const int32_t res[3],
                       const float x[3]);

/* Point -> network id for M points (ids[m] = -1 outside the AABB or, on a sparse grid, in a
 * cell without a network). */
int kno_cell_ids(const kno_scene *s, const float *points, int64_t M, int32_t *ids);

/* Stable bucketing by network id: counts[N+1] (slot N counts id=-1), offsets[N+2]
 * (exclusive scan, offsets[N+1]=M), perm[M]: sample indices ordered by id with -1 last,
 * equal ids keep ascending sample index. */
int kno_bucket(const int32_t *ids, int64_t M, int32_t N, int32_t *counts, int32_t *offsets,
               int32_t *perm);

/* One network n on one input (Sec. 3.2, Eq. 7): sigma, rgb[3]. */
int kno_mlp(const kno_scene *s, int32_t n, const float x[3], const float d[3],
            double *sigma, double *rgb);

/* eval_grouped: per point, cell id then its network.  Points outside, or in a cell without a
 * network: id -1, sigma 0, rgb 0. */
int kno_eval_points(const kno_scene *s, const float *points, const float *dirs, int64_t M,
                    double *sigma, double *rgb, int32_t *ids);

/* Sample lattice of one ray with empty-space skipping (Sec. 3.4): writes the step indices
 * k in [0,K) whose point lies inside the AABB in an occupied voxel (and, on a sparse grid, in a
 * cell that has a network), ascending; returns how many (<= K). */
int32_t kno_march(const kno_scene *s, const float o[3], const float d[3], float t_near,
                  float step, int32_t K, int32_t *ks);

/* Stratified sampling (Sec. 3.4 "Sampling" refers to NeRF's: one uniform draw per lattice interval).
 * Offset u in [0, 1) of lattice point k of ray number `ray`:
 *   mix(v): v ^= v >> 16; v *= 0x85ebca6b; v ^= v >> 13; v *= 0xc2b2ae35; v ^= v >> 16   (uint32)
 *   u = (mix(mix(mix(seed) + ray) ^ k) >> 8) * 2^-24
 * so that t_k = t_near + (k + u) * step (fp32, one fused multiply-add) lies in interval k.
 * kno_march_stratified / kno_render_stratified are kno_march / kno_render on these lattice
 * points; in the render, ray r of the arrays has ray number ray_ids[r] (r if ray_ids is NULL: a
 * caller that renders a subset of a frame's rays passes their numbers in the frame), and sample k
 * is blended with delta_k = t_(k+1) - t_k (the next lattice point, kept or not; k + 1 = K included). */
float kno_stratified_offset(uint32_t seed, uint32_t ray, int32_t k);
int32_t kno_march_stratified(const kno_scene *s, const float o[3], const float d[3], float t_near,
                             float step, int32_t K, uint32_t seed, uint32_t ray, int32_t *ks);

/* Front-to-back alpha blending with early termination (Sec. 3.1 Eq. 2-4, Sec. 3.4):
 * n samples (sigma, rgb) of constant spacing step.  Returns the number of samples
 * composited (n unless terminated early); out[3] = C + T*bg, *T_out = final T,
 * *margin_out = min over composited samples of |T_i - eps| / eps (inf if eps == 0). */
int32_t kno_composite(const double *sigma, const double *rgb, int32_t n, double step, double eps,
                      const double bg[3], double out[3], double *T_out, double *margin_out);
/* The same with a delta per sample (Eq. 4 as printed carries delta_i; stratified samples have their own). */
int32_t kno_composite_deltas(const double *sigma, const double *rgb, const double *delta, int32_t n,
                             double eps, const double bg[3], double out[3], double *T_out,
                             double *margin_out);

/* Render R rays.  rgb_out R*3.  Optional per-ray outputs (nullable): n_eval (samples
 * evaluated = composited), T_final, margin (see kno_composite).  Samples behind the
 * termination point are never evaluated. */
int kno_render(const kno_scene *s, const float *rays_o, const float *rays_d, int64_t R,
               float t_near, float step, int32_t K, float term_eps, const float bg[3],
               double *rgb_out, int32_t *n_eval, double *T_final, double *margin);

int kno_render_stratified(const kno_scene *s, const float *rays_o, const float *rays_d, int64_t R,
                          float t_near, float step, int32_t K, float term_eps, const float bg[3],
                          uint32_t seed, const uint32_t *ray_ids, double *rgb_out, int32_t *n_eval,
                          double *T_final, double *margin);

/* Occupancy grid extraction (Sec. 3.4, "Empty Space Skipping"; tau: Sec. 4.1): the density is
 * sampled on a 3x3x3 subgrid of every voxel of a grid of resolution occ_res over the AABB and the
 * voxel is marked (1) iff any of the 27 densities is above tau (strictly), else 0.  The density
 * field is the scene's own network grid (the paper samples its teacher model); a probe is
 * evaluated by the network of the cell it lies in (Eq. 6; density 0 where a sparse grid has no
 * network).  Probe positions (the paper does not
 * place the subgrid): sub-cell centres, per axis x = bmin + (v + c) * cell with c in {1/6, 1/2, 5/6},
 * cell = (bmax - bmin) / occ_res, taken in fp32 as fmaf((float)v + c, cell, bmin).
 * kno_extract_occupancy_at does this for n voxels given by linear index (x slowest);
 * kno_extract_occupancy for the whole grid.  Optional outputs per voxel (nullable): max_sigma =
 * the largest of the 27 densities, margin = min over the probes of |sigma - tau|. */
int kno_extract_occupancy_at(const kno_scene *s, const int32_t occ_res[3], float tau,
                             const int64_t *voxels, int64_t n, uint8_t *occ, double *max_sigma,
                             double *margin);
int kno_extract_occupancy(const kno_scene *s, const int32_t occ_res[3], float tau, uint8_t *occ,
                          double *max_sigma, double *margin);

/* Number of threads the loops over rays / points use (1 unless built with OpenMP). */
int kno_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
