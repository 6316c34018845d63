/*
 * kilonerf.h -- C ABI of the MI355X (gfx950) implementation of the KiloNeRF rendering path.
 *
 * Paper: "KiloNeRF: Speeding up Neural Radiance Fields with Thousands of Tiny MLPs".
 * The library evaluates a regular grid of tiny per-cell MLPs on ray samples and composites
 * them into pixels.  Every step runs in hand-written HIP kernels; there is no CPU fallback.
 *
 * Conventions
 *  - A context (kn_ctx, from kn_create) belongs to one HIP device and holds everything that is
 *    mutable: the wave schedule of kn_render, the timing switches and totals, the host
 *    mailboxes through which kn_render's kernels report counts.  A scene is immutable once
 *    created and may be used through any context of its device.  Calls on one context may come
 *    from several threads (its state is guarded by a mutex), each on a stream, workspace and
 *    outputs of its own; the context's device must be current in the calling thread.
 *  - "dev" pointers are HIP device pointers on the context's device; "host" pointers are
 *    ordinary host memory.  The library only borrows caller buffers for the duration of a call
 *    (scene inputs and the scene buffer: see kn_scene_create).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *    work on it and return without waiting unless stated otherwise.
 *    Calls that neither wait nor read results back on the host (all but kn_create / kn_destroy,
 *    kn_scene_create / kn_scene_destroy, kn_render and kn_profile_read) use only kernel launches on
 *    `stream` and may be captured into a HIP graph, with profiling off.
 *  - Every function returns 0 (KN_OK) or a negative kn_status.  Arguments are validated on
 *    the host before anything is launched; sizes of 0 are valid and do nothing.
 *  - Positions and directions are fp32, row-major (n, 3).  Directions must have unit length:
 *    the sample spacing along a ray is `step` only then.
 *
 * Canonical weight layout (what the caller supplies): for network n = (ix*ry + iy)*rz + iz the
 * P = kn_params_per_net(...) values
 *     W1[ex][H] b1[H]  W2[H][H] b2[H]  W3[H][1+H] b3[1+H]  W4[H+ed][H] b4[H]  W5[H][3] b5[3]
 * with W[row = input][column = output], ex = 3+6*L_pos, ed = 3+6*L_dir.  Column 0 of layer 3 is
 * the density, columns 1..H the feature vector; rows 0..H-1 of layer 4 take the feature vector,
 * rows H.. take gamma(d).  Activations (Sec. 3.2 "Network Architecture"): ReLU after layers
 * 1, 2, 4 and on the density; none on the feature vector; sigmoid on the colour.
 * Encoding gamma_L(p) = [p_x p_y p_z, then for k = 0..L-1: sin(2^k p) (xyz), cos(2^k p) (xyz)].
 */
#ifndef KILONERF_H
#define KILONERF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KN_OK = 0,
    KN_E_INVALID_ARG = -1, /* null pointer, negative size, bad grid, non-finite parameter   */
    KN_E_UNSUPPORTED = -2, /* valid request this build has no kernel for (H, dtype, limits) */
    KN_E_WORKSPACE = -3,   /* workspace missing, misaligned or smaller than required        */
    KN_E_HIP = -4,         /* a HIP runtime call failed (see kn_last_hip_error)             */
    KN_E_NO_DEVICE = -5,   /* no usable gfx950 device                                        */
    KN_E_STATIC_LIMIT = -6 /* kn_eval_grouped_static: M needs more than KN_STATIC_SCRATCH_BYTES */
} kn_status;

typedef enum { KN_F32 = 0, KN_F16 = 1, KN_BF16 = 2 } kn_dtype;

/* Scene = AABB + network grid + per-cell MLP weights + optional occupancy grid (Sec. 3.2, 3.4). */
typedef struct {
    int32_t res[3];          /* network grid r = (rx, ry, rz), each >= 1, product <= 65535       */
                             /* (<= 2^24 cells when cell_net is given)                            */
    float aabb_min[3];       /* b_min                                                             */
    float aabb_max[3];       /* b_max, > b_min per axis                                           */
    int32_t hidden;          /* H: 32 or 64                                                       */
    int32_t L_pos, L_dir;    /* encoding frequencies; this build supports (10, 4)                 */
    int32_t wdtype;          /* kn_dtype of `weights`.  KN_F32: fp32 weights, activations and     */
                             /* accumulation (fp32 matrix-core instructions).  KN_F16 / KN_BF16:  */
                             /* 16-bit weights and activations on the matrix cores, fp32 sums.    */
                             /* Accuracy of the 16-bit types: every operand of a layer is rounded */
                             /* to 11 (fp16) / 8 (bf16) significant bits, which leaves the        */
                             /* colour within 1e-3 / 7e-3 and the density within 2.5e-3 / 2e-2 of */
                             /* the magnitude u of the density head's output (the unit the        */
                             /* densities of the scene come in).  Eq. 4 multiplies a density      */
                             /* error by the sample spacing: rendered pixels stay within 2e-2 of  */
                             /* an exact evaluation where u * step <= 8 (fp16) / <= 1 (bf16); a   */
                             /* coarser lattice or a steeper density head needs KN_F32.           */
    const void *weights;     /* dev, N*P elements of wdtype in the canonical layout               */
    int32_t occ_res[3];      /* occupancy grid resolution; all 0 = no grid (whole AABB occupied)  */
    const uint8_t *occupancy;/* dev, occ_res[0]*occ_res[1]*occ_res[2] bytes (0 = empty), x slowest*/
    /* Sparse network grid (Sec. 5: networks instantiated only in the vicinity of surfaces).  NULL:   */
    /* one network per cell, network id = cell index.  Else dev, rx*ry*rz entries (x slowest): the     */
    /* index in [0, n_nets) of the cell's network in `weights`; any other value = the cell has no      */
    /* network.  Such a cell is empty space: density 0, its lattice points are skipped, points in it   */
    /* get id -1 and sigma = rgb = 0.  Wherever this header says "network id" / N, a sparse scene has  */
    /* the table's value / n_nets.  The library keeps its own copy.                                    */
    const int32_t *cell_net;
    int32_t n_nets;          /* networks behind `weights` when cell_net is given: 1 .. 65535         */
} kn_scene_desc;

typedef struct kn_scene kn_scene; /* opaque, immutable after kn_scene_create */
typedef struct kn_ctx kn_ctx;     /* opaque, one per device and user of the library */

/* Counters of one kn_render call (filled when requested). */
typedef struct {
    int64_t rays;             /* R                                                             */
    int64_t waves;            /* passes of the march -> bucket -> MLP -> blend loop            */
    int64_t samples_evaluated;/* samples pushed through the networks (incl. ones behind the    */
                              /* termination point inside a wave)                              */
    int64_t samples_blended;  /* samples that entered Eq. 2 (what the method itself evaluates) */
    int64_t slots;            /* sample slots sorted over all waves (incl. unused ones)        */
} kn_render_stats;

const char *kn_error_string(int status);
/* hipError_t of the most recent failed HIP call on this thread (0 if none). */
int kn_last_hip_error(void);

/* Number of parameters of one network in the canonical layout; -1 for invalid arguments. */
int64_t kn_params_per_net(int32_t hidden, int32_t L_pos, int32_t L_dir);

/* A context on HIP device `device_index` (which must be a gfx950 device; the call makes it current in the calling
 * thread).  Allocates only host memory: the pinned, device-mapped mailboxes.  kn_destroy waits for the device. */
int kn_create(kn_ctx **out, int device_index);
int kn_destroy(kn_ctx *ctx);

/*
 * Create a scene on the context's device.  Validates the descriptor, then fills, on `stream`, the scene's device
 * data: the occupancy grid packed to bits with its skip field, the weights re-ordered into matrix-core operand
 * order, the table of a sparse grid.  That data lives in `buffer` (dev, 256-byte aligned, at least kn_scene_bytes
 * bytes, owned by the caller, who keeps it until kn_scene_destroy has returned), or, with buffer = NULL, in memory the
 * library allocates itself (hipMalloc; the only allocation of device memory in the library).  The descriptor's own
 * buffers (weights, occupancy, cell_net) may be released once the call has returned: it waits for `stream`
 * because it reads the skip field back to find the box around the occupied voxels.
 * 16-bit scenes: Sec. 3.2 puts no activation between layer 3's feature vector and layer 4, and the library evaluates
 * the two as one affine map, W3f W4f and b4 + W4f^T b3f, formed here in fp32 and rounded to the scene's type (the
 * result is Eq. 7 up to the rounding that 16-bit operands have anyway).  KN_E_UNSUPPORTED if an element of that
 * product is finite but beyond the type's range (fp16: 65504): such networks belong in bf16 or fp32 scenes.
 */
int kn_scene_bytes(const kn_scene_desc *desc, int64_t *out_bytes);
int kn_scene_create(kn_ctx *ctx, const kn_scene_desc *desc, void *stream, void *buffer /*dev, nullable*/,
                    int64_t buffer_bytes, kn_scene **out);
int kn_scene_destroy(kn_scene *scene); /* waits for the device; frees what the library allocated */

/* Workspace size (bytes) that kn_bucket / kn_eval_grouped need for up to max_points points and
 * kn_render for up to max_rays rays with the context's current wave schedule (kn_set_render_params: the slot
 * budget per ray sizes it; kn_render checks its workspace against the schedule it runs with); pass 0 for the one
 * not needed.  The workspace is a dev buffer, 256-byte aligned, owned by the caller; calls sharing one workspace
 * must not overlap. */
int kn_workspace_bytes(const kn_ctx *ctx, const kn_scene *scene, int64_t max_points, int64_t max_rays,
                       int64_t *out_bytes);

/* Eq. 6: network index of M points.  ids[m] = (ix*ry + iy)*rz + iz, or -1 outside [b_min, b_max).
 * fp32 arithmetic exactly as written in Eq. 6: floor((x - b_min) / ((b_max - b_min) / r)).  On a sparse
 * grid the cell index is then mapped through the scene's table (-1 where the cell has no network). */
int kn_cell_ids(const kn_scene *scene, void *stream, const float *points /*dev M*3*/, int64_t M,
                int32_t *ids /*dev M*/);

/* Sec. 3.5 (the batch is reordered so that the inputs of one network follow one another): stable
 * bucketing of M ids in [-1, N).  counts[N+1] (slot N = outside), offsets[N+2]
 * (exclusive scan of counts), perm[M] = sample indices sorted by id, -1 last, ties by index.
 * counts / offsets may be NULL.  M <= 2^30. */
int kn_bucket(kn_ctx *ctx, const kn_scene *scene, void *stream, const int32_t *ids /*dev M*/, int64_t M,
              int32_t *counts /*dev N+1, nullable*/, int32_t *offsets /*dev N+2, nullable*/,
              int32_t *perm /*dev M*/, void *workspace, int64_t workspace_bytes);

/* Eq. 7: (c, sigma) = f_theta(g(x))(x, d) for M points: cell assignment, ordering by network (Sec. 3.5: the
 * points themselves are moved into grouped order, by a stable sort), then the fused per-network MLP (encoding +
 * 5 layers) over each bucket.  Outputs in caller order; points outside the AABB get sigma = 0, rgb = 0,
 * id = -1.  cell_id / counts / perm are optional outputs as in kn_cell_ids / kn_bucket.  Workspace: about 88 bytes
 * per point (kn_workspace_bytes). */
int kn_eval_grouped(kn_ctx *ctx, const kn_scene *scene, void *stream, const float *points /*dev M*3*/,
                    const float *dirs /*dev M*3*/, int64_t M, float *sigma /*dev M*/,
                    float *rgb /*dev M*3*/, int32_t *cell_id /*dev M, nullable*/,
                    int32_t *counts /*dev N+1, nullable*/, int32_t *perm /*dev M, nullable*/,
                    void *workspace, int64_t workspace_bytes);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): kn_eval_grouped with the library's own scratch memory in place of the
 * workspace argument.  The scratch is a static device array of KN_STATIC_SCRATCH_BYTES that every GPU the library
 * runs on holds until the process ends; its address on the context's device is looked up by kn_create.
 * The call allocates nothing (no hipMalloc / hipFree, no events, no library routine that allocates) and records no
 * stage timings; inputs and outputs are the caller's, as in kn_eval_grouped, and the results are the same bits.
 * The context's device must be current (KN_E_INVALID_ARG otherwise).  To make the array go further this call sorts
 * indices instead of moving the points (slower per point on large batches, the same results), which takes about
 * 17 bytes per point + 24 per network; M is limited to what the array then holds (roughly 980,000 points on 4,096
 * networks): KN_E_STATIC_LIMIT beyond.
 * All calls on one GPU share the one array, whose contents do not outlive a call: calls that overlap on a GPU
 * (different streams or threads) race; calls on one stream are ordered as usual. */
#define KN_STATIC_SCRATCH_BYTES (16u << 20)
int kn_eval_grouped_static(kn_ctx *ctx, const kn_scene *scene, void *stream, const float *points /*dev M*3*/,
                           const float *dirs /*dev M*3*/, int64_t M, float *sigma /*dev M*/,
                           float *rgb /*dev M*3*/, int32_t *cell_id /*dev M, nullable*/,
                           int32_t *counts /*dev N+1, nullable*/, int32_t *perm /*dev M, nullable*/);

/* Sec. 3.4 sampling with empty-space skipping, one stage on its own: for each ray, starting at
 * lattice index k_begin[r] (0 if NULL), collect up to S kept samples.  Lattice: t_k = t_near +
 * (k + 1/2)*step, x_k = o + t_k*d (fp32, one fused multiply-add each), k < K; a sample is kept
 * iff x_k is inside the AABB and its occupancy voxel is non-zero (and, on a sparse grid, its cell
 * has a network).  out_k[r*S + j] = j-th kept
 * index (unused slots -1), out_count[r] = kept, out_k_next[r] (nullable) = where to resume
 * (K when the ray is exhausted). */
int kn_march(const kn_scene *scene, void *stream, const float *rays_o /*dev R*3*/,
             const float *rays_d /*dev R*3*/, int64_t R, float t_near, float step, int32_t K,
             const int32_t *k_begin /*dev R, nullable*/, int32_t S, int32_t *out_k /*dev R*S*/,
             int32_t *out_count /*dev R*/, int32_t *out_k_next /*dev R, nullable*/);

/* Sec. 3.4 "Sampling" (stratified sampling, as in NeRF): kn_march / kn_render with one uniform draw per lattice
 * interval instead of its midpoint: t_k = t_near + (k + u) * step, u in [0, 1) from a counter-based
 * generator keyed by (seed, ray number, k), the ray number being the ray's row in rays_o / rays_d:
 *     mix(v): v ^= v >> 16; v *= 0x85ebca6b; v ^= v >> 13; v *= 0xc2b2ae35; v ^= v >> 16   (uint32)
 *     u = (mix(mix(mix(seed) + ray) ^ k) >> 8) * 2^-24
 * The same seed gives the same picture; a new seed per frame gives independent draws.  In the render
 * sample k is blended with its own delta_k = t_(k+1) - t_k, the distance to the next lattice point
 * whether or not that point is kept (k + 1 = K included); everything else is as in kn_render. */
int kn_march_stratified(const kn_scene *scene, void *stream, const float *rays_o /*dev R*3*/,
                        const float *rays_d /*dev R*3*/, int64_t R, float t_near, float step, int32_t K,
                        uint32_t seed, const int32_t *k_begin /*dev R, nullable*/, int32_t S,
                        int32_t *out_k /*dev R*S*/, int32_t *out_count /*dev R*/,
                        int32_t *out_k_next /*dev R, nullable*/);
int kn_render_stratified(kn_ctx *ctx, const kn_scene *scene, void *stream, const float *rays_o /*dev R*3*/,
                         const float *rays_d /*dev R*3, unit*/, int64_t R, float t_near, float step,
                         int32_t K, float term_eps, const float bg[3] /*host*/, uint32_t seed,
                         float *rgb_out /*dev R*3*/, kn_render_stats *stats /*host, nullable*/,
                         void *workspace, int64_t workspace_bytes);

/* Eq. 2-4 with early ray termination (Sec. 3.4), one stage on its own: ray r owns samples
 * offsets[r] .. offsets[r+1]-1 of sigma / rgb in front-to-back order; alpha = 1 - exp(-sigma*step),
 * C += T*alpha*c, T *= 1 - alpha, stop after a sample leaves T < term_eps (0 = never);
 * rgb_out = C + T*bg.  T_out / n_used are optional per-ray outputs. */
int kn_composite(void *stream, const float *sigma /*dev*/, const float *rgb /*dev n*3*/,
                 const int32_t *offsets /*dev R+1*/, int64_t R, float step, float term_eps,
                 const float bg[3] /*host*/, float *rgb_out /*dev R*3*/, float *T_out /*dev R, nullable*/,
                 int32_t *n_used /*dev R, nullable*/);
/* The same with a delta per sample (Eq. 4's delta_i; what stratified samples carry): alpha_i = 1 - exp(-sigma_i*delta_i). */
int kn_composite_deltas(void *stream, const float *sigma /*dev*/, const float *rgb /*dev n*3*/,
                        const float *delta /*dev n*/, const int32_t *offsets /*dev R+1*/, int64_t R, float term_eps,
                        const float bg[3] /*host*/, float *rgb_out /*dev R*3*/, float *T_out /*dev R, nullable*/,
                        int32_t *n_used /*dev R, nullable*/);

/* The whole path (Sec. 3.1 Eq. 1-4, Sec. 3.2, Sec. 3.4): render R rays.  Samples are taken in
 * waves from near to far; rays whose transmittance fell below term_eps, or that ran out of
 * lattice points, drop out between waves.  The result per ray equals the sequential definition
 * (march, evaluate, blend, stop at T < term_eps) regardless of how waves are cut.
 * R*2^ceil(log2 K) must be <= 2^32, R times the slot budget per ray (kn_set_render_params; 128 unless set)
 * below 2^31, and R <= 2^26: KN_E_UNSUPPORTED beyond.  The call enqueues the first two waves without looking at their outcome
 * (their shape is computed on the device) and reads the count of surviving rays on the host only to decide
 * about further waves; when it returns, the last wave has been enqueued but `stream` may still be running
 * (it does not wait at all when the slot budget guarantees that the second wave ends every ray and `stats`
 * is NULL).  Work of successive calls on one stream is ordered as usual.  Calls on different streams (and from
 * different threads) may be in flight at the same time on one scene, through one context or several, each with a
 * workspace and an output buffer of its own; one stream must not be used by two calls at once.  A context keeps 8
 * host mailboxes, one per stream with a call in flight (a mailbox whose last call has reported is handed to the
 * next stream that needs one); calls beyond that wait for their stream instead of polling.  The wave schedule is
 * read once, when the call starts (KN_E_WORKSPACE if the workspace does not fit it).  With profiling on, calls
 * on one context must not overlap: their events would interleave. */
int kn_render(kn_ctx *ctx, const kn_scene *scene, void *stream, const float *rays_o /*dev R*3*/,
              const float *rays_d /*dev R*3, unit*/, int64_t R, float t_near, float step,
              int32_t K /*max lattice points per ray*/, float term_eps /*0 = off*/,
              const float bg[3] /*host*/, float *rgb_out /*dev R*3*/,
              kn_render_stats *stats /*host, nullable*/, void *workspace, int64_t workspace_bytes);

/* Sec. 3.5: the same function as kn_eval_grouped, evaluated one layer at a time: per layer one
 * variable-batch grouped matrix product (a separate product per network, batch sizes that differ
 * from network to network) over the batch ordered by network, activations written to and read
 * from device memory between the layers (320 + 4*H bytes per point of workspace on top of
 * kn_eval_grouped's).  Same operands and order of operations as the fused kernel, so the results
 * are the same bits; it is the comparison point that shows what the fusion buys, not the fast
 * path.  16-bit scenes only (KN_E_UNSUPPORTED for KN_F32). */
int kn_layered_workspace_bytes(const kn_scene *scene, int64_t max_points, int64_t *out_bytes);
int kn_eval_grouped_layered(kn_ctx *ctx, const kn_scene *scene, void *stream, const float *points /*dev M*3*/,
                            const float *dirs /*dev M*3*/, int64_t M, float *sigma /*dev M*/,
                            float *rgb /*dev M*3*/, void *workspace, int64_t workspace_bytes);

/* Sec. 3.4 ("Empty Space Skipping"; tau: Sec. 4.1): fill an occupancy grid of resolution occ_res
 * over the scene's AABB.  The density is sampled on a 3x3x3 subgrid of every voxel and the voxel
 * is marked (byte 1, else 0) iff any of the 27 densities is above tau (strictly).  The density
 * field is the scene's own network grid (the paper samples its teacher model); a probe is
 * evaluated by the network of the cell it lies in (Eq. 6; density 0 in a cell without a network),
 * whether or not occ_res is a multiple of the network grid.  The paper does not place the subgrid; it sits at the sub-cell centres, per
 * axis x = b_min + (v + c) * cell, c in {1/6, 1/2, 5/6}, cell = (b_max - b_min) / occ_res, taken
 * in fp32 as fma((float)v + c, cell, b_min).  Only layers 1-3 of the networks run (the density
 * does not depend on the direction), with the scene's arithmetic (fp32, or 16-bit operands).
 * occupancy: dev, occ_res[0]*occ_res[1]*occ_res[2] bytes, x slowest -- the format kn_scene_desc
 * takes; any occupancy grid the scene itself was created with plays no role.  The workspace
 * (kn_extract_workspace_bytes, dev, 256-byte aligned) holds small index tables.  Asynchronous on
 * `stream`.  KN_E_UNSUPPORTED above 2^31-1 voxels, or when one network cell would own more than
 * about 79 million voxels. */
int kn_extract_workspace_bytes(const kn_scene *scene, int64_t *out_bytes);
int kn_extract_occupancy(kn_ctx *ctx, const kn_scene *scene, void *stream, const int32_t occ_res[3] /*host*/,
                         float tau, uint8_t *occupancy /*dev, out*/, void *workspace,
                         int64_t workspace_bytes);

/* The wave schedule of kn_render on this context (defaults are used otherwise):
 * samples per ray in the first wave (default max(48, K / 16), at most the slot budget), the slot
 * budget per ray (default 128; sizes the workspace, see kn_workspace_bytes; later waves share the budget out
 * among the surviving rays), and the factor by which the samples per ray grow from one wave to the next
 * (default 32).  Values <= 0 restore the default.  Calls already running keep the schedule they started with. */
int kn_set_render_params(kn_ctx *ctx, int32_t first_wave_samples, int32_t slots_per_ray, int32_t wave_growth);

/* Limits that decide between code paths, per context, so that small inputs can reach the paths of large ones (for
 * tests; value <= 0 restores the default):
 *   KN_OPT_GROUP_FUSED_MAX          largest number of networks whose per-network counters kn_render's grouping keeps
 *                                   in LDS one by one (default 8192; 0 is a valid value here: always the hash path;
 *                                   negative restores the default)
 *   KN_OPT_GROUP_HASH_SLOTS         slots of the LDS hash table used beyond that (power of two, 16 .. 2048)
 * and one setting of the stage timing (kn_profile_enable):
 *   KN_OPT_PROFILE_EVERY            events are recorded on one call in this many, counted from the moment timing is
 *                                   switched on or this option is set (default 1: every call); a benchmark that times
 *                                   a run of frames disturbs it less that way */
typedef enum { KN_OPT_GROUP_FUSED_MAX = 1, KN_OPT_GROUP_HASH_SLOTS = 2, KN_OPT_PROFILE_EVERY = 3 } kn_option;
int kn_set_option(kn_ctx *ctx, int32_t option, int64_t value);

/* Per-stage device time of kn_render / kn_eval_grouped on this context, measured with HIP events recorded on
 * the caller's stream around each stage (off by default).  Recording does not
 * synchronise; kn_profile_read synchronises the recorded stream, settles all pending intervals and
 * copies the totals accumulated since the last reset. */
typedef struct {
    double ms_cell;        /* point -> cell id (kn_eval_grouped only; fused into marching in kn_render) */
    double ms_march;       /* marching + empty-space skipping (kn_render: the per-wave marching kernel)  */
    double ms_bucket;      /* ordering by network: radix passes / grouping passes, offsets, tile list   */
    double ms_mlp;         /* the fused grouped-MLP kernel                                             */
    double ms_blend;       /* blending + early termination + live-ray compaction                       */
    int64_t mlp_launches;  /* launches of the grouped-MLP kernel                                       */
    int64_t mlp_samples;   /* samples those launches evaluated                                         */
    int64_t bucket_keys;   /* keys sorted (incl. unused slots)                                         */
    int64_t calls;         /* kn_render + kn_eval_grouped calls                                        */
    double ms_setup;       /* kn_render: ray clipping / first live list, and live-list compaction between waves */
} kn_profile;
/* on: 0 = off, 1 = every stage, 2 = only the grouped-MLP kernel, 3 = only the marching kernel (fewer events on
 * the stream: less disturbance of the run that is being timed; mlp_samples / bucket_keys / calls are not
 * gathered in modes 2 and 3, because reading them back would make kn_render wait for the frame).  Modes 1 and 3
 * time the interval between two events recorded on the stream (launch gaps included); in mode 2 the events take the
 * start and stop time stamps of the kernel's own dispatch, so ms_mlp is the kernel's execution time. */
int kn_profile_enable(kn_ctx *ctx, int on);
int kn_profile_read(kn_ctx *ctx, kn_profile *out /*host*/, int reset);

#ifdef __cplusplus
}
#endif
#endif
