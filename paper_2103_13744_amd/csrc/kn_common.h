// Internal declarations shared by the HIP translation units of libkilonerf_hip.so.
#pragma once

#include <hip/hip_runtime.h>
#include <mutex>
#include <stdint.h>

#include "kilonerf.h"

#define KN_WAVE 64
#define KN_MAX_CELLS (1 << 24) // cells of a sparse network grid

// Uniform grid over the scene AABB (Sec. 3.2).  `cell` is the fp32 quotient (b_max - b_min) / r
// computed once on the host, so that Eq. 6 is evaluated as floor((x - b_min) / cell) with the
// same two roundings everywhere.
struct KnGrid {
    float bmin[3];
    float cell[3];
    int32_t res[3];
};

// One unit of work of the grouped MLP kernels: `len` consecutive entries of the sorted sample
// list, all belonging to network `net`.
struct KnTile {
    int32_t net;
    int32_t start;
    int32_t len;
    int32_t pad;
};

constexpr int KN_MAILBOXES = 8;
// Host-visible mailbox (pinned, device-mapped, 8 words): kn_render's kernels post the live-ray count of a wave
// there, {sequence number, value, totals...}, and the host polls it instead of draining the stream.
struct KnMailbox {
    volatile unsigned long long *host; // nullptr: could not be allocated (the caller falls back to synchronising)
    unsigned long long *dev;
    unsigned long long seq;            // last sequence number handed out
    unsigned long long last_posted;    // sequence number of the last post a call asked its kernels for
    unsigned long long last_use;       // value of the context's use counter when a call last took it
    hipStream_t stream;                // owner, once taken
    bool taken;
};

enum KnStage { KN_ST_CELL = 0, KN_ST_MARCH, KN_ST_BUCKET, KN_ST_MLP, KN_ST_BLEND, KN_ST_SETUP, KN_ST_NONE };
constexpr int KN_N_EVENTS = 1024;
constexpr int KN_DEFAULT_SLOTS = 128, KN_DEFAULT_GROWTH = 32;
constexpr int KN_GROUP_FUSED_MAX_BINS = 8192; // largest grid whose histogram the grouping's fill pass scans by itself
constexpr int KN_GROUP_HASH_SLOTS_MAX = 2048; // larger grids: LDS table of the bins a workgroup meets (power of two)

// Everything mutable lives here (the scene is immutable once created).  `mutex` guards all fields below `device`.
struct kn_ctx {
    int device;
    std::mutex mutex;
    // wave schedule of kn_render (0 / defaults: see kn_set_render_params)
    int32_t first_wave_samples, slots_per_ray, wave_growth;
    // limits that decide between code paths (kn_set_option)
    int32_t group_fused_max, group_hash_slots;
    // stage timing: an event ring; intervals are settled (one stream synchronise, then hipEventElapsedTime for
    // each recorded interval) only when the ring is full, when another stream starts recording, or when the
    // totals are read
    kn_profile profile;
    bool profile_on;
    int32_t profile_every; // events on one call in this many (kn_set_option)
    int64_t profile_call;  // calls seen since profiling was switched on
    int only_stage;       // KN_ST_NONE, or the one stage that is being timed (then sample counts are not gathered)
    hipEvent_t events[KN_N_EVENTS];
    int event_stage[KN_N_EVENTS];
    int n_events;
    hipStream_t event_stream;
    bool events_ready;
    // One mailbox per stream with a render call in flight (posts of one stream arrive in order; posts of two
    // streams would overwrite each other).
    KnMailbox mailbox[KN_MAILBOXES];
    unsigned long long use_counter;
    void *static_scratch; // device address of the library's static scratch array on this device
};
// snapshot of the schedule and limits, taken under the mutex at the start of a call
struct KnKnobs {
    int32_t first_wave_samples, slots_per_ray, wave_growth, group_fused_max, group_hash_slots;
};
KnKnobs kn_knobs(const kn_ctx *ctx);

struct kn_scene {
    kn_scene_desc desc;
    int32_t N;             // number of networks
    int64_t cells;         // cells of the network grid (= N unless the grid is sparse)
    int32_t *cell_net;     // device, sparse grids only (else nullptr): cell -> network index in [0, N) or -1
    int64_t P;             // parameters per network
    int device;
    KnGrid net_grid;
    KnGrid occ_grid;
    bool has_occ;
    uint32_t *occ_bits;    // device, one bit per voxel, linear voxel index = bit index
    void *packed_w;        // device, matrix-core operand order (16-bit types only)
    int64_t packed_halfs_per_net;
    // Coarse skip field over the occupancy grid: one byte per block of KN_SKIP_BLOCK^3 voxels holding
    // the Chebyshev distance, in blocks, to the nearest block with an occupied voxel (0 = occupied
    // block, capped at KN_SKIP_MAX).  Lets marching jump over provably empty lattice points.
    uint8_t *skip_dist;    // device, skip_res[0]*[1]*[2] bytes, x slowest; nullptr without occupancy
    int32_t skip_res[3];
    // Box around all occupied voxels, as a sub-grid of the occupancy grid (whole skip blocks; the network
    // grid's box without occupancy; res = 0 when nothing is occupied): rays are clipped against it.
    KnGrid content_box;
    void *own_buffer;      // device memory the library allocated for the scene's data (nullptr: the caller lent it)
};
#define KN_SKIP_BLOCK 4
#define KN_SKIP_MAX 32

// Host-side launch helpers ----------------------------------------------------------------------
extern thread_local int g_kn_last_hip_error;
#define KN_HIP(call)                                        \
    do {                                                    \
        hipError_t e_ = (call);                             \
        if (e_ != hipSuccess) {                             \
            g_kn_last_hip_error = (int)e_;                  \
            return KN_E_HIP;                                \
        }                                                   \
    } while (0)
#define KN_CHECK_LAUNCH() KN_HIP(hipGetLastError())
#define KN_TRY(expr)                  \
    do {                              \
        int s_ = (expr);              \
        if (s_ != KN_OK) return s_;   \
    } while (0)

static inline int64_t kn_align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
static inline int64_t kn_div_up(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Bump allocator over the caller's workspace: carve() returns nullptr once the space is exhausted.
struct KnCarver {
    char *base;
    int64_t size, used;
    KnCarver(void *p, int64_t bytes) : base((char *)p), size(bytes), used(0) {}
    template <typename T> T *carve(int64_t n)
    {
        int64_t bytes = kn_align_up((n > 0 ? n : 1) * (int64_t)sizeof(T), 256);
        T *p = (base && used + bytes <= size) ? (T *)(base + used) : nullptr;
        used += bytes;
        return p;
    }
    bool ok() const { return base != nullptr && used <= size; }
};

// Device helpers --------------------------------------------------------------------------------
// Eq. 6 for one point; returns the linear index (x slowest) or -1 outside / non-finite.
__device__ __forceinline__ int32_t kn_grid_index(const KnGrid &g, float x, float y, float z)
{
    float ux = (x - g.bmin[0]) / g.cell[0];
    float uy = (y - g.bmin[1]) / g.cell[1];
    float uz = (z - g.bmin[2]) / g.cell[2];
    float fx = floorf(ux), fy = floorf(uy), fz = floorf(uz);
    bool in = (fx >= 0.0f) && (fx < (float)g.res[0]) && (fy >= 0.0f) && (fy < (float)g.res[1]) &&
              (fz >= 0.0f) && (fz < (float)g.res[2]);
    if (!in) return -1;
    return ((int32_t)fx * g.res[1] + (int32_t)fy) * g.res[2] + (int32_t)fz;
}

// Network of a cell: the cell itself on a dense grid, the table's entry (-1 = none) on a sparse one.
__device__ __forceinline__ int32_t kn_net_of_cell(const int32_t *__restrict__ cell_net, int32_t cell)
{
    return (cell_net != nullptr && cell >= 0) ? cell_net[cell] : cell;
}

// Stratified sampling (Sec. 3.4 "Sampling"): lattice point k of a ray sits at offset u in [0, 1) of its interval,
// u = (mix(mix(mix(seed) + ray) ^ k) >> 8) * 2^-24 with the 32-bit finalizer of MurmurHash3 as mix.  The host
// passes seed_key = mix(seed); a kernel forms ray_key = mix(seed_key + ray) once per ray.
__host__ __device__ __forceinline__ uint32_t kn_mix32(uint32_t v)
{
    v ^= v >> 16;
    v *= 0x85ebca6bu;
    v ^= v >> 13;
    v *= 0xc2b2ae35u;
    v ^= v >> 16;
    return v;
}
__device__ __forceinline__ float kn_strat_offset(uint32_t ray_key, int32_t k)
{
    return (float)(kn_mix32(ray_key ^ (uint32_t)k) >> 8) * (1.0f / 16777216.0f);
}

// Lattice point k of a ray (Sec. 3.4): t_k = t_near + (k + offset) step, x = o + t_k d; offset = 1/2, or the
// stratified draw of (ray, k).
template <bool STRAT = false>
__device__ __forceinline__ float kn_lattice_t(float t_near, float step, int32_t k, uint32_t ray_key = 0u)
{
    float off = 0.5f;
    if constexpr (STRAT) off = kn_strat_offset(ray_key, k);
    return fmaf((float)k + off, step, t_near);
}
template <bool STRAT = false>
__device__ __forceinline__ void kn_lattice_point(float ox, float oy, float oz, float dx, float dy,
                                                 float dz, float t_near, float step, int32_t k,
                                                 float &x, float &y, float &z, uint32_t ray_key = 0u)
{
    float t = kn_lattice_t<STRAT>(t_near, step, k, ray_key);
    x = fmaf(t, dx, ox);
    y = fmaf(t, dy, oy);
    z = fmaf(t, dz, oz);
}

// Block-wide sum and exclusive prefix sum for blocks of whole wavefronts, up to 1024 threads (a scan inside each
// wavefront, `lds` (16 ints) across wavefronts).  Every thread of the block must call them.
// Inclusive prefix sums over a wavefront whose 64 lanes are all active, with data-parallel-primitive shifts: four
// steps inside each row of 16 lanes, then the last lane of a row is added to the next row (row_bcast:15 into rows 1
// and 3) and lane 31 to the upper half (row_bcast:31 into rows 2 and 3).  No trip through the LDS crossbar.
__device__ __forceinline__ int32_t kn_wave_inclusive_scan(int32_t v)
{
    constexpr int ROW_SHR = 0x110, ROW_BCAST15 = 0x142, ROW_BCAST31 = 0x143; // dpp_ctrl encodings
    v += __builtin_amdgcn_update_dpp(0, v, ROW_SHR + 1, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, ROW_SHR + 2, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, ROW_SHR + 4, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, ROW_SHR + 8, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, ROW_BCAST15, 0xa, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, ROW_BCAST31, 0xc, 0xf, true);
    return v;
}
// (both block-wide helpers: every thread of the workgroup must call them, from uniform control flow)
__device__ __forceinline__ int32_t kn_block_sum(int32_t v, int32_t *lds)
{
    v = __builtin_amdgcn_readlane(kn_wave_inclusive_scan(v), KN_WAVE - 1);
    __syncthreads();
    if ((threadIdx.x & (KN_WAVE - 1)) == 0) lds[threadIdx.x / KN_WAVE] = v;
    __syncthreads();
    int32_t all = 0;
    for (int w = 0; w < (int)(blockDim.x / KN_WAVE); ++w) all += lds[w];
    return all;
}
__device__ __forceinline__ int32_t kn_block_exclusive_scan(int32_t v, int32_t *lds, int32_t &total)
{
    const int lane = threadIdx.x & (KN_WAVE - 1), wv = threadIdx.x / KN_WAVE;
    const int32_t inc = kn_wave_inclusive_scan(v);
    __syncthreads();
    if (lane == KN_WAVE - 1) lds[wv] = inc;
    __syncthreads();
    int32_t before = 0, all = 0;
    for (int w = 0; w < (int)(blockDim.x / KN_WAVE); ++w) {
        const int32_t s = lds[w];
        all += s;
        if (w < wv) before += s;
    }
    total = all;
    return before + inc - v;
}

// Stage entry points implemented across the translation units (host functions) -----------------
int64_t kn_bucket_ws_bytes(int64_t M, int32_t N);
int64_t kn_max_tiles(int64_t M, int32_t N, int32_t tile_len);

struct KnBucketOut {
    const int32_t *perm;    // M sorted sample indices
    const int32_t *counts;  // N+1
    const int32_t *offsets; // N+2
    const KnTile *tiles;    // up to kn_max_tiles entries
    const int32_t *n_tiles; // device scalar
};

// Sorts `keys` (values in [0, N], N = outside/unused) stably (kn_reorder.hip), fills perm/counts/offsets/tiles in
// workspace memory (or the user's buffers where given).  keys is overwritten.
int kn_bucket_run(hipStream_t st, int32_t *keys, int64_t M, int32_t N, int32_t tile_len, int32_t *user_counts, int32_t *user_offsets,
                  int32_t *user_perm, KnCarver &ws, KnBucketOut *out);
// Physical re-ordering of a batch of points by network, for kn_eval_grouped: cell ids and keys (Eq. 6), then a stable
// radix sort that moves the samples themselves (records[0], records[1]: see KnSampleSrc::records).  out->perm is nullptr;
// user_ids / user_counts / user_perm (nullable) receive what kn_eval_grouped reports.  M >= 1.
// *out4: staging array of the results, (r, g, b, sigma) per point in caller order, already zero for the points without
// a network; the MLP kernel fills the rest (KnSampleSrc::out4), kn_reorder_split_results copies it to sigma / rgb.
int64_t kn_reorder_ws_bytes(int64_t M, int32_t N);
struct KnStageTimer;
int kn_reorder_run(const kn_scene *sc, hipStream_t st, const float *points, const float *dirs, int64_t M, int32_t tile_len,
                   int32_t *user_ids, int32_t *user_counts, int32_t *user_perm, KnCarver &ws, KnBucketOut *out,
                   const uint32_t *records[2], float **out4, KnStageTimer *tm /* nullable: marks the end of the cell-id stage */);
int kn_reorder_configure(); // once per device: lifts the dynamic-LDS limit of the scatter kernels
int kn_reorder_split_results(hipStream_t st, const float *out4, int64_t M, float *sigma, float *rgb);
// Unstable grouping of a render wave's samples (row layout: row i holds cnt[i] samples in slots i*S ..).
// out->perm lists slot numbers group by group, in no particular order inside a group or between groups;
// out->counts / out->offsets are not produced.
//
// `hist` (N ints) holds the wave's histogram, accumulated by the caller (the marching kernel) on a zeroed array;
// `cursor` are the N ints behind it.  Where kn_group_fused(N) holds (small grids: the fill pass derives the
// offsets itself) `cursor` must be zero before the run and the caller clears both arrays afterwards; otherwise
// kn_group_run leaves the histogram zero and overwrites the cursors.  hash_slots: size of the LDS hash
// table (a power of two) that kernels use for per-workgroup counters where a counter per network does not fit.
inline bool kn_group_fused(const KnKnobs &k, int32_t N) { return N <= k.group_fused_max; }
int kn_group_configure(); // once per device: lifts the dynamic-LDS limit of the grouping kernels
struct KnGroupWs {
    int32_t *hist, *cursor, *n_tiles, *perm;
    KnTile *tiles;
};
int64_t kn_group_ws_bytes(int64_t slots, int32_t N);
void kn_group_carve(KnCarver &ws, int64_t slots, int32_t N, KnGroupWs *w);
// ctl (device): ctl[0] = number of rows, ctl[1] = S; max_rows: host-side upper bound of ctl[0] (sizes the grid).
int kn_group_run(hipStream_t st, const KnKnobs &knobs, const int32_t *row_keys, const int32_t *cnt, const int32_t *ctl,
                 int64_t max_rows, int32_t N, int32_t tile_len, const KnGroupWs &w, KnBucketOut *out);

// Sample source of the grouped MLP kernels: either explicit points/dirs (eval_grouped) or the
// packed (ray, k) records of a render wave.
struct KnSampleSrc {
    const float *points;   // M*3 or nullptr
    const float *dirs;     // M*3 or nullptr
    // eval_grouped after the physical re-ordering (kn_reorder_run): the samples in grouped order, 4 words each in two
    // arrays, (x, y, z, key) and (dx, dy, dz, caller index); then the sorted list is the samples themselves and
    // `perm` is not read
    const uint32_t *records, *records_dir;
    const uint32_t *rec;   // per sample: ray << kbits | k   (render)
    const float *rays_o;   // R*3
    const float *rays_d;   // R*3
    float t_near, step;
    int32_t kbits;
    float *out4;           // render: (r, g, b, sigma) per sample, 16 bytes each; nullptr = separate sigma / rgb arrays
    // Stratified sampling (render only): lattice points sit at their drawn offsets, and the density that goes to
    // out4 is scaled by delta_k / step, delta_k = t_(k+1) - t_k, so that the blend's exp(-sigma * step) is Eq. 4
    // with the sample's own delta.
    int32_t strat;         // 0 = midpoint lattice
    uint32_t seed_key;     // kn_mix32(seed)
    // render, 16-bit scenes: gamma(d) per ray, already rounded and in the operand order of the direction block of the
    // last hidden layer: 4 lane groups x 16 bytes per ray (written by the render's set-up kernel for the rays that live)
    const uint16_t *dir_table;
};

// ev_start / ev_stop (both or neither): HIP events that take the kernel's own start and stop time stamps (the
// extended launch call: no marker packets on the stream around the kernel)
int kn_mlp_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b,
                  int64_t M, float *sigma, float *rgb, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
int kn_mlp_pack_weights(kn_scene *sc, hipStream_t st);
int kn_mlp_tile_len(const kn_scene *sc);

int kn_fill_i32(hipStream_t st, int32_t *p, int64_t n, int32_t v);

// Optional per-stage timing with HIP events on the caller's stream (see kn_profile in the header).
// begin() records a start event, mark(stage) an event that closes an interval charged to `stage`.
// Elapsed times are read later, in batches (kn_profile_read forces it), so recording does not
// synchronise the stream.  `allowed` false: never record (for calls that must not allocate: creating the events does).
struct KnStageTimer {
    kn_ctx *ctx;
    hipStream_t st;
    bool on;
    bool counts; // every stage is timed: sample counts are gathered as well
    KnStageTimer(kn_ctx *c, hipStream_t s, bool allowed = true);
    void begin() { mark(KN_ST_NONE); }
    void mark(int stage_id);
    // Where only one stage is being timed and that stage is one kernel (the grouped MLP), the kernel's dispatch takes its
    // own start and stop time stamps instead of marks around it: the two events for the launch, or false (events
    // untouched) when `stage_id` is not timed that way.
    bool kernel_events(int stage_id, hipEvent_t *start, hipEvent_t *stop);
    // totals that are counted, not timed
    void add(int64_t mlp_launches, int64_t mlp_samples, int64_t bucket_keys, int64_t calls);
};
