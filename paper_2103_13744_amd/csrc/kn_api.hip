// Host side of the C ABI: scene objects, validation, workspace sizing, kn_eval_grouped.
#include "kn_common.h"
#include "kn_probe.h"

#include <math.h>
#include <new>
#include <string.h>
#include <vector>

thread_local int g_kn_last_hip_error = 0;

int kn_cell_keys(const kn_scene *sc, hipStream_t st, const float *points, int64_t M, int32_t *ids, int32_t *keys);
int64_t kn_render_ws_bytes(const kn_scene *sc, int64_t R, int32_t slots_per_ray);
int kn_mlp_f32_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t max_tiles,
                      float *sigma, float *rgb, hipEvent_t ev_start, hipEvent_t ev_stop);
int kn_mlp_mfma_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t max_tiles,
                       float *sigma, float *rgb, hipEvent_t ev_start, hipEvent_t ev_stop);
int kn_mlp_mfma_tile_len(const kn_scene *sc);
int kn_mlp_f32_tile_len(const kn_scene *sc);
int kn_mlp_f32_pack_weights(kn_scene *sc, hipStream_t st);
int kn_probe_mfma_launch(const kn_scene *sc, hipStream_t st, const KnProbeJob &job);
int kn_probe_f32_launch(const kn_scene *sc, hipStream_t st, const KnProbeJob &job);
int64_t kn_layered_act_bytes(const kn_scene *sc, int64_t M);
int kn_mlp_layered_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t M,
                          int64_t max_tiles, void *acts, float *sigma, float *rgb);

int64_t kn_mlp_packed_bytes(int32_t H, int64_t N);
int64_t kn_mlp_f32_packed_bytes(int32_t H, int64_t N);

// Scratch memory of kn_eval_grouped_static, the entry point for callers that cannot allocate: a file-scope device
// array that every GPU the library runs on holds until the process ends.  In host code the array's name is only a
// stand-in for the symbol, not a device address; the address on a device comes from hipGetSymbolAddress with that
// device current (static_scratch_address, called by kn_create), and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[KN_STATIC_SCRATCH_BYTES];
constexpr int KN_MAX_DEVICES = 64;
static void *g_scratch_ptr[KN_MAX_DEVICES] = {};
static bool g_device_configured[KN_MAX_DEVICES] = {};
static std::mutex g_device_mutex;

// once per device, with that device current: the address of the device's copy of `scratch`
static int static_scratch_address(int dev, void **out)
{
    if (dev < 0 || dev >= KN_MAX_DEVICES) return KN_E_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_device_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        KN_HIP(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr & 255)) return KN_E_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    if (!g_device_configured[dev]) {
        KN_TRY(kn_group_configure());
        KN_TRY(kn_reorder_configure());
        g_device_configured[dev] = true;
    }
    *out = g_scratch_ptr[dev];
    return KN_OK;
}

KnKnobs kn_knobs(const kn_ctx *c)
{
    kn_ctx *ctx = const_cast<kn_ctx *>(c); // (the mutex)
    std::lock_guard<std::mutex> lock(ctx->mutex);
    return KnKnobs{ctx->first_wave_samples, ctx->slots_per_ray, ctx->wave_growth, ctx->group_fused_max, ctx->group_hash_slots};
}

// (ctx->mutex held)
static int settle_events(kn_ctx *ctx)
{
    if (ctx->n_events >= 2) {
        KN_HIP(hipStreamSynchronize(ctx->event_stream));
        for (int i = 1; i < ctx->n_events; ++i) {
            float ms = 0.0f;
            if (ctx->event_stage[i] == KN_ST_NONE || hipEventElapsedTime(&ms, ctx->events[i - 1], ctx->events[i]) != hipSuccess)
                continue;
            switch (ctx->event_stage[i]) {
            case KN_ST_CELL: ctx->profile.ms_cell += ms; break;
            case KN_ST_MARCH: ctx->profile.ms_march += ms; break;
            case KN_ST_BUCKET: ctx->profile.ms_bucket += ms; break;
            case KN_ST_MLP: ctx->profile.ms_mlp += ms; break;
            case KN_ST_BLEND: ctx->profile.ms_blend += ms; break;
            case KN_ST_SETUP: ctx->profile.ms_setup += ms; break;
            default: break;
            }
        }
    }
    ctx->n_events = 0;
    return KN_OK;
}

KnStageTimer::KnStageTimer(kn_ctx *c, hipStream_t s, bool allowed) : ctx(c), st(s), on(false), counts(false)
{
    if (!allowed || !ctx) return;
    std::lock_guard<std::mutex> lock(ctx->mutex);
    on = ctx->profile_on && (ctx->profile_call++ % ctx->profile_every) == 0;
    if (on && !ctx->events_ready) {
        for (auto &e : ctx->events)
            if (hipEventCreate(&e) != hipSuccess) on = false;
        ctx->events_ready = on;
    }
    if (on && ctx->n_events > 0 && ctx->event_stream != s) (void)settle_events(ctx);
    if (on) ctx->event_stream = s;
    counts = on && ctx->only_stage == KN_ST_NONE;
}
void KnStageTimer::mark(int stage_id)
{
    if (!on) return;
    std::lock_guard<std::mutex> lock(ctx->mutex);
    if (ctx->only_stage == KN_ST_MLP) return; // that stage is one kernel: its launch takes the time stamps (kernel_events)
    if (ctx->only_stage != KN_ST_NONE) {
        // the mark before the stage of interest opens its interval; everything else is dropped
        const bool opens = stage_id == KN_ST_NONE || stage_id == KN_ST_SETUP;
        const bool closes = stage_id == ctx->only_stage;
        if (!opens && !closes) return;
        if (opens) stage_id = KN_ST_NONE;
    }
    if (ctx->n_events == KN_N_EVENTS) {
        (void)settle_events(ctx);
        if (stage_id != KN_ST_NONE) { // re-open the interval that the settle cut short
            ctx->event_stage[0] = KN_ST_NONE;
            (void)hipEventRecord(ctx->events[0], st);
            ctx->n_events = 1;
        }
    }
    ctx->event_stage[ctx->n_events] = stage_id;
    (void)hipEventRecord(ctx->events[ctx->n_events++], st);
}
bool KnStageTimer::kernel_events(int stage_id, hipEvent_t *start, hipEvent_t *stop)
{
    if (!on) return false;
    std::lock_guard<std::mutex> lock(ctx->mutex);
    if (ctx->only_stage != stage_id || stage_id != KN_ST_MLP) return false;
    if (ctx->n_events + 2 > KN_N_EVENTS) (void)settle_events(ctx);
    ctx->event_stage[ctx->n_events] = KN_ST_NONE;
    *start = ctx->events[ctx->n_events++];
    ctx->event_stage[ctx->n_events] = stage_id;
    *stop = ctx->events[ctx->n_events++];
    return true;
}
void KnStageTimer::add(int64_t mlp_launches, int64_t mlp_samples, int64_t bucket_keys, int64_t calls)
{
    if (!on) return;
    std::lock_guard<std::mutex> lock(ctx->mutex);
    ctx->profile.mlp_launches += mlp_launches;
    ctx->profile.mlp_samples += mlp_samples;
    ctx->profile.bucket_keys += bucket_keys;
    ctx->profile.calls += calls;
}

extern "C" int kn_profile_enable(kn_ctx *ctx, int on)
{
    if (!ctx) return KN_E_INVALID_ARG;
    std::lock_guard<std::mutex> lock(ctx->mutex);
    if (ctx->profile_on) (void)settle_events(ctx);
    ctx->profile_on = on != 0;
    ctx->profile_call = 0;
    ctx->only_stage = on == 2 ? KN_ST_MLP : on == 3 ? KN_ST_MARCH : KN_ST_NONE;
    return KN_OK;
}

extern "C" int kn_profile_read(kn_ctx *ctx, kn_profile *out, int reset)
{
    if (!ctx || !out) return KN_E_INVALID_ARG;
    std::lock_guard<std::mutex> lock(ctx->mutex);
    KN_TRY(settle_events(ctx));
    *out = ctx->profile;
    if (reset) ctx->profile = kn_profile{};
    return KN_OK;
}

extern "C" int kn_set_render_params(kn_ctx *ctx, int32_t first_wave_samples, int32_t slots_per_ray, int32_t wave_growth)
{
    if (!ctx) return KN_E_INVALID_ARG;
    std::lock_guard<std::mutex> lock(ctx->mutex);
    ctx->wave_growth = wave_growth >= 2 ? wave_growth : KN_DEFAULT_GROWTH;
    ctx->first_wave_samples = first_wave_samples > 0 ? first_wave_samples : 0;
    ctx->slots_per_ray = slots_per_ray > 0 ? slots_per_ray : KN_DEFAULT_SLOTS;
    if (ctx->slots_per_ray < ctx->first_wave_samples) ctx->slots_per_ray = ctx->first_wave_samples;
    return KN_OK;
}

extern "C" int kn_set_option(kn_ctx *ctx, int32_t option, int64_t value)
{
    if (!ctx) return KN_E_INVALID_ARG;
    std::lock_guard<std::mutex> lock(ctx->mutex);
    switch (option) {
    case KN_OPT_GROUP_FUSED_MAX:
        if (value > KN_GROUP_FUSED_MAX_BINS) return KN_E_INVALID_ARG;
        ctx->group_fused_max = value < 0 ? KN_GROUP_FUSED_MAX_BINS : (int32_t)value;
        return KN_OK;
    case KN_OPT_GROUP_HASH_SLOTS:
        if (value > 0 && (value < 16 || value > KN_GROUP_HASH_SLOTS_MAX || (value & (value - 1)) != 0)) return KN_E_INVALID_ARG;
        ctx->group_hash_slots = value <= 0 ? KN_GROUP_HASH_SLOTS_MAX : (int32_t)value;
        return KN_OK;
    case KN_OPT_PROFILE_EVERY:
        if (value > 0x7fffffffLL) return KN_E_INVALID_ARG;
        ctx->profile_every = value <= 0 ? 1 : (int32_t)value;
        ctx->profile_call = 0;
        return KN_OK;
    default: return KN_E_INVALID_ARG;
    }
}

extern "C" int kn_create(kn_ctx **out, int device_index)
{
    if (!out) return KN_E_INVALID_ARG;
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || device_index < 0 || device_index >= n_dev) return KN_E_NO_DEVICE;
    hipDeviceProp_t prop;
    KN_HIP(hipGetDeviceProperties(&prop, device_index));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return KN_E_NO_DEVICE;
    KN_HIP(hipSetDevice(device_index));
    void *scratch_ptr = nullptr;
    KN_TRY(static_scratch_address(device_index, &scratch_ptr));
    kn_ctx *ctx = new (std::nothrow) kn_ctx();
    if (!ctx) return KN_E_INVALID_ARG;
    ctx->device = device_index;
    ctx->first_wave_samples = 0;
    ctx->slots_per_ray = KN_DEFAULT_SLOTS;
    ctx->wave_growth = KN_DEFAULT_GROWTH;
    ctx->group_fused_max = KN_GROUP_FUSED_MAX_BINS;
    ctx->group_hash_slots = KN_GROUP_HASH_SLOTS_MAX;
    ctx->profile = kn_profile{};
    ctx->profile_on = false;
    ctx->profile_every = 1;
    ctx->profile_call = 0;
    ctx->only_stage = KN_ST_NONE;
    ctx->n_events = 0;
    ctx->event_stream = nullptr;
    ctx->events_ready = false;
    ctx->use_counter = 0;
    ctx->static_scratch = scratch_ptr;
    for (auto &m : ctx->mailbox) m = KnMailbox{nullptr, nullptr, 0ull, 0ull, 0ull, nullptr, false};
    void *hp = nullptr, *dp = nullptr;
    if (hipHostMalloc(&hp, 64 * KN_MAILBOXES, hipHostMallocMapped) == hipSuccess && hipHostGetDevicePointer(&dp, hp, 0) == hipSuccess) {
        memset(hp, 0, 64 * KN_MAILBOXES);
        for (int i = 0; i < KN_MAILBOXES; ++i) {
            ctx->mailbox[i].host = (volatile unsigned long long *)((char *)hp + 64 * i);
            ctx->mailbox[i].dev = (unsigned long long *)((char *)dp + 64 * i);
        }
    } else if (hp) {
        (void)hipHostFree(hp); // (kn_render then waits for its stream instead of polling)
    }
    *out = ctx;
    return KN_OK;
}

extern "C" int kn_destroy(kn_ctx *ctx)
{
    if (!ctx) return KN_OK;
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
    if (ctx->events_ready)
        for (auto &e : ctx->events) (void)hipEventDestroy(e);
    if (ctx->mailbox[0].host) (void)hipHostFree((void *)ctx->mailbox[0].host);
    delete ctx;
    return KN_OK;
}

namespace {

// one thread packs 32 consecutive voxels into one word (bit i of word w = voxel 32*w + i)
__global__ void k_pack_occupancy(const uint8_t *__restrict__ occ, int64_t n_vox, uint32_t *__restrict__ bits)
{
    const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w * 32 >= n_vox) return;
    uint32_t v = 0;
    for (int i = 0; i < 32; ++i) {
        const int64_t j = w * 32 + i;
        if (j < n_vox && occ[j] != 0) v |= (1u << i);
    }
    bits[w] = v;
}

// skip field, step 1: 0 for blocks of 4^3 voxels that contain an occupied voxel, 255 otherwise
__global__ void k_skip_seed(const uint8_t *__restrict__ occ, int ox, int oy, int oz, int sx, int sy, int sz,
                            uint8_t *__restrict__ dist)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= (int64_t)sx * sy * sz) return;
    const int cz = (int)(c % sz), cy = (int)((c / sz) % sy), cx = (int)(c / ((int64_t)sz * sy));
    bool any = false;
    for (int x = cx * KN_SKIP_BLOCK; x < min((cx + 1) * KN_SKIP_BLOCK, ox) && !any; ++x)
        for (int y = cy * KN_SKIP_BLOCK; y < min((cy + 1) * KN_SKIP_BLOCK, oy) && !any; ++y)
            for (int z = cz * KN_SKIP_BLOCK; z < min((cz + 1) * KN_SKIP_BLOCK, oz); ++z)
                if (occ[((int64_t)x * oy + y) * oz + z] != 0) { any = true; break; }
    dist[c] = any ? 0 : 255;
}

// skip field, step 2 (repeated): one Jacobi sweep of d = min(d, 1 + min over the 26 neighbours);
// after n sweeps every value <= n is the exact Chebyshev distance
__global__ void k_skip_sweep(const uint8_t *__restrict__ in, int sx, int sy, int sz, uint8_t *__restrict__ out)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= (int64_t)sx * sy * sz) return;
    const int cz = (int)(c % sz), cy = (int)((c / sz) % sy), cx = (int)(c / ((int64_t)sz * sy));
    int best = in[c];
    for (int x = max(cx - 1, 0); x <= min(cx + 1, sx - 1); ++x)
        for (int y = max(cy - 1, 0); y <= min(cy + 1, sy - 1); ++y)
            for (int z = max(cz - 1, 0); z <= min(cz + 1, sz - 1); ++z)
                best = min(best, (int)in[((int64_t)x * sy + y) * sz + z] + 1);
    out[c] = (uint8_t)min(best, 255);
}

__global__ void k_skip_cap(uint8_t *__restrict__ d, int64_t n)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c < n && d[c] > KN_SKIP_MAX) d[c] = KN_SKIP_MAX;
}

// zero the outputs of the points that fell outside the AABB (bucket N of the sorted list)
__global__ void k_zero_outside(const int32_t *__restrict__ perm, const int32_t *__restrict__ offsets, int32_t N, int64_t M,
                               float *__restrict__ sigma, float *__restrict__ rgb)
{
    const int64_t first = offsets[N];
    const int64_t j = first + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= M) return;
    const int64_t idx = perm[j];
    sigma[idx] = 0.0f;
    rgb[3 * idx] = rgb[3 * idx + 1] = rgb[3 * idx + 2] = 0.0f;
}

// the library's copy of a sparse grid's table: entries outside [0, n_nets) become -1 (no network)
__global__ void k_copy_cell_net(const int32_t *__restrict__ in, int64_t cells, int32_t n_nets, int32_t *__restrict__ out)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= cells) return;
    const int32_t v = in[c];
    out[c] = (v >= 0 && v < n_nets) ? v : -1;
}

bool make_grid(const float bmin[3], const float bmax[3], const int32_t res[3], KnGrid &g)
{
    for (int a = 0; a < 3; ++a) {
        if (res[a] < 1 || !isfinite(bmin[a]) || !isfinite(bmax[a]) || !(bmax[a] > bmin[a])) return false;
        const float extent = bmax[a] - bmin[a];
        const float cell = extent / (float)res[a]; // Eq. 6: (b_max - b_min) / r in fp32
        if (!isfinite(cell) || !(cell > 0.0f)) return false;
        g.bmin[a] = bmin[a];
        g.cell[a] = cell;
        g.res[a] = res[a];
    }
    return true;
}

} // namespace

extern "C" const char *kn_error_string(int status)
{
    switch (status) {
    case KN_OK: return "ok";
    case KN_E_INVALID_ARG: return "invalid argument";
    case KN_E_UNSUPPORTED: return "unsupported configuration";
    case KN_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case KN_E_HIP: return "HIP runtime error";
    case KN_E_NO_DEVICE: return "no usable gfx950 device";
    case KN_E_STATIC_LIMIT: return "input needs more scratch memory than the static buffer of kn_eval_grouped_static holds";
    default: return "unknown status";
    }
}

extern "C" int kn_last_hip_error(void) { return g_kn_last_hip_error; }

extern "C" int64_t kn_params_per_net(int32_t H, int32_t L_pos, int32_t L_dir)
{
    if (H < 1 || L_pos < 0 || L_dir < 0 || H > 4096 || L_pos > 64 || L_dir > 64) return -1;
    const int64_t ex = 3 + 6 * (int64_t)L_pos, ed = 3 + 6 * (int64_t)L_dir, h = H;
    return (ex * h + h) + (h * h + h) + (h * (h + 1) + (h + 1)) + ((h + ed) * h + h) + (h * 3 + 3);
}

static int validate_desc(const kn_scene_desc *d)
{
    if (!d || !d->weights) return KN_E_INVALID_ARG;
    KnGrid g;
    if (!make_grid(d->aabb_min, d->aabb_max, d->res, g)) return KN_E_INVALID_ARG;
    const int64_t n = (int64_t)d->res[0] * d->res[1] * d->res[2];
    if (d->cell_net) { // sparse grid: many cells, the networks are what is limited
        if (d->n_nets < 1) return KN_E_INVALID_ARG;
        if (n > KN_MAX_CELLS || d->n_nets > 65535) return KN_E_UNSUPPORTED;
    } else if (n > 65535) {
        return KN_E_UNSUPPORTED;
    }
    if (d->wdtype != KN_F32 && d->wdtype != KN_F16 && d->wdtype != KN_BF16) return KN_E_INVALID_ARG;
    if (d->hidden < 1 || d->L_pos < 0 || d->L_dir < 0) return KN_E_INVALID_ARG;
    if ((d->hidden != 32 && d->hidden != 64) || d->L_pos != 10 || d->L_dir != 4) return KN_E_UNSUPPORTED;
    const bool any = d->occ_res[0] || d->occ_res[1] || d->occ_res[2];
    if (any) {
        if (!d->occupancy) return KN_E_INVALID_ARG;
        if (!make_grid(d->aabb_min, d->aabb_max, d->occ_res, g)) return KN_E_INVALID_ARG;
        const int64_t v = (int64_t)d->occ_res[0] * d->occ_res[1] * d->occ_res[2];
        if (v > 0x7fffffffLL) return KN_E_UNSUPPORTED;
    }
    return KN_OK;
}

// Bounding box of the occupied skip blocks (distance 0), read back once at scene creation.
static int content_box_from_skip_field(kn_scene *sc, int64_t cells)
{
    std::vector<uint8_t> h((size_t)cells);
    if (hipMemcpy(h.data(), sc->skip_dist, (size_t)cells, hipMemcpyDeviceToHost) != hipSuccess) return KN_E_HIP;
    int lo[3] = {INT32_MAX, INT32_MAX, INT32_MAX}, hi[3] = {-1, -1, -1};
    const int *sr = sc->skip_res;
    for (int x = 0; x < sr[0]; ++x)
        for (int y = 0; y < sr[1]; ++y)
            for (int z = 0; z < sr[2]; ++z)
                if (h[((size_t)x * sr[1] + y) * sr[2] + z] == 0) {
                    const int c[3] = {x, y, z};
                    for (int a = 0; a < 3; ++a) {
                        lo[a] = c[a] < lo[a] ? c[a] : lo[a];
                        hi[a] = c[a] > hi[a] ? c[a] : hi[a];
                    }
                }
    KnGrid &b = sc->content_box;
    b = sc->occ_grid;
    for (int a = 0; a < 3; ++a) {
        if (hi[a] < 0) { // nothing occupied
            b.res[a] = 0;
            continue;
        }
        const int v0 = lo[a] * KN_SKIP_BLOCK;
        int v1 = (hi[a] + 1) * KN_SKIP_BLOCK;
        if (v1 > sc->occ_grid.res[a]) v1 = sc->occ_grid.res[a];
        b.bmin[a] = sc->occ_grid.bmin[a] + sc->occ_grid.cell[a] * (float)v0;
        b.res[a] = v1 - v0;
    }
    return KN_OK;
}

// The scene's device data: one buffer (the caller's or the library's), carved in this order.
struct SceneLayout {
    int64_t cells, words, skip_cells, packed_bytes;
    int32_t n_nets;
    bool has_occ, sparse;
};
static SceneLayout scene_layout(const kn_scene_desc *d)
{
    SceneLayout l{};
    l.cells = (int64_t)d->res[0] * d->res[1] * d->res[2];
    l.sparse = d->cell_net != nullptr;
    l.n_nets = l.sparse ? d->n_nets : (int32_t)l.cells;
    l.has_occ = d->occ_res[0] != 0;
    if (l.has_occ) {
        l.words = kn_div_up((int64_t)d->occ_res[0] * d->occ_res[1] * d->occ_res[2], 32);
        l.skip_cells = 1;
        for (int a = 0; a < 3; ++a) l.skip_cells *= kn_div_up(d->occ_res[a], KN_SKIP_BLOCK);
    }
    l.packed_bytes = d->wdtype == KN_F32 ? kn_mlp_f32_packed_bytes(d->hidden, l.n_nets) : kn_mlp_packed_bytes(d->hidden, l.n_nets);
    return l;
}
struct SceneBufs {
    int32_t *cell_net;
    uint32_t *occ_bits;
    uint8_t *skip_dist, *skip_tmp;
    char *packed_w;
};
static void carve_scene(KnCarver &c, const SceneLayout &l, SceneBufs &b)
{
    b = SceneBufs{};
    if (l.sparse) b.cell_net = c.carve<int32_t>(l.cells);
    if (l.has_occ) {
        b.occ_bits = c.carve<uint32_t>(l.words);
        b.skip_dist = c.carve<uint8_t>(l.skip_cells);
        b.skip_tmp = c.carve<uint8_t>(l.skip_cells); // second buffer of the sweeps (unused afterwards)
    }
    b.packed_w = c.carve<char>(l.packed_bytes);
}

extern "C" int kn_scene_bytes(const kn_scene_desc *desc, int64_t *out_bytes)
{
    if (!out_bytes) return KN_E_INVALID_ARG;
    KN_TRY(validate_desc(desc));
    KnCarver c((void *)256, INT64_MAX / 2);
    SceneBufs b;
    carve_scene(c, scene_layout(desc), b);
    *out_bytes = c.used;
    return KN_OK;
}

extern "C" int kn_scene_create(kn_ctx *ctx, const kn_scene_desc *desc, void *stream, void *buffer, int64_t buffer_bytes,
                               kn_scene **out)
{
    if (!out) return KN_E_INVALID_ARG;
    *out = nullptr;
    if (!ctx) return KN_E_INVALID_ARG;
    KN_TRY(validate_desc(desc));
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return KN_E_NO_DEVICE;
    if (dev != ctx->device) return KN_E_INVALID_ARG; // the context's device must be current
    const SceneLayout lay = scene_layout(desc);
    int64_t need = 0;
    {
        KnCarver c((void *)256, INT64_MAX / 2);
        SceneBufs b;
        carve_scene(c, lay, b);
        need = c.used;
    }
    if (buffer && (((uintptr_t)buffer & 255) || buffer_bytes < need)) return KN_E_WORKSPACE;

    kn_scene *sc = new (std::nothrow) kn_scene();
    if (!sc) return KN_E_INVALID_ARG;
    sc->desc = *desc;
    sc->cells = lay.cells;
    sc->N = lay.n_nets;
    sc->P = kn_params_per_net(desc->hidden, desc->L_pos, desc->L_dir);
    sc->device = dev;
    make_grid(desc->aabb_min, desc->aabb_max, desc->res, sc->net_grid);
    sc->has_occ = lay.has_occ;
    sc->packed_halfs_per_net = 0;
    sc->skip_res[0] = sc->skip_res[1] = sc->skip_res[2] = 0;
    sc->own_buffer = nullptr;
    if (!buffer) {
        if (hipMalloc(&sc->own_buffer, (size_t)need) != hipSuccess) {
            delete sc;
            return KN_E_HIP;
        }
        buffer = sc->own_buffer;
        buffer_bytes = need;
    }
    KnCarver carver(buffer, buffer_bytes);
    SceneBufs bufs;
    carve_scene(carver, lay, bufs);
    sc->cell_net = bufs.cell_net;
    sc->occ_bits = bufs.occ_bits;
    sc->skip_dist = bufs.skip_dist;
    sc->packed_w = bufs.packed_w;
    hipStream_t st = (hipStream_t)stream;
    int rc = carver.ok() ? KN_OK : KN_E_WORKSPACE;
    if (rc == KN_OK && lay.sparse) {
        hipLaunchKernelGGL(k_copy_cell_net, dim3((unsigned)kn_div_up(sc->cells, 256)), dim3(256), 0, st, desc->cell_net,
                           sc->cells, sc->N, sc->cell_net);
        if (hipGetLastError() != hipSuccess) rc = KN_E_HIP;
    }
    if (rc == KN_OK && sc->has_occ) {
        make_grid(desc->aabb_min, desc->aabb_max, desc->occ_res, sc->occ_grid);
        const int64_t vox = (int64_t)desc->occ_res[0] * desc->occ_res[1] * desc->occ_res[2];
        hipLaunchKernelGGL(k_pack_occupancy, dim3((unsigned)kn_div_up(lay.words, 256)), dim3(256), 0, st, desc->occupancy, vox,
                           sc->occ_bits);
        if (hipGetLastError() != hipSuccess) rc = KN_E_HIP;
        if (rc == KN_OK) { // skip field: seed, KN_SKIP_MAX sweeps (ping-pong), cap
            int sr[3];
            for (int a = 0; a < 3; ++a) sr[a] = sc->skip_res[a] = (int)kn_div_up(desc->occ_res[a], KN_SKIP_BLOCK);
            const int64_t cells = lay.skip_cells;
            const dim3 grid((unsigned)kn_div_up(cells, 256)), block(256);
            hipLaunchKernelGGL(k_skip_seed, grid, block, 0, st, desc->occupancy, desc->occ_res[0], desc->occ_res[1],
                               desc->occ_res[2], sr[0], sr[1], sr[2], sc->skip_dist);
            uint8_t *a = sc->skip_dist, *b = bufs.skip_tmp;
            for (int it = 0; it < KN_SKIP_MAX; ++it) { // even count: the result ends in skip_dist
                hipLaunchKernelGGL(k_skip_sweep, grid, block, 0, st, a, sr[0], sr[1], sr[2], b);
                uint8_t *t = a; a = b; b = t;
            }
            hipLaunchKernelGGL(k_skip_cap, grid, block, 0, st, sc->skip_dist, cells);
            if (hipGetLastError() != hipSuccess || hipStreamSynchronize(st) != hipSuccess) rc = KN_E_HIP;
            if (rc == KN_OK) rc = content_box_from_skip_field(sc, cells);
        }
    } else if (rc == KN_OK) {
        sc->occ_grid = sc->net_grid;
        sc->content_box = sc->net_grid;
    }
    if (rc == KN_OK) rc = desc->wdtype == KN_F32 ? kn_mlp_f32_pack_weights(sc, st) : kn_mlp_pack_weights(sc, st);
    // the descriptor's buffers may go once the call returns
    if (rc == KN_OK && hipStreamSynchronize(st) != hipSuccess) rc = KN_E_HIP;
    if (rc != KN_OK) {
        kn_scene_destroy(sc);
        return rc;
    }
    sc->desc.weights = nullptr; // not the scene's to keep
    sc->desc.occupancy = nullptr;
    sc->desc.cell_net = nullptr;
    *out = sc;
    return KN_OK;
}

extern "C" int kn_scene_destroy(kn_scene *sc)
{
    if (!sc) return KN_OK;
    (void)hipDeviceSynchronize();
    if (sc->own_buffer) (void)hipFree(sc->own_buffer);
    delete sc;
    return KN_OK;
}

int kn_mlp_tile_len(const kn_scene *sc) { return sc->desc.wdtype == KN_F32 ? kn_mlp_f32_tile_len(sc) : kn_mlp_mfma_tile_len(sc); }

int kn_mlp_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t M, float *sigma,
                  float *rgb, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (M <= 0) return KN_OK;
    const int64_t max_tiles = kn_max_tiles(M, sc->N, kn_mlp_tile_len(sc));
    if (sc->desc.wdtype == KN_F32) return kn_mlp_f32_launch(sc, st, src, b, max_tiles, sigma, rgb, ev_start, ev_stop);
    return kn_mlp_mfma_launch(sc, st, src, b, max_tiles, sigma, rgb, ev_start, ev_stop);
}

// workspace of an evaluation that sorts indices (layer-at-a-time path, static scratch entry point) ...
static int64_t index_ws_bytes(const kn_scene *sc, int64_t M)
{
    return kn_align_up((M > 0 ? M : 1) * 4, 256) + kn_bucket_ws_bytes(M, sc->N);
}
// ... and of kn_eval_grouped, which moves the samples themselves
static int64_t eval_ws_bytes(const kn_scene *sc, int64_t M)
{
    const int64_t a = index_ws_bytes(sc, M), b = kn_reorder_ws_bytes(M, sc->N);
    return a > b ? a : b;
}

extern "C" int kn_workspace_bytes(const kn_ctx *ctx, const kn_scene *sc, int64_t max_points, int64_t max_rays,
                                  int64_t *out_bytes)
{
    if (!ctx || !sc || !out_bytes || max_points < 0 || max_rays < 0) return KN_E_INVALID_ARG;
    if (max_points > (1ll << 30) || max_rays > (1ll << 30)) return KN_E_UNSUPPORTED;
    int64_t a = max_points > 0 ? eval_ws_bytes(sc, max_points) : 0;
    int64_t b = max_rays > 0 ? kn_render_ws_bytes(sc, max_rays, kn_knobs(ctx).slots_per_ray) : 0;
    *out_bytes = (a > b ? a : b) + 256;
    return KN_OK;
}

// `timed`: stage events may be recorded (creating the events allocates; the static entry point never does)
static int eval_grouped_impl(kn_ctx *ctx, const kn_scene *sc, hipStream_t st, const float *points, const float *dirs, int64_t M,
                             float *sigma, float *rgb, int32_t *cell_id, int32_t *counts, int32_t *perm, void *workspace,
                             int64_t workspace_bytes, bool timed, bool reorder)
{
    KnCarver ws(workspace, workspace_bytes);
    KnStageTimer tm(ctx, st, timed);
    if (reorder && M > 0) {
        // the samples themselves are brought into grouped order (Sec. 3.5); the kernel reads them contiguously
        tm.begin();
        KnBucketOut bo;
        const uint32_t *records[2] = {nullptr, nullptr};
        float *out4 = nullptr;
        KN_TRY(kn_reorder_run(sc, st, points, dirs, M, kn_mlp_tile_len(sc), cell_id, counts, perm, ws, &bo, records, &out4, &tm));
        tm.mark(KN_ST_BUCKET);
        KnSampleSrc src{};
        src.records = records[0];
        src.records_dir = records[1];
        src.out4 = out4;
        hipEvent_t e0 = nullptr, e1 = nullptr;
        (void)tm.kernel_events(KN_ST_MLP, &e0, &e1);
        KN_TRY(kn_mlp_launch(sc, st, src, bo, M, sigma, rgb, e0, e1));
        tm.mark(KN_ST_MLP);
        KN_TRY(kn_reorder_split_results(st, out4, M, sigma, rgb));
        tm.mark(KN_ST_BUCKET); // the way back to the caller's order is charged to the re-ordering
        tm.add(1, M, M, 1);
        return KN_OK;
    }
    int32_t *keys = ws.carve<int32_t>(M);
    if (!ws.ok()) return KN_E_WORKSPACE;
    tm.begin();
    KN_TRY(kn_cell_keys(sc, st, points, M, cell_id, keys));
    tm.mark(KN_ST_CELL);
    KnBucketOut bo;
    KN_TRY(kn_bucket_run(st, keys, M, sc->N, kn_mlp_tile_len(sc), counts, nullptr, perm, ws, &bo));
    if (M == 0) return KN_OK;
    tm.mark(KN_ST_BUCKET);
    KnSampleSrc src{};
    src.points = points;
    src.dirs = dirs;
    src.out4 = nullptr;
    KN_TRY(kn_mlp_launch(sc, st, src, bo, M, sigma, rgb));
    hipLaunchKernelGGL(k_zero_outside, dim3((unsigned)kn_div_up(M, 256)), dim3(256), 0, st, bo.perm, bo.offsets, sc->N, M, sigma,
                       rgb);
    KN_CHECK_LAUNCH();
    tm.mark(KN_ST_MLP);
    tm.add(1, M, M, 1); // (M includes points outside the AABB: they cost no MLP work)
    return KN_OK;
}

extern "C" int kn_eval_grouped(kn_ctx *ctx, const kn_scene *sc, void *stream, const float *points, const float *dirs, int64_t M,
                               float *sigma, float *rgb, int32_t *cell_id, int32_t *counts, int32_t *perm, void *workspace,
                               int64_t workspace_bytes)
{
    if (!ctx || !sc || M < 0 || (M > 0 && (!points || !dirs || !sigma || !rgb))) return KN_E_INVALID_ARG;
    if (M > (1ll << 30)) return KN_E_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < eval_ws_bytes(sc, M)) return KN_E_WORKSPACE;
    return eval_grouped_impl(ctx, sc, (hipStream_t)stream, points, dirs, M, sigma, rgb, cell_id, counts, perm, workspace,
                             workspace_bytes, true, true);
}

// kn_eval_grouped on the library's static scratch array instead of a caller workspace: nothing is allocated, here
// or in anything this calls (no stage events either).  All calls on one GPU share the array.
extern "C" int kn_eval_grouped_static(kn_ctx *ctx, const kn_scene *sc, void *stream, const float *points, const float *dirs,
                                      int64_t M, float *sigma, float *rgb, int32_t *cell_id, int32_t *counts, int32_t *perm)
{
    if (!ctx || !sc || M < 0 || (M > 0 && (!points || !dirs || !sigma || !rgb))) return KN_E_INVALID_ARG;
    if (M > (1ll << 30) || index_ws_bytes(sc, M) > (int64_t)KN_STATIC_SCRATCH_BYTES) return KN_E_STATIC_LIMIT;
    int dev = -1;
    KN_HIP(hipGetDevice(&dev));
    if (dev != ctx->device || dev != sc->device) return KN_E_INVALID_ARG; // the context's device must be current
    void *ptr = ctx->static_scratch; // this device's copy of the array, looked up by kn_create
    if (!ptr) return KN_E_HIP;
    // (indices are sorted, not the samples: the batches that fit the array are small, and so is the workspace then)
    return eval_grouped_impl(ctx, sc, (hipStream_t)stream, points, dirs, M, sigma, rgb, cell_id, counts, perm, ptr,
                             (int64_t)KN_STATIC_SCRATCH_BYTES, false, false);
}

// ---------------------------------------------------------------------------------------------
// Layer-at-a-time evaluation (the comparison point for the fused kernel)
extern "C" int kn_layered_workspace_bytes(const kn_scene *sc, int64_t max_points, int64_t *out_bytes)
{
    if (!sc || !out_bytes || max_points < 0) return KN_E_INVALID_ARG;
    if (max_points > (1ll << 30)) return KN_E_UNSUPPORTED;
    *out_bytes = index_ws_bytes(sc, max_points) + kn_layered_act_bytes(sc, max_points) + 512;
    return KN_OK;
}

extern "C" int kn_eval_grouped_layered(kn_ctx *ctx, const kn_scene *sc, void *stream, const float *points, const float *dirs,
                                       int64_t M, float *sigma, float *rgb, void *workspace, int64_t workspace_bytes)
{
    if (!ctx || !sc || M < 0 || (M > 0 && (!points || !dirs || !sigma || !rgb))) return KN_E_INVALID_ARG;
    if (M > (1ll << 30) || sc->desc.wdtype == KN_F32) return KN_E_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) ||
        workspace_bytes < index_ws_bytes(sc, M) + kn_layered_act_bytes(sc, M) + 256)
        return KN_E_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    KnCarver ws(workspace, workspace_bytes);
    void *acts = ws.carve<char>(kn_layered_act_bytes(sc, M));
    int32_t *keys = ws.carve<int32_t>(M);
    if (!ws.ok()) return KN_E_WORKSPACE;
    KnStageTimer tm(ctx, st);
    tm.begin();
    KN_TRY(kn_cell_keys(sc, st, points, M, nullptr, keys));
    tm.mark(KN_ST_CELL);
    KnBucketOut bo;
    const int tile_len = kn_mlp_tile_len(sc);
    KN_TRY(kn_bucket_run(st, keys, M, sc->N, tile_len, nullptr, nullptr, nullptr, ws, &bo));
    if (M == 0) return KN_OK;
    tm.mark(KN_ST_BUCKET);
    KnSampleSrc src{};
    src.points = points;
    src.dirs = dirs;
    KN_TRY(kn_mlp_layered_launch(sc, st, src, bo, M, kn_max_tiles(M, sc->N, tile_len), acts, sigma, rgb));
    hipLaunchKernelGGL(k_zero_outside, dim3((unsigned)kn_div_up(M, 256)), dim3(256), 0, st, bo.perm, bo.offsets, sc->N, M, sigma,
                       rgb);
    KN_CHECK_LAUNCH();
    tm.mark(KN_ST_MLP);
    tm.add(6, M, M, 1);
    return KN_OK;
}

// ---------------------------------------------------------------------------------------------
// Occupancy grid extraction (Sec. 3.4)
namespace {

__global__ void k_zero_bytes(uint8_t *p, int64_t n)
{
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 16;
    if (i + 16 <= n && ((uintptr_t)(p + i) & 15) == 0) {
        *(uint4 *)(p + i) = make_uint4(0u, 0u, 0u, 0u);
    } else {
        for (int64_t j = i; j < n && j < i + 16; ++j) p[j] = 0;
    }
}

// first[c] = first voxel along axis blockIdx.x whose centre lies in network cell c or beyond (res + 1 entries):
// the voxels whose centre lies in cell c are first[c] .. first[c+1]-1.
__global__ void k_probe_ranges(KnGrid occ, KnGrid net, int32_t *first0, int32_t *first1, int32_t *first2)
{
    const int a = blockIdx.x;
    int32_t *first = a == 0 ? first0 : (a == 1 ? first1 : first2);
    const int nc = net.res[a], nv = occ.res[a];
    for (int c = threadIdx.x; c <= nc; c += blockDim.x) first[c] = nv;
    __syncthreads();
    auto home = [&](int v) {
        const float x = fmaf((float)v + 0.5f, occ.cell[a], occ.bmin[a]);
        const float f = floorf((x - net.bmin[a]) / net.cell[a]);
        return (int)fminf(fmaxf(f, 0.0f), (float)(nc - 1));
    };
    for (int v = threadIdx.x; v < nv; v += blockDim.x) {
        const int h = home(v), before = v == 0 ? -1 : home(v - 1); // non-decreasing in v
        for (int c = before + 1; c <= h; ++c) first[c] = v;
    }
}

int64_t extract_ws_bytes(const kn_scene *sc)
{
    int64_t b = 0;
    for (int a = 0; a < 3; ++a) b += kn_align_up(((int64_t)sc->desc.res[a] + 1) * 4, 256);
    return b;
}

} // namespace

extern "C" int kn_extract_workspace_bytes(const kn_scene *sc, int64_t *out_bytes)
{
    if (!sc || !out_bytes) return KN_E_INVALID_ARG;
    *out_bytes = extract_ws_bytes(sc) + 256;
    return KN_OK;
}

extern "C" int kn_extract_occupancy(kn_ctx *ctx, const kn_scene *sc, void *stream, const int32_t occ_res[3], float tau,
                                    uint8_t *occupancy, void *workspace, int64_t workspace_bytes)
{
    if (!ctx || !sc || !occ_res || !occupancy || tau != tau) return KN_E_INVALID_ARG;
    KnProbeJob job{};
    if (!make_grid(sc->desc.aabb_min, sc->desc.aabb_max, occ_res, job.occ)) return KN_E_INVALID_ARG;
    const int64_t voxels = (int64_t)occ_res[0] * occ_res[1] * occ_res[2];
    if (voxels > 0x7fffffffLL) return KN_E_UNSUPPORTED;
    // upper bound of the voxels one network cell can own, and the nominal number of tiles per cell
    int64_t box = 1;
    for (int a = 0; a < 3; ++a) box *= kn_div_up(occ_res[a], sc->desc.res[a]) + 1;
    if (box > KN_PROBE_MAX_BOX) return KN_E_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < extract_ws_bytes(sc)) return KN_E_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    KnCarver ws(workspace, workspace_bytes);
    int32_t *first[3];
    for (int a = 0; a < 3; ++a) first[a] = ws.carve<int32_t>(sc->desc.res[a] + 1);
    if (!ws.ok()) return KN_E_WORKSPACE;
    job.net = sc->net_grid;
    job.cell_net = sc->cell_net;
    for (int a = 0; a < 3; ++a) job.first[a] = first[a];
    job.tau = tau;
    job.occupancy = occupancy;
    // Where the grid being filled refines the network grid, a probe lies at least a sixth of a voxel from the faces of
    // its voxel's home cell; if that is far more than the rounding of its position and of Eq. 6 can amount to (a few
    // units in the last place of the largest coordinate), Eq. 6 gives the home cell for every probe and is skipped.
    job.nested = 1;
    for (int a = 0; a < 3; ++a) {
        const float reach = fabsf(sc->desc.aabb_min[a]) + fabsf(sc->desc.aabb_max[a]) + (sc->desc.aabb_max[a] - sc->desc.aabb_min[a]);
        if (occ_res[a] % sc->desc.res[a] != 0 || !(job.occ.cell[a] > 48.0f * 2.4e-7f * reach)) job.nested = 0;
    }
    // enough workgroups to fill the chip several times over, but at least some tens of tiles per wavefront
    const int64_t tiles_per_cell = kn_div_up(KN_PROBES * kn_div_up(voxels, sc->cells), KN_WAVE);
    int64_t parts = kn_div_up(2048, sc->cells);
    if (parts > tiles_per_cell / 32) parts = tiles_per_cell / 32;
    if (parts < 1) parts = 1;
    job.parts = (int32_t)parts;

    KnStageTimer tm(ctx, st);
    tm.begin();
    hipLaunchKernelGGL(k_zero_bytes, dim3((unsigned)kn_div_up(kn_div_up(voxels, 16), 256)), dim3(256), 0, st, occupancy, voxels);
    KN_CHECK_LAUNCH();
    hipLaunchKernelGGL(k_probe_ranges, dim3(3), dim3(256), 0, st, job.occ, job.net, first[0], first[1], first[2]);
    KN_CHECK_LAUNCH();
    tm.mark(KN_ST_SETUP);
    if (sc->desc.wdtype == KN_F32)
        KN_TRY(kn_probe_f32_launch(sc, st, job));
    else
        KN_TRY(kn_probe_mfma_launch(sc, st, job));
    tm.mark(KN_ST_MLP);
    tm.add(1, KN_PROBES * voxels, 0, 1);
    return KN_OK;
}
