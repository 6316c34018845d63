// Host side of the C ABI: scene objects, validation, workspace sizing, kn_eval_grouped.
#include "kn_common.h"
#include "kn_probe.h"

#include <math.h>
#include <new>
#include <string.h>
#include <vector>

thread_local int g_kn_last_hip_error = 0;

int kn_cell_keys(const kn_scene *sc, hipStream_t st, const float *points, int64_t M, int32_t *ids, int32_t *keys,
                 int32_t *zero, int64_t n_zero);
int64_t kn_render_ws_bytes(const kn_scene *sc, int64_t R);
int kn_mlp_f32_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t max_tiles,
                      float *sigma, float *rgb);
int kn_mlp_mfma_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t max_tiles,
                       float *sigma, float *rgb);
int kn_mlp_mfma_tile_len(const kn_scene *sc);
int kn_mlp_f32_tile_len(const kn_scene *sc);
int kn_mlp_f32_pack_weights(kn_scene *sc, hipStream_t st);
int kn_probe_mfma_launch(const kn_scene *sc, hipStream_t st, const KnProbeJob &job);
int kn_probe_f32_launch(const kn_scene *sc, hipStream_t st, const KnProbeJob &job);
int64_t kn_layered_act_bytes(const kn_scene *sc, int64_t M);
int kn_mlp_layered_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t M,
                          int64_t max_tiles, void *acts, float *sigma, float *rgb);

kn_profile g_kn_profile = {};
bool g_kn_profile_on = false;
int g_only_stage = KN_ST_NONE; // != NONE: only this stage's intervals are recorded (and no sample counts)
// Event ring shared by all calls: intervals are settled (one stream synchronise, then
// hipEventElapsedTime for each recorded interval) only when the ring is full, when another stream
// starts recording, or when the totals are read.
constexpr int KN_N_EVENTS = 1024;
static hipEvent_t g_events[KN_N_EVENTS];
static int g_event_stage[KN_N_EVENTS];
static int g_n_events = 0;
static hipStream_t g_event_stream = nullptr;
static bool g_events_ready = false;

// Scratch memory of kn_eval_grouped_static, the entry point for callers that cannot allocate: a file-scope device
// array that every GPU the library runs on holds until the process ends.  In host code the array's name is only a
// stand-in for the symbol, not a device address; the address on a device comes from hipGetSymbolAddress with that
// device current (static_scratch_init, called by kn_scene_create), and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[KN_STATIC_SCRATCH_BYTES];
constexpr int KN_MAX_DEVICES = 64;
static void *g_scratch_ptr[KN_MAX_DEVICES] = {};
static std::mutex g_scratch_mutex;

// once per device, with that device current
static int static_scratch_init(int dev)
{
    if (dev < 0 || dev >= KN_MAX_DEVICES) return KN_E_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev]) return KN_OK;
    void *ptr = nullptr;
    KN_HIP(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || ((uintptr_t)ptr & 255)) return KN_E_HIP;
    g_scratch_ptr[dev] = ptr;
    return KN_OK;
}

static int settle_events()
{
    if (g_n_events >= 2) {
        KN_HIP(hipStreamSynchronize(g_event_stream));
        for (int i = 1; i < g_n_events; ++i) {
            float ms = 0.0f;
            if (g_event_stage[i] == KN_ST_NONE || hipEventElapsedTime(&ms, g_events[i - 1], g_events[i]) != hipSuccess)
                continue;
            switch (g_event_stage[i]) {
            case KN_ST_CELL: g_kn_profile.ms_cell += ms; break;
            case KN_ST_MARCH: g_kn_profile.ms_march += ms; break;
            case KN_ST_BUCKET: g_kn_profile.ms_bucket += ms; break;
            case KN_ST_MLP: g_kn_profile.ms_mlp += ms; break;
            case KN_ST_BLEND: g_kn_profile.ms_blend += ms; break;
            case KN_ST_SETUP: g_kn_profile.ms_setup += ms; break;
            default: break;
            }
        }
    }
    g_n_events = 0;
    return KN_OK;
}

KnStageTimer::KnStageTimer(hipStream_t s, bool allowed) : st(s), on(allowed && g_kn_profile_on)
{
    if (on && !g_events_ready) {
        for (auto &e : g_events)
            if (hipEventCreate(&e) != hipSuccess) on = false;
        g_events_ready = on;
    }
    if (on && g_n_events > 0 && g_event_stream != s) (void)settle_events();
    g_event_stream = s;
}
void KnStageTimer::mark(int stage_id)
{
    if (!on) return;
    if (g_only_stage != KN_ST_NONE) {
        // the mark before the stage of interest opens its interval; everything else is dropped
        const bool opens = g_only_stage == KN_ST_MLP ? stage_id == KN_ST_BUCKET
                                                     : (stage_id == KN_ST_NONE || stage_id == KN_ST_SETUP);
        const bool closes = stage_id == g_only_stage;
        if (!opens && !closes) return;
        if (opens) stage_id = KN_ST_NONE;
    }
    if (g_n_events == KN_N_EVENTS) {
        (void)settle_events();
        if (stage_id != KN_ST_NONE) { // re-open the interval that the settle cut short
            g_event_stage[0] = KN_ST_NONE;
            (void)hipEventRecord(g_events[0], st);
            g_n_events = 1;
        }
    }
    g_event_stage[g_n_events] = stage_id;
    (void)hipEventRecord(g_events[g_n_events++], st);
}

extern "C" int kn_profile_enable(int on)
{
    if (g_kn_profile_on) (void)settle_events();
    g_kn_profile_on = on != 0;
    g_only_stage = on == 2 ? KN_ST_MLP : on == 3 ? KN_ST_MARCH : KN_ST_NONE;
    return KN_OK;
}

extern "C" int kn_profile_read(kn_profile *out, int reset)
{
    if (!out) return KN_E_INVALID_ARG;
    KN_TRY(settle_events());
    *out = g_kn_profile;
    if (reset) g_kn_profile = kn_profile{};
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

extern "C" int kn_scene_create(const kn_scene_desc *desc, void *stream, kn_scene **out)
{
    if (!out) return KN_E_INVALID_ARG;
    *out = nullptr;
    KN_TRY(validate_desc(desc));
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return KN_E_NO_DEVICE;
    hipDeviceProp_t prop;
    KN_HIP(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return KN_E_NO_DEVICE;
    KN_TRY(static_scratch_init(dev));

    kn_scene *sc = new (std::nothrow) kn_scene();
    if (!sc) return KN_E_INVALID_ARG;
    sc->desc = *desc;
    sc->cells = (int64_t)desc->res[0] * desc->res[1] * desc->res[2];
    sc->N = desc->cell_net ? desc->n_nets : (int32_t)sc->cells;
    sc->cell_net = nullptr;
    sc->P = kn_params_per_net(desc->hidden, desc->L_pos, desc->L_dir);
    sc->device = dev;
    make_grid(desc->aabb_min, desc->aabb_max, desc->res, sc->net_grid);
    sc->has_occ = desc->occ_res[0] != 0;
    sc->occ_bits = nullptr;
    sc->packed_w = nullptr;
    sc->packed_halfs_per_net = 0;
    sc->skip_dist = nullptr;
    sc->skip_res[0] = sc->skip_res[1] = sc->skip_res[2] = 0;
    for (auto &m : sc->mailbox) m = KnMailbox{nullptr, nullptr, 0ull, nullptr, false};
    {
        void *hp = nullptr, *dp = nullptr;
        if (hipHostMalloc(&hp, 64 * KN_MAILBOXES, hipHostMallocMapped) == hipSuccess &&
            hipHostGetDevicePointer(&dp, hp, 0) == hipSuccess) {
            memset(hp, 0, 64 * KN_MAILBOXES);
            for (int i = 0; i < KN_MAILBOXES; ++i) {
                sc->mailbox[i].host = (volatile unsigned long long *)((char *)hp + 64 * i);
                sc->mailbox[i].dev = (unsigned long long *)((char *)dp + 64 * i);
            }
        } else if (hp) {
            (void)hipHostFree(hp);
        }
    }
    hipStream_t st = (hipStream_t)stream;
    int rc = KN_OK;
    if (desc->cell_net) {
        if (hipMalloc((void **)&sc->cell_net, (size_t)sc->cells * 4) != hipSuccess) {
            rc = KN_E_HIP;
        } else {
            hipLaunchKernelGGL(k_copy_cell_net, dim3((unsigned)kn_div_up(sc->cells, 256)), dim3(256), 0, st, desc->cell_net,
                               sc->cells, sc->N, sc->cell_net);
            if (hipGetLastError() != hipSuccess) rc = KN_E_HIP;
        }
    }
    if (rc != KN_OK) {
        // (the clean-up below)
    } else if (sc->has_occ) {
        make_grid(desc->aabb_min, desc->aabb_max, desc->occ_res, sc->occ_grid);
        const int64_t vox = (int64_t)desc->occ_res[0] * desc->occ_res[1] * desc->occ_res[2];
        const int64_t words = kn_div_up(vox, 32);
        if (hipMalloc((void **)&sc->occ_bits, (size_t)words * 4) != hipSuccess) {
            rc = KN_E_HIP;
        } else {
            hipLaunchKernelGGL(k_pack_occupancy, dim3((unsigned)kn_div_up(words, 256)), dim3(256), 0, st, desc->occupancy, vox,
                               sc->occ_bits);
            if (hipGetLastError() != hipSuccess) rc = KN_E_HIP;
        }
        if (rc == KN_OK) { // skip field: seed, KN_SKIP_MAX sweeps (ping-pong), cap
            int sr[3];
            for (int a = 0; a < 3; ++a) sr[a] = sc->skip_res[a] = (int)kn_div_up(desc->occ_res[a], KN_SKIP_BLOCK);
            const int64_t cells = (int64_t)sr[0] * sr[1] * sr[2];
            uint8_t *tmp = nullptr;
            if (hipMalloc((void **)&sc->skip_dist, (size_t)cells) != hipSuccess ||
                hipMalloc((void **)&tmp, (size_t)cells) != hipSuccess) {
                rc = KN_E_HIP;
            } else {
                const dim3 grid((unsigned)kn_div_up(cells, 256)), block(256);
                hipLaunchKernelGGL(k_skip_seed, grid, block, 0, st, desc->occupancy, desc->occ_res[0], desc->occ_res[1],
                                   desc->occ_res[2], sr[0], sr[1], sr[2], sc->skip_dist);
                uint8_t *a = sc->skip_dist, *b = tmp;
                for (int it = 0; it < KN_SKIP_MAX; ++it) { // even count: the result ends in skip_dist
                    hipLaunchKernelGGL(k_skip_sweep, grid, block, 0, st, a, sr[0], sr[1], sr[2], b);
                    uint8_t *t = a; a = b; b = t;
                }
                hipLaunchKernelGGL(k_skip_cap, grid, block, 0, st, sc->skip_dist, cells);
                if (hipGetLastError() != hipSuccess || hipStreamSynchronize(st) != hipSuccess) rc = KN_E_HIP;
                if (rc == KN_OK) rc = content_box_from_skip_field(sc, cells);
            }
            if (tmp) (void)hipFree(tmp);
        }
    } else {
        sc->occ_grid = sc->net_grid;
        sc->content_box = sc->net_grid;
    }
    if (rc == KN_OK) rc = desc->wdtype == KN_F32 ? kn_mlp_f32_pack_weights(sc, st) : kn_mlp_pack_weights(sc, st);
    if (rc != KN_OK) {
        kn_scene_destroy(sc);
        return rc;
    }
    *out = sc;
    return KN_OK;
}

extern "C" int kn_scene_destroy(kn_scene *sc)
{
    if (!sc) return KN_OK;
    (void)hipDeviceSynchronize();
    if (sc->occ_bits) (void)hipFree(sc->occ_bits);
    if (sc->packed_w) (void)hipFree(sc->packed_w);
    if (sc->skip_dist) (void)hipFree(sc->skip_dist);
    if (sc->cell_net) (void)hipFree(sc->cell_net);
    if (sc->mailbox[0].host) (void)hipHostFree((void *)sc->mailbox[0].host);
    delete sc;
    return KN_OK;
}

int kn_mlp_tile_len(const kn_scene *sc) { return sc->desc.wdtype == KN_F32 ? kn_mlp_f32_tile_len(sc) : kn_mlp_mfma_tile_len(sc); }

int kn_mlp_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t M, float *sigma,
                  float *rgb)
{
    if (M <= 0) return KN_OK;
    const int64_t max_tiles = kn_max_tiles(M, sc->N, kn_mlp_tile_len(sc));
    if (sc->desc.wdtype == KN_F32) return kn_mlp_f32_launch(sc, st, src, b, max_tiles, sigma, rgb);
    return kn_mlp_mfma_launch(sc, st, src, b, max_tiles, sigma, rgb);
}

static int64_t eval_ws_bytes(const kn_scene *sc, int64_t M)
{
    return kn_align_up((M > 0 ? M : 1) * 4, 256) + kn_bucket_ws_bytes(M, sc->N);
}

extern "C" int kn_workspace_bytes(const kn_scene *sc, int64_t max_points, int64_t max_rays, int64_t *out_bytes)
{
    if (!sc || !out_bytes || max_points < 0 || max_rays < 0) return KN_E_INVALID_ARG;
    if (max_points > (1ll << 30) || max_rays > (1ll << 30)) return KN_E_UNSUPPORTED;
    int64_t a = max_points > 0 ? eval_ws_bytes(sc, max_points) : 0;
    int64_t b = max_rays > 0 ? kn_render_ws_bytes(sc, max_rays) : 0;
    *out_bytes = (a > b ? a : b) + 256;
    return KN_OK;
}

// `timed`: stage events may be recorded (creating the events allocates; the static entry point never does)
static int eval_grouped_impl(const kn_scene *sc, hipStream_t st, const float *points, const float *dirs, int64_t M,
                             float *sigma, float *rgb, int32_t *cell_id, int32_t *counts, int32_t *perm, void *workspace,
                             int64_t workspace_bytes, bool timed)
{
    KnCarver ws(workspace, workspace_bytes);
    int32_t *keys = ws.carve<int32_t>(M);
    if (!ws.ok()) return KN_E_WORKSPACE;
    KnStageTimer tm(st, timed);
    tm.begin();
    int32_t *scratch = nullptr;
    int64_t n_scratch = 0;
    kn_bucket_scratch(ws, M, sc->N, &scratch, &n_scratch);
    KN_TRY(kn_cell_keys(sc, st, points, M, cell_id, keys, scratch, scratch ? n_scratch : 0));
    tm.mark(KN_ST_CELL);
    KnBucketOut bo;
    KN_TRY(kn_bucket_run(st, keys, M, nullptr, sc->N, kn_mlp_tile_len(sc), counts, nullptr, perm, ws, &bo, scratch != nullptr));
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
    if (tm.on) {
        g_kn_profile.mlp_launches += 1;
        g_kn_profile.mlp_samples += M; // includes points outside the AABB (they cost no MLP work)
        g_kn_profile.bucket_keys += M;
        g_kn_profile.calls += 1;
    }
    return KN_OK;
}

extern "C" int kn_eval_grouped(const kn_scene *sc, void *stream, const float *points, const float *dirs, int64_t M,
                               float *sigma, float *rgb, int32_t *cell_id, int32_t *counts, int32_t *perm, void *workspace,
                               int64_t workspace_bytes)
{
    if (!sc || M < 0 || (M > 0 && (!points || !dirs || !sigma || !rgb))) return KN_E_INVALID_ARG;
    if (M > (1ll << 30)) return KN_E_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < eval_ws_bytes(sc, M)) return KN_E_WORKSPACE;
    return eval_grouped_impl(sc, (hipStream_t)stream, points, dirs, M, sigma, rgb, cell_id, counts, perm, workspace,
                             workspace_bytes, true);
}

// kn_eval_grouped on the library's static scratch array instead of a caller workspace: nothing is allocated, here
// or in anything this calls (no stage events either).  All calls on one GPU share the array.
extern "C" int kn_eval_grouped_static(const kn_scene *sc, void *stream, const float *points, const float *dirs, int64_t M,
                                      float *sigma, float *rgb, int32_t *cell_id, int32_t *counts, int32_t *perm)
{
    if (!sc || M < 0 || (M > 0 && (!points || !dirs || !sigma || !rgb))) return KN_E_INVALID_ARG;
    if (M > (1ll << 30) || eval_ws_bytes(sc, M) > (int64_t)KN_STATIC_SCRATCH_BYTES) return KN_E_STATIC_LIMIT;
    int dev = -1;
    KN_HIP(hipGetDevice(&dev));
    if (dev != sc->device || dev < 0 || dev >= KN_MAX_DEVICES) return KN_E_INVALID_ARG; // the scene's device must be current
    void *ptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        ptr = g_scratch_ptr[dev]; // set when the scene was created on this device
    }
    if (!ptr) return KN_E_HIP;
    return eval_grouped_impl(sc, (hipStream_t)stream, points, dirs, M, sigma, rgb, cell_id, counts, perm, ptr,
                             (int64_t)KN_STATIC_SCRATCH_BYTES, false);
}

// ---------------------------------------------------------------------------------------------
// Layer-at-a-time evaluation (the comparison point for the fused kernel)
extern "C" int kn_layered_workspace_bytes(const kn_scene *sc, int64_t max_points, int64_t *out_bytes)
{
    if (!sc || !out_bytes || max_points < 0) return KN_E_INVALID_ARG;
    if (max_points > (1ll << 30)) return KN_E_UNSUPPORTED;
    *out_bytes = eval_ws_bytes(sc, max_points) + kn_layered_act_bytes(sc, max_points) + 512;
    return KN_OK;
}

extern "C" int kn_eval_grouped_layered(const kn_scene *sc, void *stream, const float *points, const float *dirs, int64_t M,
                                       float *sigma, float *rgb, void *workspace, int64_t workspace_bytes)
{
    if (!sc || M < 0 || (M > 0 && (!points || !dirs || !sigma || !rgb))) return KN_E_INVALID_ARG;
    if (M > (1ll << 30) || sc->desc.wdtype == KN_F32) return KN_E_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) ||
        workspace_bytes < eval_ws_bytes(sc, M) + kn_layered_act_bytes(sc, M) + 256)
        return KN_E_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    KnCarver ws(workspace, workspace_bytes);
    void *acts = ws.carve<char>(kn_layered_act_bytes(sc, M));
    int32_t *keys = ws.carve<int32_t>(M);
    if (!ws.ok()) return KN_E_WORKSPACE;
    KnStageTimer tm(st);
    tm.begin();
    int32_t *scratch = nullptr;
    int64_t n_scratch = 0;
    kn_bucket_scratch(ws, M, sc->N, &scratch, &n_scratch);
    KN_TRY(kn_cell_keys(sc, st, points, M, nullptr, keys, scratch, scratch ? n_scratch : 0));
    tm.mark(KN_ST_CELL);
    KnBucketOut bo;
    const int tile_len = kn_mlp_tile_len(sc);
    KN_TRY(kn_bucket_run(st, keys, M, nullptr, sc->N, tile_len, nullptr, nullptr, nullptr, ws, &bo, scratch != nullptr));
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
    if (tm.on) {
        g_kn_profile.mlp_launches += 6;
        g_kn_profile.mlp_samples += M;
        g_kn_profile.bucket_keys += M;
        g_kn_profile.calls += 1;
    }
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

extern "C" int kn_extract_occupancy(const kn_scene *sc, void *stream, const int32_t occ_res[3], float tau,
                                    uint8_t *occupancy, void *workspace, int64_t workspace_bytes)
{
    if (!sc || !occ_res || !occupancy || tau != tau) return KN_E_INVALID_ARG;
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

    KnStageTimer tm(st);
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
    if (tm.on) {
        g_kn_profile.mlp_launches += 1;
        g_kn_profile.mlp_samples += KN_PROBES * voxels;
        g_kn_profile.calls += 1;
    }
    return KN_OK;
}
