// Point -> cell assignment (Eq. 6) and the stage entry points kn_cell_ids and kn_bucket (Sec. 3.5: inputs are ordered so
// that consecutive inputs belong to the same network).  The sort itself is in kn_reorder.hip.
#include "kn_common.h"

namespace {

// ---------------------------------------------------------------------------------------------
__global__ void k_fill_i32(int32_t *p, int64_t n, int32_t v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void k_cell_ids(const float *__restrict__ pts, int64_t M, KnGrid g, const int32_t *__restrict__ cell_net,
                           int32_t *__restrict__ ids, int32_t *__restrict__ keys, int32_t N)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    float x = pts[3 * i], y = pts[3 * i + 1], z = pts[3 * i + 2];
    int32_t id = kn_net_of_cell(cell_net, kn_grid_index(g, x, y, z)); // Eq. 6, then the table of a sparse grid
    if (ids) ids[i] = id;
    if (keys) keys[i] = id < 0 ? N : id;
}

__global__ void k_ids_to_keys(const int32_t *__restrict__ ids, int64_t M, int32_t N, int32_t *__restrict__ keys)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    int32_t id = ids[i];
    keys[i] = (id < 0 || id > N) ? N : id;
}

int launch_1d(int64_t n, int threads, dim3 &grid)
{
    int64_t blocks = kn_div_up(n, threads);
    if (blocks > 0x7fffffffLL) return KN_E_UNSUPPORTED;
    grid = dim3((unsigned)blocks);
    return KN_OK;
}

} // namespace

// ---------------------------------------------------------------------------------------------
int kn_fill_i32(hipStream_t st, int32_t *p, int64_t n, int32_t v)
{
    if (n <= 0) return KN_OK;
    dim3 grid;
    KN_TRY(launch_1d(n, 256, grid));
    hipLaunchKernelGGL(k_fill_i32, grid, dim3(256), 0, st, p, n, v);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

int64_t kn_max_tiles(int64_t M, int32_t N, int32_t tile_len)
{
    return M / tile_len + (M < N ? M : N) + 1;
}


// ---------------------------------------------------------------------------------------------
// C ABI: stage entry points of this file
extern "C" int kn_cell_ids(const kn_scene *sc, void *stream, const float *points, int64_t M, int32_t *ids)
{
    if (!sc || M < 0 || (M > 0 && (!points || !ids))) return KN_E_INVALID_ARG;
    if (M == 0) return KN_OK;
    dim3 grid;
    KN_TRY(launch_1d(M, 256, grid));
    hipLaunchKernelGGL(k_cell_ids, grid, dim3(256), 0, (hipStream_t)stream, points, M, sc->net_grid, sc->cell_net, ids,
                       (int32_t *)nullptr, sc->N);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

// ids (optional) and sort keys in one pass over the points
int kn_cell_keys(const kn_scene *sc, hipStream_t st, const float *points, int64_t M, int32_t *ids, int32_t *keys)
{
    if (M == 0) return KN_OK;
    dim3 grid;
    KN_TRY(launch_1d(M, 256, grid));
    hipLaunchKernelGGL(k_cell_ids, grid, dim3(256), 0, st, points, M, sc->net_grid, sc->cell_net, ids, keys, sc->N);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

extern "C" int kn_bucket(kn_ctx *ctx, const kn_scene *sc, void *stream, const int32_t *ids, int64_t M, int32_t *counts,
                         int32_t *offsets, int32_t *perm, void *workspace, int64_t workspace_bytes)
{
    if (!ctx || !sc || M < 0 || (M > 0 && (!ids || !perm))) return KN_E_INVALID_ARG;
    if (M > (1ll << 30)) return KN_E_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < kn_bucket_ws_bytes(M, sc->N) + kn_align_up(M * 4, 256))
        return KN_E_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    KnCarver ws(workspace, workspace_bytes);
    int32_t *keys = ws.carve<int32_t>(M);
    if (M > 0) {
        dim3 grid;
        KN_TRY(launch_1d(M, 256, grid));
        hipLaunchKernelGGL(k_ids_to_keys, grid, dim3(256), 0, st, ids, M, sc->N, keys);
        KN_CHECK_LAUNCH();
    }
    KnBucketOut bo;
    return kn_bucket_run(st, keys, M, sc->N, 64, counts, offsets, perm, ws, &bo);
}
