// Micro-benchmarks of this machine's own limits, for the benchmark's "fraction of measured peak" figures: what a
// plain device copy, a read-only sweep, a register-only MFMA loop and a register-only FMA / sine loop reach on the
// GPU the benchmark runs on.  Built into a library of its own (libkn_peaks.so); nothing in libkilonerf_hip.so uses it.
//
// Every function launches on `stream`, times `reps` launches with HIP events on that stream (best of them) and
// returns the rate; device buffers are the caller's.  Return value 0 = ok, negative = error.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(256) k_copy(const float4 *__restrict__ in, float4 *__restrict__ out, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = in[i];
}

__global__ void __launch_bounds__(256) k_read(const float4 *__restrict__ in, size_t n, float *__restrict__ sink)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    for (; i + 3 * stride < n; i += 4 * stride) { // four independent loads in flight per thread
        const float4 v0 = in[i], v1 = in[i + stride], v2 = in[i + 2 * stride], v3 = in[i + 3 * stride];
        a.x += v0.x + v1.x + v2.x + v3.x;
        a.y += v0.y + v1.y + v2.y + v3.y;
        a.z += v0.z + v1.z + v2.z + v3.z;
        a.w += v0.w + v1.w + v2.w + v3.w;
    }
    for (; i < n; i += stride) a.x += in[i].x;
    if (a.x + a.y + a.z + a.w == 1.2345e-30f) sink[0] = 1.0f; // keeps the loads alive; practically never true
}

// 4 independent accumulators per wavefront: the matrix pipeline is never waiting for a result
template <int KIND> __global__ void __launch_bounds__(256) k_mfma(float *out, int iters)
{
    f4 acc[4];
    for (int u = 0; u < 4; ++u) acc[u] = (f4){0.f, 0.f, 0.f, 0.f};
    if constexpr (KIND == 0) {
        h8 a, b;
        for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(threadIdx.x * 0.001f); b[i] = (_Float16)0.5f; }
        for (int i = 0; i < iters; ++i)
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[u], 0, 0, 0);
    } else if constexpr (KIND == 1) {
        b8 a, b;
        for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.001f); b[i] = (__bf16)0.5f; }
        for (int i = 0; i < iters; ++i)
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[u], 0, 0, 0);
    } else {
        const float a = threadIdx.x * 0.001f, b = 0.5f;
        for (int i = 0; i < iters; ++i)
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[u], 0, 0, 0);
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc[0][0] + acc[1][0] + acc[2][0] + acc[3][0];
}

// KIND 0: 16 independent fp32 FMAs per iteration; KIND 1: 8 independent hardware sines
template <int KIND> __global__ void __launch_bounds__(256) k_valu(float *out, int iters)
{
    float a[8];
    for (int u = 0; u < 8; ++u) a[u] = threadIdx.x * 1e-3f + u * 0.1f;
    const float b = 1.0001f, c = 0.5f;
    for (int i = 0; i < iters; ++i) {
        if constexpr (KIND == 0) {
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = __builtin_fmaf(a[u], b, c);
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = __builtin_fmaf(a[u], b, c);
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = __builtin_amdgcn_sinf(a[u]);
        }
    }
    float s = 0.f;
    for (int u = 0; u < 8; ++u) s += a[u];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <typename F> int best_ms(hipStream_t st, int reps, F launch, float *ms_out)
{
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -4;
    launch(); // warm-up
    float best = 1e30f;
    int rc = 0;
    for (int r = 0; r < reps && rc == 0; ++r) {
        float ms = 0.f;
        if (hipEventRecord(e0, st) != hipSuccess) rc = -4;
        launch();
        if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess)
            rc = -4;
        if (ms < best) best = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *ms_out = best;
    return rc;
}

constexpr int BLOCKS = 256 * 8; // eight workgroups of four wavefronts per compute unit

} // namespace

extern "C" {

// plain copy of `bytes` (a multiple of 16) from src to dst: bytes read + bytes written per second
int kn_peak_copy(void *stream, const void *src, void *dst, int64_t bytes, int reps, double *bytes_per_sec)
{
    if (!src || !dst || bytes < 16 || (bytes & 15) || reps < 1 || !bytes_per_sec) return -1;
    hipStream_t st = (hipStream_t)stream;
    float ms;
    const size_t n = (size_t)bytes / 16;
    const int rc = best_ms(st, reps, [&] { hipLaunchKernelGGL(k_copy, dim3(256 * 16), dim3(256), 0, st, (const float4 *)src, (float4 *)dst, n); }, &ms);
    *bytes_per_sec = 2.0 * (double)bytes / (ms * 1e-3);
    return rc;
}

// read-only sweep over `bytes` (a multiple of 16): bytes read per second.  sink: one float of device memory
int kn_peak_read(void *stream, const void *src, int64_t bytes, float *sink, int reps, double *bytes_per_sec)
{
    if (!src || !sink || bytes < 16 || (bytes & 15) || reps < 1 || !bytes_per_sec) return -1;
    hipStream_t st = (hipStream_t)stream;
    float ms;
    const size_t n = (size_t)bytes / 16;
    const int rc = best_ms(st, reps, [&] { hipLaunchKernelGGL(k_read, dim3(256 * 16), dim3(256), 0, st, (const float4 *)src, n, sink); }, &ms);
    *bytes_per_sec = (double)bytes / (ms * 1e-3);
    return rc;
}

// register-only MFMA loop: kind 0 = v_mfma_f32_16x16x32_f16, 1 = ..._bf16, 2 = v_mfma_f32_16x16x4_f32.
// out: 256 * 8 * 256 floats of device memory.  FLOP per second (2 per multiply-add).
int kn_peak_mfma(void *stream, int kind, float *out, int iters, int reps, double *flop_per_sec)
{
    if (!out || kind < 0 || kind > 2 || iters < 1 || reps < 1 || !flop_per_sec) return -1;
    hipStream_t st = (hipStream_t)stream;
    float ms;
    const int rc = best_ms(st, reps, [&] {
        if (kind == 0) hipLaunchKernelGGL(k_mfma<0>, dim3(BLOCKS), dim3(256), 0, st, out, iters);
        else if (kind == 1) hipLaunchKernelGGL(k_mfma<1>, dim3(BLOCKS), dim3(256), 0, st, out, iters);
        else hipLaunchKernelGGL(k_mfma<2>, dim3(BLOCKS), dim3(256), 0, st, out, iters);
    }, &ms);
    const double mac = kind == 2 ? 16.0 * 16 * 4 : 16.0 * 16 * 32; // per instruction and wavefront
    *flop_per_sec = 2.0 * mac * 4.0 * iters * ((double)BLOCKS * 4) / (ms * 1e-3);
    return rc;
}

// register-only vector-ALU loop: kind 0 = fp32 FMA (FLOP per second, 2 per FMA), kind 1 = v_sin_f32 (sines per second)
int kn_peak_valu(void *stream, int kind, float *out, int iters, int reps, double *per_sec)
{
    if (!out || kind < 0 || kind > 1 || iters < 1 || reps < 1 || !per_sec) return -1;
    hipStream_t st = (hipStream_t)stream;
    float ms;
    const int rc = best_ms(st, reps, [&] {
        if (kind == 0) hipLaunchKernelGGL(k_valu<0>, dim3(BLOCKS), dim3(256), 0, st, out, iters);
        else hipLaunchKernelGGL(k_valu<1>, dim3(BLOCKS), dim3(256), 0, st, out, iters);
    }, &ms);
    const double per_thread = kind == 0 ? 2.0 * 16 * iters : 8.0 * iters;
    *per_sec = per_thread * (double)BLOCKS * 256 / (ms * 1e-3);
    return rc;
}

} // extern "C"
