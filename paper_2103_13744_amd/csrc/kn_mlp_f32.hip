// Grouped tiny-MLP evaluation in fp32 on the vector ALUs (scenes with KN_F32 weights).
//
// One wavefront per tile of the sorted sample list; every lane carries one sample through the
// encoding and the five layers (Sec. 3.2 "Network Architecture", Eq. 7).  All lanes of a wave use
// the same network, so weight addresses are wave-uniform and are fetched through the scalar
// path; activations stay in registers (all loops have compile-time bounds and are unrolled).
// Accumulation order: bias first, then inputs in index order.
#include "kn_common.h"
#include "kn_mlp_shared.h"

namespace {

template <int L> __device__ __forceinline__ void posenc_f32(float px, float py, float pz, float *out)
{
    out[0] = px;
    out[1] = py;
    out[2] = pz;
#pragma unroll
    for (int k = 0; k < L; ++k) {
        const float f = (float)(1 << k); // 2^k * p is exact in fp32
        out[3 + 6 * k + 0] = sinf(f * px);
        out[3 + 6 * k + 1] = sinf(f * py);
        out[3 + 6 * k + 2] = sinf(f * pz);
        out[3 + 6 * k + 3] = cosf(f * px);
        out[3 + 6 * k + 4] = cosf(f * py);
        out[3 + 6 * k + 5] = cosf(f * pz);
    }
}

template <int NI, int NO> __device__ __forceinline__ void affine_f32(const float *__restrict__ W, const float *__restrict__ b,
                                                                     const float *in, float *out)
{
#pragma unroll
    for (int o = 0; o < NO; ++o) out[o] = b[o];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const float v = in[i];
#pragma unroll
        for (int o = 0; o < NO; ++o) out[o] = fmaf(v, W[i * NO + o], out[o]);
    }
}

template <int H>
__global__ void __launch_bounds__(KN_WAVE) k_mlp_f32(const float *__restrict__ weights, int64_t P, KnSampleSrc src,
                                                     const int32_t *__restrict__ perm, const KnTile *__restrict__ tiles,
                                                     const int32_t *__restrict__ n_tiles, float *__restrict__ sigma,
                                                     float *__restrict__ rgb)
{
    constexpr int EX = 63, ED = 27;
    const int tile = blockIdx.x;
    if (tile >= *n_tiles) return;
    const KnTile tl = tiles[tile];
    const float *__restrict__ w = weights + (int64_t)tl.net * P;
    const float *W1 = w, *b1 = W1 + EX * H;
    const float *W2 = b1 + H, *b2 = W2 + H * H;
    const float *W3 = b2 + H, *b3 = W3 + H * (H + 1);
    const float *W4 = b3 + (H + 1), *b4 = W4 + (H + ED) * H;
    const float *W5 = b4 + H, *b5 = W5 + H * 3;
    const int lane = threadIdx.x;

    for (int base = 0; base < tl.len; base += KN_WAVE) {
        const int j = base + lane;
        const bool active = j < tl.len;
        const int32_t idx = perm[tl.start + (active ? j : 0)];
        float x, y, z, dx, dy, dz;
        kn_load_sample(src, idx, x, y, z, dx, dy, dz);

        float a[EX > H + ED ? EX : H + ED]; // input of the current layer
        float h[H + 1];
        posenc_f32<10>(x, y, z, a);
        affine_f32<EX, H>(W1, b1, a, h);
#pragma unroll
        for (int i = 0; i < H; ++i) a[i] = fmaxf(h[i], 0.0f);
        affine_f32<H, H>(W2, b2, a, h);
#pragma unroll
        for (int i = 0; i < H; ++i) a[i] = fmaxf(h[i], 0.0f);
        affine_f32<H, H + 1>(W3, b3, a, h);
        const float sg = fmaxf(h[0], 0.0f);
#pragma unroll
        for (int i = 0; i < H; ++i) a[i] = h[1 + i]; // feature vector, no activation
        posenc_f32<4>(dx, dy, dz, a + H);
        affine_f32<H + ED, H>(W4, b4, a, h);
#pragma unroll
        for (int i = 0; i < H; ++i) a[i] = fmaxf(h[i], 0.0f);
        float o5[3];
        affine_f32<H, 3>(W5, b5, a, o5);
        if (active) {
            float col[3];
#pragma unroll
            for (int c = 0; c < 3; ++c) col[c] = 1.0f / (1.0f + expf(-o5[c]));
            if (src.out4) {
                float *o = src.out4 + 4 * (int64_t)idx;
                o[0] = col[0];
                o[1] = col[1];
                o[2] = col[2];
                o[3] = sg;
            } else {
                sigma[idx] = sg;
#pragma unroll
                for (int c = 0; c < 3; ++c) rgb[3 * (int64_t)idx + c] = col[c];
            }
        }
    }
}

} // namespace

int kn_mlp_f32_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t max_tiles,
                      float *sigma, float *rgb)
{
    if (max_tiles <= 0) return KN_OK;
    const float *w = (const float *)sc->desc.weights;
    dim3 grid((unsigned)max_tiles), block(KN_WAVE);
    if (sc->desc.hidden == 32)
        hipLaunchKernelGGL(k_mlp_f32<32>, grid, block, 0, st, w, sc->P, src, b.perm, b.tiles, b.n_tiles, sigma, rgb);
    else if (sc->desc.hidden == 64)
        hipLaunchKernelGGL(k_mlp_f32<64>, grid, block, 0, st, w, sc->P, src, b.perm, b.tiles, b.n_tiles, sigma, rgb);
    else
        return KN_E_UNSUPPORTED;
    KN_CHECK_LAUNCH();
    return KN_OK;
}
