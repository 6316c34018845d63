// Grouped tiny-MLP evaluation in fp32 (scenes with KN_F32 weights) on the matrix cores' fp32 path.
//
// Same decomposition as the 16-bit kernel: a wavefront takes a contiguous range of tiles (<= 64 consecutive
// entries of the grouped sample list, all of one network) and keeps the network's weights in registers until
// the network changes.  Every layer of Sec. 3.2 / Eq. 7 is computed transposed, out^T = W^T * act^T, with
// v_mfma_f32_16x16x4_f32: the A operand is a 16(out) x 4(in) block of W^T (lane (m, g) = (lane%16, lane/16)
// supplies W[in slot g][out m]), the B operand a 4(in) x 16(samples) block of activations (lane (n, g)
// supplies input slot g of sample n), the accumulator a 16(out) x 16(samples) tile of which lane (n, g)
// holds outputs 4g + 0..3 of sample n.  An accumulator register is therefore already the B operand of one
// MFMA of the next layer: MFMA (t, j) of a layer consumes, from lane group g, hidden unit 16t + 4g + j.
// Which input sits in which slot is free as long as the A operand follows; weights are gathered from the
// canonical layout into that order once per scene (k_pack_weights_f32), as an image of the register file.
//
// Input slots.
//   gamma(x), 16 MFMAs q: group g < 3: axis g, frequency q/2, sin for even q, cos for odd q;
//                         group 3:    q < 12: axis q/4, frequency 8 + (q/2)%2, sin / cos; q = 12..14: x, y, z;
//                                     q = 15: the constant 1 that multiplies b1.
//   gamma(d), 8 MFMAs q:  group g < 3: axis g, frequency q/2, sin / cos; group 3: dx, dy, dz, 1 (b4), 0 x 4.
// b2, b3 and b5 initialise accumulators.
//
// Density and colour (1 + 3 output rows) share one accumulator among the four 16-sample tiles of a chunk:
// for tile u the A operand is masked to rows 4u..4u+3 (colour 4u+0..2, density 4u+3), after which lane l holds
// (r, g, b, sigma) of sample l of the 64.
//
// Encoding: accurate sincosf at frequencies 0, 4 (positions), 0 (directions) and 8 (group 3), up to three steps
// of the double-angle recurrence in between; all in fp32.
#include "kn_common.h"
#include "kn_mlp_shared.h"
#include <hip/hip_ext.h>
#include "kn_probe.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int F32_WAVES = 4;
constexpr int F32_TILE_LEN = 64;

__device__ __forceinline__ f4 mfma4(float a, float b, f4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

__device__ __forceinline__ void double_angle(float s, float c, float &s2, float &c2)
{
    s2 = 2.0f * (s * c);
    c2 = fmaf(-2.0f * s, s, 1.0f);
}

// Register file image of one network: register r of lane l sits at packed[(net * N + r) * 64 + l].
template <int H> struct Regs {
    static constexpr int HT = H / 16, HQ = H / 4;
    static constexpr int W1 = 0;                     // (t, q)  -> W1 + 16 t + q
    static constexpr int W2 = W1 + 16 * HT;          // (t, k)  -> W2 + HQ t + k
    static constexpr int W3 = W2 + HQ * HT;          // feature rows
    static constexpr int W4 = W3 + HQ * HT;          // (t, k)  -> W4 + (HQ + 8) t + k; k >= HQ: gamma(d)
    static constexpr int WO = W4 + (HQ + 8) * HT;    // colour rows (A rows with m%4 < 3) and the density row (m%4 = 3)
    static constexpr int B2 = WO + HQ;               // (t, j): accumulator initial values of this lane
    static constexpr int B3 = B2 + 4 * HT;
    static constexpr int BO = B3 + 4 * HT;
    static constexpr int N = BO + 4;
    // canonical offsets (Sec. 3.2: five layers, weights before biases)
    static constexpr int oW1 = 0, ob1 = 63 * H, oW2 = ob1 + H, ob2 = oW2 + H * H, oW3 = ob2 + H, ob3 = oW3 + H * (H + 1),
                         oW4 = ob3 + H + 1, ob4 = oW4 + (H + 27) * H, oW5 = ob4 + H, ob5 = oW5 + 3 * H;
};

// canonical index of the value in register r of lane `lane`; -1 = zero
template <int H> __device__ int reg_source(int r, int lane)
{
    using R = Regs<H>;
    constexpr int HQ = R::HQ;
    const int m = lane & 15, g = lane >> 4;
    auto unit = [&](int k) { return 16 * (k >> 2) + 4 * g + (k & 3); }; // hidden unit behind MFMA k for this lane group
    if (r < R::W2) {
        const int t = (r - R::W1) >> 4, q = (r - R::W1) & 15, col = 16 * t + m;
        if (g < 3) return R::oW1 + (3 + 6 * (q >> 1) + 3 * (q & 1) + g) * H + col;
        if (q < 12) return R::oW1 + (3 + 6 * (8 + ((q >> 1) & 1)) + 3 * (q & 1) + (q >> 2)) * H + col;
        return q < 15 ? R::oW1 + (q - 12) * H + col : R::ob1 + col;
    }
    if (r < R::W3) {
        const int t = (r - R::W2) / HQ, k = (r - R::W2) % HQ;
        return R::oW2 + unit(k) * H + 16 * t + m;
    }
    if (r < R::W4) {
        const int t = (r - R::W3) / HQ, k = (r - R::W3) % HQ;
        return R::oW3 + unit(k) * (H + 1) + 1 + 16 * t + m;
    }
    if (r < R::WO) {
        const int t = (r - R::W4) / (HQ + 8), k = (r - R::W4) % (HQ + 8), col = 16 * t + m;
        if (k < HQ) return R::oW4 + unit(k) * H + col;
        const int q = k - HQ;
        if (g < 3) return R::oW4 + (H + 3 + 6 * (q >> 1) + 3 * (q & 1) + g) * H + col;
        if (q < 3) return R::oW4 + (H + q) * H + col;
        return q == 3 ? R::ob4 + col : -1;
    }
    if (r < R::B2) {
        const int k = r - R::WO;
        return (m & 3) < 3 ? R::oW5 + unit(k) * 3 + (m & 3) : R::oW3 + unit(k) * (H + 1);
    }
    if (r < R::B3) return R::ob2 + 16 * ((r - R::B2) >> 2) + 4 * g + ((r - R::B2) & 3);
    if (r < R::BO) return R::ob3 + 1 + 16 * ((r - R::B3) >> 2) + 4 * g + ((r - R::B3) & 3);
    const int j = r - R::BO;
    return j < 3 ? R::ob5 + j : R::ob3;
}

template <int H>
__global__ void k_pack_weights_f32(const float *__restrict__ w, int64_t P, int32_t N, float *__restrict__ packed)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    constexpr int64_t per = Regs<H>::N * KN_WAVE;
    if (i >= per * N) return;
    const int64_t net = i / per;
    const int e = (int)(i - net * per);
    const int s = reg_source<H>(e >> 6, e & 63);
    packed[i] = s < 0 ? 0.0f : w[net * P + s];
}

template <int H>
__global__ void __launch_bounds__(F32_WAVES *KN_WAVE) __attribute__((amdgpu_waves_per_eu(H == 32 ? 2 : 1, H == 32 ? 2 : 1)))
    k_mlp_f32(const float *__restrict__ packed, KnSampleSrc src, const int32_t *__restrict__ perm,
              const KnTile *__restrict__ tiles, const int32_t *__restrict__ n_tiles, float *__restrict__ sigma,
              float *__restrict__ rgb)
{
    constexpr int HT = H / 16, HQ = H / 4; // output tiles per layer, MFMAs per hidden input vector
    __shared__ float stage[F32_WAVES][KN_WAVE][8]; // x, y, z, dx, dy, dz of the chunk's samples

    const int wave = threadIdx.x / KN_WAVE, lane = threadIdx.x & (KN_WAVE - 1);
    const int n = lane & 15, g = lane >> 4;
    const bool g3 = g == 3;
    const f4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};

    const int total_tiles = *n_tiles;
    const int total_waves = gridDim.x * F32_WAVES;
    // workgroup b runs on XCD b % 8: renumbered so that an XCD (one L2) works on a contiguous eighth of the tile list
    const int xcd_share = gridDim.x >> 3;
    const int block_no = (gridDim.x & 7) == 0 ? (int)(blockIdx.x & 7) * xcd_share + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int wid = __builtin_amdgcn_readfirstlane(block_no * F32_WAVES + wave);
    const int t_lo = __builtin_amdgcn_readfirstlane((int)((int64_t)wid * total_tiles / total_waves));
    const int t_hi = __builtin_amdgcn_readfirstlane((int)((int64_t)(wid + 1) * total_tiles / total_waves));
    if (t_lo >= t_hi) return;

    using R = Regs<H>;
    float w1[HT][16], w2[HT][HQ], w3[HT][HQ], w4[HT][HQ + 8], wo[HQ];
    f4 bias2[HT], bias3[HT], bias_out;
    auto load_network = [&](int32_t net) {
        const float *__restrict__ wp = packed + (int64_t)net * (R::N * KN_WAVE) + lane;
        auto reg = [&](int r) { return wp[r * KN_WAVE]; };
#pragma unroll
        for (int t = 0; t < HT; ++t) {
#pragma unroll
            for (int q = 0; q < 16; ++q) w1[t][q] = reg(R::W1 + 16 * t + q);
#pragma unroll
            for (int k = 0; k < HQ; ++k) {
                w2[t][k] = reg(R::W2 + HQ * t + k);
                w3[t][k] = reg(R::W3 + HQ * t + k);
            }
#pragma unroll
            for (int k = 0; k < HQ + 8; ++k) w4[t][k] = reg(R::W4 + (HQ + 8) * t + k);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bias2[t][j] = reg(R::B2 + 4 * t + j);
                bias3[t][j] = reg(R::B3 + 4 * t + j);
            }
        }
#pragma unroll
        for (int k = 0; k < HQ; ++k) wo[k] = reg(R::WO + k);
#pragma unroll
        for (int j = 0; j < 4; ++j) bias_out[j] = reg(R::BO + j);
    };

    auto descriptor = [&](int t) -> KnTile { return tiles[min(t, t_hi - 1)]; };
    auto sample_index = [&](const KnTile &d) {
        const int32_t pos = d.start + min(lane, d.len - 1);
        return src.records ? pos : perm[pos]; // re-ordered records: the sorted list holds the samples themselves
    };
    KnTile dsc_next = descriptor(t_lo);
    int32_t idx_next = sample_index(dsc_next);
    int32_t net_cur = -1;

    for (int t = t_lo; t < t_hi; ++t) {
        const KnTile tl = dsc_next;
        const int32_t idx = idx_next;
        float x, y, z, dx, dy, dz, dscale;
        int32_t out_idx;
        kn_load_sample(src, idx, x, y, z, dx, dy, dz, dscale, out_idx);
        dsc_next = descriptor(t + 1);
        idx_next = sample_index(dsc_next);
        if (tl.net != net_cur) { // uniform
            load_network(tl.net);
            net_cur = tl.net;
        }
        *(f4 *)&stage[wave][lane][0] = (f4){x, y, z, dx};
        *(f4 *)&stage[wave][lane][4] = (f4){dy, dz, 0.0f, 0.0f};
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        f4 out = bias_out;
#pragma unroll 1
        for (int u = 0; u < 4; ++u) {
            const f4 s0 = *(const f4 *)&stage[wave][16 * u + n][0];
            const f4 s1 = *(const f4 *)&stage[wave][16 * u + n][4];
            const float p[3] = {s0[0], s0[1], s0[2]}, d[3] = {s0[3], s1[0], s1[1]};
            const float pg = g == 0 ? p[0] : (g == 1 ? p[1] : p[2]);
            const float dg = g == 0 ? d[0] : (g == 1 ? d[1] : d[2]);
            // three accurate evaluations per lane; groups 0..2: axis g at frequencies 0 and 4 and the direction at 0,
            // group 3: the three axes at frequency 8
            const float ang[3] = {g3 ? 256.0f * p[0] : pg, g3 ? 256.0f * p[1] : 16.0f * pg, g3 ? 256.0f * p[2] : dg};
            float cs[3][4], cc[3][4];
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                sincosf(ang[c], &cs[c][0], &cc[c][0]);
#pragma unroll
                for (int k = 1; k < 4; ++k) double_angle(cs[c][k - 1], cc[c][k - 1], cs[c][k], cc[c][k]);
            }
            float enc[16], dirv[8];
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int f = q >> 1;
                const float axis_v = (q & 1) ? cc[f >> 2][f & 3] : cs[f >> 2][f & 3];
                const float g3_v = q < 12 ? ((q & 1) ? cc[q >> 2][(q >> 1) & 1] : cs[q >> 2][(q >> 1) & 1])
                                          : (q < 15 ? p[q >= 12 && q < 15 ? q - 12 : 0] : 1.0f);
                enc[q] = g3 ? g3_v : axis_v;
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const float axis_v = (q & 1) ? cc[2][q >> 1] : cs[2][q >> 1];
                const float g3_v = q < 3 ? d[q < 3 ? q : 0] : (q == 3 ? 1.0f : 0.0f);
                dirv[q] = g3 ? g3_v : axis_v;
            }
            const bool my_tile = (n >> 2) == u;
            const bool sig_row = my_tile && (n & 3) == 3, col_row = my_tile && (n & 3) < 3;

            f4 acc[HT], h[HT];
            // layer 1: gamma(x) -> H, ReLU
#pragma unroll
            for (int t2 = 0; t2 < HT; ++t2) {
                acc[t2] = zero4;
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[t2] = mfma4(w1[t2][q], enc[q], acc[t2]);
            }
#pragma unroll
            for (int t2 = 0; t2 < HT; ++t2)
#pragma unroll
                for (int j = 0; j < 4; ++j) h[t2][j] = fmaxf(acc[t2][j], 0.0f);
            // layer 2: H -> H, ReLU
#pragma unroll
            for (int t2 = 0; t2 < HT; ++t2) {
                acc[t2] = bias2[t2];
#pragma unroll
                for (int k = 0; k < HQ; ++k) acc[t2] = mfma4(w2[t2][k], h[k >> 2][k & 3], acc[t2]);
            }
#pragma unroll
            for (int t2 = 0; t2 < HT; ++t2)
#pragma unroll
                for (int j = 0; j < 4; ++j) h[t2][j] = fmaxf(acc[t2][j], 0.0f);
            // layer 3: H -> feature (no activation) and density (row 4u + 3 of the shared tile)
#pragma unroll
            for (int t2 = 0; t2 < HT; ++t2) {
                acc[t2] = bias3[t2];
#pragma unroll
                for (int k = 0; k < HQ; ++k) acc[t2] = mfma4(w3[t2][k], h[k >> 2][k & 3], acc[t2]);
            }
#pragma unroll
            for (int k = 0; k < HQ; ++k) out = mfma4(sig_row ? wo[k] : 0.0f, h[k >> 2][k & 3], out);
#pragma unroll
            for (int t2 = 0; t2 < HT; ++t2) h[t2] = acc[t2];
            // layer 4: [feature, gamma(d)] -> H, ReLU
#pragma unroll
            for (int t2 = 0; t2 < HT; ++t2) {
                acc[t2] = zero4;
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[t2] = mfma4(w4[t2][HQ + q], dirv[q], acc[t2]);
#pragma unroll
                for (int k = 0; k < HQ; ++k) acc[t2] = mfma4(w4[t2][k], h[k >> 2][k & 3], acc[t2]);
            }
#pragma unroll
            for (int t2 = 0; t2 < HT; ++t2)
#pragma unroll
                for (int j = 0; j < 4; ++j) h[t2][j] = fmaxf(acc[t2][j], 0.0f);
            // layer 5: H -> colour rows 4u + 0..2 of the shared tile
#pragma unroll
            for (int k = 0; k < HQ; ++k) out = mfma4(col_row ? wo[k] : 0.0f, h[k >> 2][k & 3], out);
        }
        __builtin_amdgcn_wave_barrier(); // the staging buffer is rewritten by the next iteration

        if (lane < tl.len) {
            const float sg = fmaxf(out[3], 0.0f) * dscale;
            float col[3];
#pragma unroll
            for (int c = 0; c < 3; ++c) col[c] = 1.0f / (1.0f + expf(-out[c]));
            if (src.out4) {
                *(f4 *)(src.out4 + 4 * (int64_t)out_idx) = (f4){col[0], col[1], col[2], sg};
            } else {
                sigma[out_idx] = sg;
#pragma unroll
                for (int c = 0; c < 3; ++c) rgb[3 * (int64_t)out_idx + c] = col[c];
            }
        }
    }
}


// Density only, for occupancy extraction (Sec. 3.4): layers 1 and 2 and the density row of layer 3 at the probe
// points of one network cell's voxels, which are generated in the kernel.  Same formulation as k_mlp_f32.
template <int H>
__global__ void __launch_bounds__(F32_WAVES *KN_WAVE) __attribute__((amdgpu_waves_per_eu(2, 2)))
    k_probe_f32(const float *__restrict__ packed, KnProbeJob job)
{
    using R = Regs<H>;
    constexpr int HT = H / 16, HQ = H / 4;
    __shared__ float stage[F32_WAVES][KN_WAVE][4];
    const int wave = threadIdx.x / KN_WAVE, lane = threadIdx.x & (KN_WAVE - 1);
    const int n = lane & 15, g = lane >> 4;
    const bool g3 = g == 3;
    const f4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};

    const int32_t cell = blockIdx.x / job.parts, part = blockIdx.x - cell * job.parts;
    const KnProbeBox box = kn_probe_box(job, cell);
    if (box.points == 0) return;
    const int shares = job.parts * F32_WAVES, share = part * F32_WAVES + wave;
    const int t_lo = __builtin_amdgcn_readfirstlane((int)((int64_t)share * box.tiles / shares));
    const int t_hi = __builtin_amdgcn_readfirstlane((int)((int64_t)(share + 1) * box.tiles / shares));
    if (t_lo >= t_hi) return;

    float w1[HT][16], w2[HT][HQ], wo[HQ], bias_sig = 0.0f;
    f4 bias2[HT];
    auto load_network = [&](int32_t net) {
        const float *__restrict__ wp = packed + (int64_t)net * (R::N * KN_WAVE) + lane;
        auto reg = [&](int r) { return wp[r * KN_WAVE]; };
#pragma unroll
        for (int t = 0; t < HT; ++t) {
#pragma unroll
            for (int q = 0; q < 16; ++q) w1[t][q] = reg(R::W1 + 16 * t + q);
#pragma unroll
            for (int k = 0; k < HQ; ++k) w2[t][k] = reg(R::W2 + HQ * t + k);
#pragma unroll
            for (int j = 0; j < 4; ++j) bias2[t][j] = reg(R::B2 + 4 * t + j);
        }
#pragma unroll
        for (int k = 0; k < HQ; ++k) wo[k] = reg(R::WO + k);
        bias_sig = reg(R::BO + 3);
    };
    int32_t net_loaded = -1;

    // every probe of a voxel in its home cell: one network for the whole box (none: nothing to mark)
    const int32_t home_net = kn_net_of_cell(job.cell_net, cell);
    if (job.nested && home_net < 0) return;
    KnProbeCursor cur = kn_probe_cursor(box, t_lo * KN_WAVE + lane);
    for (int t = t_lo; t < t_hi; ++t, kn_probe_cursor_step(box, cur)) {
        const int32_t p = t * KN_WAVE + lane;
        const bool active = p < box.points; // (beyond the box's last probe the cursor points past the box: unused)
        float x, y, z;
        int64_t voxel;
        const int32_t probe = cur.probe;
        kn_probe_point(job, box, cur, x, y, z, voxel);
        const int32_t net = job.nested ? home_net : kn_net_of_cell(job.cell_net, kn_grid_index(job.net, x, y, z));
        bool todo = active && net >= 0;
        float sg = 0.0f;
        *(f4 *)&stage[wave][lane][0] = (f4){x, y, z, 0.0f};
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // one pass per network met in the tile (a single one when the grids nest)
        for (;;) {
            const unsigned long long pending = __ballot(todo);
            if (pending == 0ull) break;
            const int32_t nsel = __builtin_amdgcn_readlane(net, (int)__builtin_ctzll(pending));
            if (nsel != net_loaded) {
                load_network(nsel);
                net_loaded = nsel;
            }
            f4 out = {0.0f, 0.0f, 0.0f, bias_sig};
#pragma unroll 1
            for (int u = 0; u < 4; ++u) {
                const f4 s0 = *(const f4 *)&stage[wave][16 * u + n][0];
                const float pt[3] = {s0[0], s0[1], s0[2]};
                const float pg = g == 0 ? pt[0] : (g == 1 ? pt[1] : pt[2]);
                // groups 0..2: axis g at frequencies 0 and 4; group 3: the three axes at frequency 8
                const float ang[3] = {g3 ? 256.0f * pt[0] : pg, g3 ? 256.0f * pt[1] : 16.0f * pg, 256.0f * pt[2]};
                float cs[3][4], cc[3][4];
#pragma unroll
                for (int c = 0; c < 3; ++c) {
                    sincosf(ang[c], &cs[c][0], &cc[c][0]);
#pragma unroll
                    for (int k = 1; k < 4; ++k) double_angle(cs[c][k - 1], cc[c][k - 1], cs[c][k], cc[c][k]);
                }
                float enc[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int f = q >> 1;
                    const float axis_v = (q & 1) ? cc[f >> 2][f & 3] : cs[f >> 2][f & 3];
                    const float g3_v = q < 12 ? ((q & 1) ? cc[q >> 2][(q >> 1) & 1] : cs[q >> 2][(q >> 1) & 1])
                                              : (q < 15 ? pt[q >= 12 && q < 15 ? q - 12 : 0] : 1.0f);
                    enc[q] = g3 ? g3_v : axis_v;
                }
                const bool sig_row = (n >> 2) == u && (n & 3) == 3;
                f4 acc[HT], h[HT];
#pragma unroll
                for (int t2 = 0; t2 < HT; ++t2) {
                    acc[t2] = zero4;
#pragma unroll
                    for (int q = 0; q < 16; ++q) acc[t2] = mfma4(w1[t2][q], enc[q], acc[t2]);
                }
#pragma unroll
                for (int t2 = 0; t2 < HT; ++t2)
#pragma unroll
                    for (int j = 0; j < 4; ++j) h[t2][j] = fmaxf(acc[t2][j], 0.0f);
#pragma unroll
                for (int t2 = 0; t2 < HT; ++t2) {
                    acc[t2] = bias2[t2];
#pragma unroll
                    for (int k = 0; k < HQ; ++k) acc[t2] = mfma4(w2[t2][k], h[k >> 2][k & 3], acc[t2]);
                }
#pragma unroll
                for (int t2 = 0; t2 < HT; ++t2)
#pragma unroll
                    for (int j = 0; j < 4; ++j) h[t2][j] = fmaxf(acc[t2][j], 0.0f);
#pragma unroll
                for (int k = 0; k < HQ; ++k) out = mfma4(sig_row ? wo[k] : 0.0f, h[k >> 2][k & 3], out);
            }
            if (todo && net == nsel) {
                sg = fmaxf(out[3], 0.0f);
                todo = false;
            }
        }
        __builtin_amdgcn_wave_barrier(); // the staging buffer is rewritten by the next iteration
        kn_probe_mark(job, active, sg > job.tau, voxel, probe, lane);
    }
}

} // namespace

int kn_mlp_f32_tile_len(const kn_scene *) { return F32_TILE_LEN; }

// bytes of the packed weights of N networks of width H (0: no kernel for that width)
int64_t kn_mlp_f32_packed_bytes(int32_t H, int64_t N)
{
    if (H != 32 && H != 64) return 0;
    return (int64_t)(H == 32 ? Regs<32>::N : Regs<64>::N) * KN_WAVE * 4 * N;
}

// fills sc->packed_w (kn_mlp_f32_packed_bytes bytes, assigned by the caller)
int kn_mlp_f32_pack_weights(kn_scene *sc, hipStream_t st)
{
    const int H = sc->desc.hidden;
    if (H != 32 && H != 64) return KN_E_UNSUPPORTED;
    if (!sc->packed_w) return KN_E_INVALID_ARG;
    const int64_t per = (H == 32 ? Regs<32>::N : Regs<64>::N) * KN_WAVE;
    const int64_t blocks = kn_div_up(per * sc->N, 256);
    if (blocks > 0x7fffffffLL) return KN_E_UNSUPPORTED;
    const float *w = (const float *)sc->desc.weights;
    if (H == 32)
        hipLaunchKernelGGL(k_pack_weights_f32<32>, dim3((unsigned)blocks), dim3(256), 0, st, w, sc->P, sc->N, (float *)sc->packed_w);
    else
        hipLaunchKernelGGL(k_pack_weights_f32<64>, dim3((unsigned)blocks), dim3(256), 0, st, w, sc->P, sc->N, (float *)sc->packed_w);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

int kn_mlp_f32_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t max_tiles,
                      float *sigma, float *rgb, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (max_tiles <= 0) return KN_OK;
    const float *w = (const float *)sc->packed_w;
    const int H = sc->desc.hidden;
    if (H != 32 && H != 64) return KN_E_UNSUPPORTED;
    // one workgroup of 4 wavefronts per compute unit and resident wavefront (H = 32: two per SIMD, H = 64: one)
    int64_t blocks = kn_div_up(max_tiles, F32_WAVES);
    const int64_t fill = H == 32 ? 512 : 256;
    if (blocks > fill) blocks = fill;
    dim3 grid((unsigned)blocks), block(F32_WAVES * KN_WAVE);
    auto kernel = H == 32 ? k_mlp_f32<32> : k_mlp_f32<64>;
    if (ev_start && ev_stop)
        hipExtLaunchKernelGGL(kernel, grid, block, 0, st, ev_start, ev_stop, 0, w, src, b.perm, b.tiles, b.n_tiles, sigma, rgb);
    else
        hipLaunchKernelGGL(kernel, grid, block, 0, st, w, src, b.perm, b.tiles, b.n_tiles, sigma, rgb);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

int kn_probe_f32_launch(const kn_scene *sc, hipStream_t st, const KnProbeJob &job)
{
    const int H = sc->desc.hidden;
    if (H != 32 && H != 64) return KN_E_UNSUPPORTED;
    const dim3 grid((unsigned)(sc->cells * job.parts)), block(F32_WAVES * KN_WAVE);
    const float *w = (const float *)sc->packed_w;
    if (H == 32)
        hipLaunchKernelGGL(k_probe_f32<32>, grid, block, 0, st, w, job);
    else
        hipLaunchKernelGGL(k_probe_f32<64>, grid, block, 0, st, w, job);
    KN_CHECK_LAUNCH();
    return KN_OK;
}
