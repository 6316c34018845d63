// Grouped tiny-MLP evaluation on the matrix cores (scenes with KN_F16 / KN_BF16 weights).
//
// A wavefront evaluates tiles (<= 64 consecutive entries of the grouped sample list, all of one
// network): encoding, the five layers of Sec. 3.2 and the output activations in one kernel
// (the paper's Sec. 3.5 fuses the whole network evaluation into one kernel as well; everything
// below that sentence is this library's own design for 64-wide wavefronts and MFMA).  Every
// wavefront takes a contiguous range of the tile list and re-fetches weights only when the network
// changes from one tile to the next.
//
// Formulation.  Every layer is computed transposed, out^T = W^T * act^T, with
// v_mfma_f32_16x16x32_{f16,bf16}: the A operand is a 16(out) x 32(in) block of W^T, the B operand
// a 32(in) x 16(samples) block of activations, the accumulator a 16(out) x 16(samples) tile in
// fp32.  In that orientation lane (n = lane%16, g = lane/16) of the accumulator holds outputs
// 16t+4g+{0..3} of sample n, and the same lane must supply 8 inputs of sample n to the next MFMA;
// so accumulators are activated, rounded to 16 bit, packed and used as the next B operand in
// place, with no shuffle and no LDS round trip.  Which input sits in which of the 8 slots of a
// lane is a free choice as long as the weight block uses the same order: weights are re-ordered
// once per scene (k_pack_weights) into that "slot order".
//
// Slot order (kb = 32-input block, g = lane/16, j = 0..7):
//   hidden vector : feature 16*(2kb + j/4) + 4g + j%4   (= what the accumulators hold)
//   gamma(x), 64 slots: g < 3: axis g, frequency 4kb + j/2, sin for even j, cos for odd j;
//                       g = 3: kb 0: x f8, x f9, y f8, y f9 (sin, cos each);
//                              kb 1: z f8, z f9, then x, y, z, 1 (the 1 multiplies the bias b1)
//   gamma(d), 32 slots: g < 3: axis g, frequency j/2, sin/cos;  g = 3: dx, dy, dz, 1 (bias b4), 0 x 4
// Biases b1 and b4 ride in the constant-1 slots; b2, b5 and the density bias initialise the accumulators.
//
// Feature layer.  Layer 3's feature vector has no activation (Sec. 3.2: it is handed to the last hidden layer together
// with gamma(d)), so feature layer and layer 4 are one affine map of the second hidden vector h2:
//   W4f^T (W3f^T h2 + b3f) + W4d^T gamma(d) + b4 = (W3f W4f)^T h2 + W4d^T gamma(d) + (b4 + W4f^T b3f).
// k_pack_weights forms W3f W4f and the bias once per scene (fp32 sums, rounded to the scene's 16-bit type like every
// other operand), and the kernels evaluate layer 4 on h2 directly: per 16 samples H/16 * H/32 MFMAs and H/8 conversions
// fewer, and the feature vector is never rounded to 16 bit.  Layer 3 proper is then the density row alone.
//
// Density and colour.  Layer 3's density row and layer 5's three colour rows would each waste a
// 16-row output tile.  Instead four sample tiles (64 samples) share two extra accumulators: for
// sample tile u the density row sits at row 4u+3 and the colour rows at 4u+0..2 of one weight block
// (masked to those four rows); the block multiplies h2 into the first accumulator, whose rows 4u+3
// are the densities, and h4 into the second, whose rows 4u+0..2 are the colours.  Afterwards
// lane l holds (r, g, b, sigma) pre-activations of sample l of the 64, one sample per lane.
//
// Encoding.  sin/cos of 2^f * p come from v_sin_f32 / v_cos_f32 at three "restart" frequencies
// per lane and the double-angle recurrence in between (fp32), which is far inside the 16-bit
// rounding of the operands.  The coordinates of the 64 samples of a tile are staged in LDS, scaled
// to revolutions per restart frequency, so that each lane group reads exactly the operands of its
// role.
#include "kn_common.h"
#include "kn_dir_encode.h"
#include <hip/hip_ext.h>
#include "kn_mlp_shared.h"
#include "kn_probe.h"

namespace {

using kn_enc::double_angle;
using kn_enc::INV_2PI;
using kn_enc::pk;
using kn_enc::sincos_rev;

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef __bf16 b2 __attribute__((ext_vector_type(2)));
typedef short s2 __attribute__((ext_vector_type(2)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned u4 __attribute__((ext_vector_type(4)));

constexpr int MLP_WAVES = 4;     // wavefronts per workgroup (one per SIMD of a compute unit)
constexpr int MLP_TILE_LEN = 64; // one chunk: the unit in which work is dealt out to the wavefronts

template <int H> struct Lay {
    static constexpr int HT = H / 16, HK = H / 32;
    static constexpr int L1 = 0;                          // (t, kb) -> L1 + 2t + kb
    static constexpr int L2 = L1 + 2 * HT;                // (t, kb) -> L2 + t*HK + kb
    static constexpr int LS = L2 + HT * HK;               // density row of layer 3, (kb)
    static constexpr int L4 = LS + HK;                    // (t, kb) -> L4 + t*(HK+1) + kb; kb < HK: h2 through the folded
                                                          // feature layer, kb = HK: gamma(d)
    static constexpr int L5 = L4 + HT * (HK + 1);         // colour rows, (kb)
    static constexpr int NBLK = L5 + HK;
    static constexpr int TAIL_FLOATS = H + 4;             // b2[H], b5[3], b3 density
    static constexpr int HALFS = NBLK * 512 + TAIL_FLOATS * 2;
    // canonical offsets
    static constexpr int oW1 = 0, ob1 = 63 * H, oW2 = ob1 + H, ob2 = oW2 + H * H, oW3 = ob2 + H,
                         ob3 = oW3 + H * (H + 1), oW4 = ob3 + H + 1, ob4 = oW4 + (H + 27) * H, oW5 = ob4 + H,
                         ob5 = oW5 + 3 * H;
};

__host__ __device__ inline int hid_feat(int kb, int g, int j) { return 16 * (2 * kb + j / 4) + 4 * g + j % 4; }

// canonical row of W1 behind slot (kb, g, j); 63 = the bias slot
__host__ __device__ inline int l1_row(int kb, int g, int j)
{
    if (g < 3) return 3 + 6 * (4 * kb + j / 2) + 3 * (j & 1) + g;
    const int p = 4 * kb + j / 2; // pair index 0..7 of the fourth lane group
    if (p < 6) return 3 + 6 * (8 + (p & 1)) + 3 * (j & 1) + p / 2;
    return (p == 6) ? (j & 1) : ((j & 1) ? 63 : 2);
}

// canonical row of W4 (relative to its first gamma(d) row) behind slot (g, j): -1 = bias, -2 = zero
__host__ __device__ inline int dir_row(int g, int j)
{
    if (g < 3) return 3 + 6 * (j / 2) + 3 * (j & 1) + g;
    if (j < 3) return j;
    return j == 3 ? -1 : -2;
}

// source element (canonical index) of packed 16-bit element e of one network; -1 = zero; FOLD_ROW - (k * H + col):
// element (k, col) of the product of feature layer and layer 4; FOLD_BIAS - col: element col of the folded bias
constexpr int FOLD_ROW = -2, FOLD_BIAS = -2 - 64 * 64;
template <int H> __device__ int pack_source(int e)
{
    using L = Lay<H>;
    const int blk = e >> 9, lane = (e >> 3) & 63, j = e & 7, m = lane & 15, g = lane >> 4;
    if (blk < L::L2) {
        const int t = (blk - L::L1) >> 1, kb = (blk - L::L1) & 1, col = 16 * t + m, r = l1_row(kb, g, j);
        return r < 63 ? L::oW1 + r * H + col : L::ob1 + col;
    }
    if (blk < L::LS) {
        const int t = (blk - L::L2) / L::HK, kb = (blk - L::L2) % L::HK;
        return L::oW2 + hid_feat(kb, g, j) * H + 16 * t + m;
    }
    if (blk < L::L4) {
        const int kb = blk - L::LS;
        return (m & 3) == 3 ? L::oW3 + hid_feat(kb, g, j) * (H + 1) : -1;
    }
    if (blk < L::L5) {
        const int t = (blk - L::L4) / (L::HK + 1), kb = (blk - L::L4) % (L::HK + 1), col = 16 * t + m;
        if (kb < L::HK) return FOLD_ROW - (hid_feat(kb, g, j) * H + col); // column `col` of row hid_feat of W3f W4f
        const int r = dir_row(g, j);
        if (r == -2) return -1;
        return r == -1 ? FOLD_BIAS - col : L::oW4 + (H + r) * H + col;     // b4 + W4f^T b3f
    }
    const int kb = blk - L::L5;
    return (m & 3) < 3 ? L::oW5 + hid_feat(kb, g, j) * 3 + (m & 3) : -1;
}

template <int H> __device__ int tail_source(int q)
{
    using L = Lay<H>;
    if (q < H) return L::ob2 + q;
    if (q < H + 3) return L::ob5 + (q - H);
    return L::ob3;
}

__device__ __forceinline__ float half_bits_to_float(uint16_t v, bool bf)
{
    if (bf) return __uint_as_float((uint32_t)v << 16);
    return (float)__builtin_bit_cast(_Float16, v);
}

// fp32 -> the scene's 16-bit type, round to nearest even
__device__ __forceinline__ uint16_t float_to_half_bits(float v, bool bf)
{
    if (!bf) return __builtin_bit_cast(uint16_t, (_Float16)v);
    const uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)0x7fc0; // NaN
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// `overflow`: set when a folded element leaves the range of the 16-bit type although its factors are finite
template <int H>
__global__ void k_pack_weights(const uint16_t *__restrict__ w, int64_t P, int32_t N, bool bf, uint16_t *__restrict__ packed,
                               int32_t *__restrict__ overflow)
{
    using L = Lay<H>;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t per = L::NBLK * 512 + L::TAIL_FLOATS;
    if (i >= per * N) return;
    const int64_t net = i / per;
    const int e = (int)(i - net * per);
    const uint16_t *src = w + net * P;
    uint16_t *dst = packed + net * (int64_t)L::HALFS;
    if (e < L::NBLK * 512) {
        const int s = pack_source<H>(e);
        if (s >= -1) {
            dst[e] = s < 0 ? (uint16_t)0 : src[s];
        } else {
            // feature layer folded into layer 4 (Sec. 3.2: no activation between them): sum over the feature index f of
            // (row k of W3's feature columns, or b3's feature part) times W4's feature row f, fp32, in index order
            const bool bias = s <= FOLD_BIAS;
            const int k = bias ? 0 : (FOLD_ROW - s) / H, col = bias ? FOLD_BIAS - s : (FOLD_ROW - s) % H;
            float acc = bias ? half_bits_to_float(src[L::ob4 + col], bf) : 0.0f;
            for (int f = 0; f < H; ++f) {
                const float a = half_bits_to_float(bias ? src[L::ob3 + 1 + f] : src[L::oW3 + k * (H + 1) + 1 + f], bf);
                acc = fmaf(a, half_bits_to_float(src[L::oW4 + f * H + col], bf), acc);
            }
            const uint16_t r = float_to_half_bits(acc, bf);
            if (isfinite(acc) && !isfinite(half_bits_to_float(r, bf))) atomicOr(overflow, 1);
            dst[e] = r;
        }
    } else {
        const int q = e - L::NBLK * 512;
        const float v = half_bits_to_float(src[tail_source<H>(q)], bf);
        ((float *)(dst + L::NBLK * 512))[q] = v;
    }
}
__global__ void k_clear_flag(int32_t *flag) { *flag = 0; }

// ---------------------------------------------------------------------------------------------
template <bool BF> __device__ __forceinline__ f4 mfma(u4 a, u4 b, f4 c)
{
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0);
}

// ReLU on two packed 16-bit floats: as signed 16-bit integers every negative float is negative
__device__ __forceinline__ unsigned relu2(unsigned v)
{
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(s2, v), (s2){0, 0}));
}

// accumulators of one layer (HT tiles) -> B operands of the next (HK blocks)
template <int H, bool BF, bool RELU> __device__ __forceinline__ void pack_acts(const f4 *acc, u4 *B)
{
#pragma unroll
    for (int kb = 0; kb < H / 32; ++kb) {
        unsigned r0 = pk<BF>(acc[2 * kb][0], acc[2 * kb][1]);
        unsigned r1 = pk<BF>(acc[2 * kb][2], acc[2 * kb][3]);
        unsigned r2 = pk<BF>(acc[2 * kb + 1][0], acc[2 * kb + 1][1]);
        unsigned r3 = pk<BF>(acc[2 * kb + 1][2], acc[2 * kb + 1][3]);
        if (RELU) { r0 = relu2(r0); r1 = relu2(r1); r2 = relu2(r2); r3 = relu2(r3); }
        B[kb] = (u4){r0, r1, r2, r3};
    }
}

// B operands of layer 1 for one lane: gamma(x) slots of lane group g (see "Slot order").  ang[0..2]: the lane's three
// restart angles in revolutions; ident[0..1]: the packed pairs (x, y), (z, 1) that sit in group 3's last slots.
template <bool BF, bool WRAP> __device__ __forceinline__ void encode_position(f4 ang, u4 ident, unsigned m3, u4 (&Bx)[2])
{
    // s[q] = sin, m[q] = cos of the q-th angle of this lane
    float s[8], m[8];
    sincos_rev<WRAP>(ang[0], s[0], m[0]);
    double_angle(s[0], m[0], s[1], m[1]);
    sincos_rev<WRAP>(ang[1], s[2], m[2]);
    double_angle(s[2], m[2], s[3], m[3]);
    sincos_rev<WRAP>(ang[2], s[4], m[4]);
    double_angle(s[4], m[4], s[5], m[5]);
    double_angle(s[5], m[5], s[6], m[6]);
    double_angle(s[6], m[6], s[7], m[7]);
    unsigned p[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) p[q] = pk<BF>(s[q], m[q]);
    p[6] = (ident[0] & m3) | (p[6] & ~m3);
    p[7] = (ident[1] & m3) | (p[7] & ~m3);
    Bx[0] = (u4){p[0], p[1], p[2], p[3]};
    Bx[1] = (u4){p[4], p[5], p[6], p[7]};
}
// The gamma(d) block of layer 4.  rev: the lane's direction component in revolutions; ident[2..3]: (dx, dy), (dz, 1).
template <bool BF> __device__ __forceinline__ u4 encode_direction(float rev, u4 ident, unsigned m3)
{
    float s[4], m[4];
    sincos_rev<false>(rev, s[0], m[0]); // directions: |d| far below 256 revolutions
    double_angle(s[0], m[0], s[1], m[1]);
    double_angle(s[1], m[1], s[2], m[2]);
    double_angle(s[2], m[2], s[3], m[3]);
    // group 3: slots 0..3 hold dx, dy, dz, 1; its slots 4..7 meet zero weights, any finite value does
    return (u4){(ident[2] & m3) | (pk<BF>(s[0], m[0]) & ~m3), (ident[3] & m3) | (pk<BF>(s[1], m[1]) & ~m3),
                pk<BF>(s[2], m[2]), pk<BF>(s[3], m[3])};
}

// Weights stay in registers: 12 blocks (48 VGPRs) for H = 32, four wavefronts per SIMD; 32 blocks (128 VGPRs) for
// H = 64, two wavefronts per SIMD (the matrix-core operands are read straight from the register file either way).
// STRAT (render with stratified sampling): the lattice points sit at their drawn offsets and the density is
// scaled by delta_k / step on the way out (see KnSampleSrc).
// SRC: where the samples come from (a compile-time choice: the width-64 kernel has no register to spare for the
// paths it does not take).  SRC_RAYS (render): lattice points rebuilt from packed (ray, k) records; gamma(d) is the
// same for every sample of a ray, so the render's set-up kernel encodes it once per ray, already in operand order
// (KnSampleSrc::dir_table), and a lane fetches its 16 bytes instead of computing them.  SRC_POINTS: the caller's
// arrays through the sorted index list `perm`.  SRC_RECORDS: the re-ordered samples themselves (`perm` is not read).
enum { SRC_RAYS = 0, SRC_POINTS = 1, SRC_RECORDS = 2 };
template <int H, bool BF, int WAVES, bool WRAP, bool STRAT, int SRC>
__global__ void __launch_bounds__(WAVES *KN_WAVE) __attribute__((amdgpu_waves_per_eu(H == 32 ? 4 : 2, H == 32 ? 4 : 2)))
    k_mlp_mfma(const uint16_t *__restrict__ packed, KnSampleSrc src, const int32_t *__restrict__ perm,
               const KnTile *__restrict__ tiles, const int32_t *__restrict__ n_tiles, float *__restrict__ sigma,
               float *__restrict__ rgb)
{
    using L = Lay<H>;
    constexpr int HT = L::HT, HK = L::HK, NBLK = L::NBLK;
    // Staging buffer: for each of the 64 samples of a chunk and each of the 4 lane groups, the 8 words that
    // lane group needs, so a lane reads its operands without selecting:
    //   [0..3] pre-scaled angles (revolutions) of the three restart points of gamma(x) and of gamma(d)
    //   [4..7] (group 3 only) the packed 16-bit pairs (x,y), (z,1), (dx,dy), (dz,1) that sit in its slots
    __shared__ f4 stage[WAVES][4][2][KN_WAVE]; // [lane group][half][sample]: conflict-free for writers and readers

    const int wave = threadIdx.x / KN_WAVE, lane = threadIdx.x & (KN_WAVE - 1);
    const int n = lane & 15, g = lane >> 4;
    const unsigned m3 = (g == 3) ? 0xffffffffu : 0u; // bit mask of lane group 3, for branch-free selects
    const int mrow = n >> 2; // the A-operand row of this lane is n; rows 4u..4u+3 belong to sample tile u
    const f4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    const u4 zero_u4 = {0u, 0u, 0u, 0u};
    // The tile list is cut into one contiguous range per wavefront (tiles are chunks of at most 64 samples, so
    // the ranges differ by one chunk at most).  Neighbouring tiles mostly belong to the same network: weights
    // are fetched only when the network changes.
    const int total_tiles = *n_tiles;
    const int total_waves = gridDim.x * WAVES;
    // Workgroups are dealt to the eight XCDs round-robin (workgroup b runs on XCD b % 8, each with an L2 of its
    // own).  Renumbered so that an XCD works on one contiguous eighth of the tile list, i.e. on neighbouring
    // networks: a ray's data and a network's weights are then fetched into one L2 instead of several.
    const int xcd_share = gridDim.x >> 3;
    const int block_no = (gridDim.x & 7) == 0 ? (int)(blockIdx.x & 7) * xcd_share + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int wid = __builtin_amdgcn_readfirstlane(block_no * WAVES + wave);
    // (kept in scalar registers: tile descriptors are then fetched through the scalar cache, whose counter is
    // separate from the one of the vector loads and stores in flight)
    const int t_lo = __builtin_amdgcn_readfirstlane((int)((int64_t)wid * total_tiles / total_waves));
    const int t_hi = __builtin_amdgcn_readfirstlane((int)((int64_t)(wid + 1) * total_tiles / total_waves));
    if (t_lo >= t_hi) return;

    u4 areg[NBLK];
    auto A = [&](int b) -> u4 {
        return areg[b];
    };
    // Density / colour rows: two accumulators shared by the four sample tiles (one fed with h2, one with h4), through
    // copies of one block that holds the density row and the colour rows side by side (they are disjoint rows of
    // period four in their blocks), restricted to the four output rows of tile u and made once per network: the
    // density accumulator's colour rows and the colour accumulator's density row hold sums nobody reads.  (Separate
    // masked copies of the two blocks cost 16 registers more at H = 32, which is the fourth wavefront per SIMD; an
    // accumulator per sample tile fed by the unmasked blocks, with lane group g keeping tile g, is 7 % slower at either
    // width.)
    u4 a_out[4][HK];
    f4 bias2[HT], bias_out;
    auto load_network = [&](int32_t net) {
        const u4 *__restrict__ wp = (const u4 *)(packed + (int64_t)net * L::HALFS);
#pragma unroll
        for (int b = 0; b < NBLK; ++b) areg[b] = wp[b * KN_WAVE + lane];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int kb = 0; kb < HK; ++kb) a_out[u][kb] = mrow == u ? (areg[L::LS + kb] | areg[L::L5 + kb]) : zero_u4;
        const float *__restrict__ tail = (const float *)(wp + NBLK * KN_WAVE);
#pragma unroll
        for (int t = 0; t < HT; ++t) bias2[t] = *(const f4 *)(tail + 16 * t + 4 * g);
        bias_out = *(const f4 *)(tail + H);
    };

    // Input pipeline.  A sample's inputs sit behind a chain of dependent loads (tile descriptor -> sorted
    // position -> sample index -> [render: packed (ray, k) record -> ray origin and direction]); each level is
    // issued one tile ahead of the next, so a level's operands have arrived by the time the following level
    // needs them: tile t is computed while the last level of tile t+1, the record of t+2, the index of t+3 and
    // the descriptor of t+4 are in flight.
    constexpr bool from_rays = SRC == SRC_RAYS, from_records = SRC == SRC_RECORDS, DIRTAB = SRC == SRC_RAYS;
    auto descriptor = [&](int t) -> KnTile { return tiles[min(t, t_hi - 1)]; };
    auto sorted_pos = [&](const KnTile &d) { return d.start + min(lane, d.len - 1); };
    auto sample_at = [&](const KnTile &d) -> int32_t {
        if constexpr (from_records) return sorted_pos(d);
        else return perm[sorted_pos(d)];
    };
    auto load_record = [&](int32_t i) -> uint32_t {
        if constexpr (from_rays) return src.rec[i];
        else return 0u;
    };
    struct Raw { float a[3], b[3]; int32_t out; }; // eval: point, direction; render: ray origin, ray direction; where the result goes
    auto load_raw = [&](int32_t i, uint32_t r) -> Raw {
        Raw q;
        if constexpr (from_records) {
            const u4 h0 = *(const u4 *)(src.records + 4 * (int64_t)i), h1 = *(const u4 *)(src.records_dir + 4 * (int64_t)i);
#pragma unroll
            for (int c = 0; c < 3; ++c) { q.a[c] = __uint_as_float(h0[c]); q.b[c] = __uint_as_float(h1[c]); }
            q.out = (int32_t)h1[3];
        } else {
            const float *pa = from_rays ? src.rays_o + 3 * (int64_t)(r >> src.kbits) : src.points + 3 * (int64_t)i;
            const float *pb = from_rays ? src.rays_d + 3 * (int64_t)(r >> src.kbits) : src.dirs + 3 * (int64_t)i;
#pragma unroll
            for (int c = 0; c < 3; ++c) { q.a[c] = pa[c]; q.b[c] = pb[c]; }
            q.out = i;
        }
        return q;
    };
    auto finish = [&](const Raw &q, uint32_t r, float &x, float &y, float &z, float &dscale) {
        dscale = 1.0f;
        if constexpr (STRAT) {
            const int32_t k = (int32_t)(r & ((1u << src.kbits) - 1u));
            const uint32_t ray_key = kn_mix32(src.seed_key + (r >> src.kbits));
            const float t0 = kn_lattice_t<true>(src.t_near, src.step, k, ray_key);
            const float t1 = kn_lattice_t<true>(src.t_near, src.step, k + 1, ray_key);
            x = fmaf(t0, q.b[0], q.a[0]);
            y = fmaf(t0, q.b[1], q.a[1]);
            z = fmaf(t0, q.b[2], q.a[2]);
            dscale = (t1 - t0) / src.step;
        } else if constexpr (from_rays)
            kn_lattice_point(q.a[0], q.a[1], q.a[2], q.b[0], q.b[1], q.b[2], src.t_near, src.step,
                             (int32_t)(r & ((1u << src.kbits) - 1u)), x, y, z);
        else { x = q.a[0]; y = q.a[1]; z = q.a[2]; }
    };
    KnTile dsc0 = descriptor(t_lo), dsc1 = descriptor(t_lo + 1), dsc2 = descriptor(t_lo + 2), dsc3 = descriptor(t_lo + 3);
    int32_t idx0 = sample_at(dsc0), idx1 = sample_at(dsc1), idx2 = sample_at(dsc2);
    // Width 32: the first network's weights are requested here, behind the sample indices and in front of the two levels
    // that depend on them, so that they arrive while those levels are waited for, not after them.  (Width 64 has no
    // register to spare for the overlap: there the same move costs 9 %.)
    int32_t net_cur = -1;
    if constexpr (H == 32) {
        load_network(dsc0.net);
        net_cur = dsc0.net;
    }
    uint32_t rec0 = load_record(idx0), rec1 = load_record(idx1);
    Raw raw0 = load_raw(idx0, rec0);
    // Results of a tile are written in the next iteration, between its wait for the loads issued one iteration
    // earlier and the loads it issues itself: the memory counter is in order, so a store must be older than
    // every load that is going to be waited for, or the wait covers the store's full round trip as well.
    f4 pend = zero4;
    int32_t pend_idx = -1;
    auto write_out = [&]() {
        if (pend_idx >= 0) {
            if constexpr (SRC != SRC_POINTS) { // (the staging array of the render / of the re-ordered evaluation)
                *(f4 *)(src.out4 + 4 * (int64_t)pend_idx) = pend;
            } else {
                sigma[pend_idx] = pend[3];
                float *o = rgb + 3 * (int64_t)pend_idx;
                o[0] = pend[0];
                o[1] = pend[1];
                o[2] = pend[2];
            }
        }
    };

    // The hardware issues from the oldest ready wavefront first, so the wavefronts that share a SIMD would finish
    // one after the other and the last one would run alone; a wavefront lowers its own issue priority as it gets
    // through its range, which lets the ones behind catch up and ends all of them together.  The steps are at a half,
    // a quarter and an eighth of the range to go: what the wavefronts drift apart after the last step is what they end
    // apart (time stamps per tile: with steps at the quarters of the range the ends of a SIMD's wavefronts (three at the time) lay
    // 9 us apart in a 58 us launch, with these 6.5).
    const int n_t = t_hi - t_lo;
    const int drop_to_2 = t_hi - (n_t >> 1), drop_to_1 = t_hi - (n_t >> 2), drop_to_0 = t_hi - (n_t >> 3);
    __builtin_amdgcn_s_setprio(3);

    // (render) gamma(d) fragment of the first sample tile of the tile that comes next: requested at the end of the
    // tile before it.  (Fragments are addressed with a 32-bit byte offset from the table's start, 64 bytes per ray: one
    // instruction instead of four per gather; kn_render limits the number of rays to 2^26.)
    u4 Bd_first = zero_u4;
    if constexpr (DIRTAB) Bd_first = *(const u4 *)((const char *)src.dir_table + ((uint32_t)__shfl((int)(rec0 >> src.kbits), n, KN_WAVE) * 64u + (uint32_t)g * 16u));
    for (int t = t_lo; t < t_hi; ++t) {
        if (t == drop_to_2) __builtin_amdgcn_s_setprio(2); // (uniform; the lowest wins where steps coincide)
        if (t == drop_to_1) __builtin_amdgcn_s_setprio(1);
        if (t == drop_to_0) __builtin_amdgcn_s_setprio(0);
        const KnTile tl = dsc0;
        if (tl.net != net_cur) { // uniform
            load_network(tl.net);
            net_cur = tl.net;
        }
        const bool active = lane < tl.len;
        const int32_t idx = raw0.out;
        float nx, ny, nz, dscale;
        finish(raw0, rec0, nx, ny, nz, dscale);
        const float ndx = raw0.b[0], ndy = raw0.b[1], ndz = raw0.b[2];
        const uint32_t ray_no = rec0 >> src.kbits; // (render)
        write_out(); // after the loads of the last iteration have been waited for, before new ones are issued
        // next levels for the following tiles (their operands were loaded one iteration ago)
        raw0 = load_raw(idx1, rec1);
        rec0 = rec1;
        rec1 = load_record(idx2);
        idx0 = idx1;
        idx1 = idx2;
        idx2 = sample_at(dsc3);
        dsc0 = dsc1;
        dsc1 = dsc2;
        dsc2 = dsc3;
        {
            // lane groups 0..2 encode one axis each at frequencies 0..7 (restarts at 2^0, 2^2, 2^4) and the
            // direction at 0..3; group 3 encodes frequencies 8, 9 of all three axes (restarts at 2^8)
            const float p3[3] = {nx, ny, nz}, d3[3] = {ndx, ndy, ndz};
            // fourth word: the direction component in revolutions, or (DIRTAB) the ray's number for every lane group
            const float ray_bits = __builtin_bit_cast(float, ray_no);
#pragma unroll
            for (int a = 0; a < 3; ++a)
                stage[wave][a][0][lane] = (f4){p3[a] * INV_2PI, p3[a] * (4.0f * INV_2PI), p3[a] * (16.0f * INV_2PI),
                                               DIRTAB ? ray_bits : d3[a] * INV_2PI};
            stage[wave][3][0][lane] = (f4){nx * (256.0f * INV_2PI), ny * (256.0f * INV_2PI), nz * (256.0f * INV_2PI),
                                           DIRTAB ? ray_bits : 0.0f};
            const u4 ident = {pk<BF>(nx, ny), pk<BF>(nz, 1.0f), DIRTAB ? 0u : pk<BF>(ndx, ndy), DIRTAB ? 0u : pk<BF>(ndz, 1.0f)};
            stage[wave][3][1][lane] = __builtin_bit_cast(f4, ident);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        f4 out_sig = bias_out, out_col = bias_out;
        u4 Bd_ahead = Bd_first;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            { // all four sample tiles are always computed: straight-line code lets the scheduler interleave them
                const f4 ang = stage[wave][g][0][16 * u + n];
                const u4 ident = __builtin_bit_cast(u4, stage[wave][g][1][16 * u + n]); // meaningful in group 3 only
                u4 Bx[2];
                encode_position<BF, WRAP>(ang, ident, m3, Bx);
                u4 Bd;
                if constexpr (DIRTAB) {
                    // The fragment of sample tile u was requested a whole sample tile ago; the one of tile u + 1 is requested
                    // here (the ray's number travels in the fourth word of the staged angles), and nothing may be
                    // scheduled across that point: left to itself the compiler puts such a gather a few instructions in
                    // front of its use, and the wavefront then waits for a round trip to the L2 per sample tile.
                    Bd = Bd_ahead;
                    if (u < 3) {
                        const float ray_word = stage[wave][g][0][16 * (u + 1) + n][3];
                        Bd_ahead = *(const u4 *)((const char *)src.dir_table + (__float_as_uint(ray_word) * 64u + (uint32_t)g * 16u));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
                    Bd = encode_direction<BF>(ang[3], ident, m3);
                }
                f4 acc[HT];
                u4 Bh[HK];
                // layer 1: gamma(x) -> H, ReLU (bias through the constant-1 slot)
#pragma unroll
                for (int t = 0; t < HT; ++t) {
                    acc[t] = mfma<BF>(A(L::L1 + 2 * t), Bx[0], zero4);
                    acc[t] = mfma<BF>(A(L::L1 + 2 * t + 1), Bx[1], acc[t]);
                }
                pack_acts<H, BF, true>(acc, Bh);
                // layer 2: H -> H, ReLU
#pragma unroll
                for (int t = 0; t < HT; ++t) {
                    acc[t] = bias2[t];
#pragma unroll
                    for (int kb = 0; kb < HK; ++kb) acc[t] = mfma<BF>(A(L::L2 + t * HK + kb), Bh[kb], acc[t]);
                }
                pack_acts<H, BF, true>(acc, Bh);
                // layer 3: the density (row 4u+3 of the shared tile); its feature vector is folded into layer 4
#pragma unroll
                for (int kb = 0; kb < HK; ++kb) out_sig = mfma<BF>(a_out[u][kb], Bh[kb], out_sig);
                // layer 4: [second hidden vector through the folded feature layer, gamma(d)] -> H, ReLU (bias through
                // the constant-1 slot)
#pragma unroll
                for (int t = 0; t < HT; ++t) {
                    acc[t] = mfma<BF>(A(L::L4 + t * (HK + 1) + HK), Bd, zero4);
#pragma unroll
                    for (int kb = 0; kb < HK; ++kb) acc[t] = mfma<BF>(A(L::L4 + t * (HK + 1) + kb), Bh[kb], acc[t]);
                }
                pack_acts<H, BF, true>(acc, Bh);
                // layer 5: H -> colour rows 4u+0..2 of the shared tile
#pragma unroll
                for (int kb = 0; kb < HK; ++kb) out_col = mfma<BF>(a_out[u][kb], Bh[kb], out_col);
            }
        }
        if constexpr (DIRTAB) { // first direction fragment of the next tile: its sample n's ray is known to lane n
            const uint32_t ray_next = (uint32_t)__shfl((int)(rec0 >> src.kbits), n, KN_WAVE);
            Bd_first = *(const u4 *)((const char *)src.dir_table + (ray_next * 64u + (uint32_t)g * 16u));
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_wave_barrier(); // staging buffer is rewritten by the next iteration
        // The next descriptor comes through the scalar cache, which shares its counter with LDS: fetched here,
        // behind the last LDS read of the iteration, its latency is not part of any wait for staged data.
        dsc3 = descriptor(t + 4);

        // output activations; the store itself is issued at the top of the next iteration (see write_out).
        // Lane l holds sample l of the 64.
        {
            const f4 out = (f4){out_col[0], out_col[1], out_col[2], out_sig[3]};
            float sg = fmaxf(out[3], 0.0f);
            if constexpr (STRAT) sg *= dscale;
            float col[3];
#pragma unroll
            for (int c = 0; c < 3; ++c)
                col[c] = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * out[c]));
            pend = (f4){col[0], col[1], col[2], sg};
            pend_idx = active ? idx : -1;
        }
    }
    write_out();
}


// Density only, for occupancy extraction (Sec. 3.4): layers 1 and 2 and the density row of layer 3 at the probe
// points of one network cell's voxels, which are generated in the kernel.  Same formulation as k_mlp_mfma.
template <int H, bool BF, int WAVES, bool WRAP>
__global__ void __launch_bounds__(WAVES *KN_WAVE) __attribute__((amdgpu_waves_per_eu(H == 32 ? 4 : 3, H == 32 ? 4 : 3)))
    k_probe_mfma(const uint16_t *__restrict__ packed, KnProbeJob job)
{
    using L = Lay<H>;
    constexpr int HT = L::HT, HK = L::HK;
    __shared__ f4 stage[WAVES][4][2][KN_WAVE]; // as in k_mlp_mfma, without the direction
    const int wave = threadIdx.x / KN_WAVE, lane = threadIdx.x & (KN_WAVE - 1);
    const int n = lane & 15, g = lane >> 4;
    const unsigned m3 = (g == 3) ? 0xffffffffu : 0u;
    const int mrow = n >> 2;
    const f4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    const u4 zero_u4 = {0u, 0u, 0u, 0u};

    const int32_t cell = blockIdx.x / job.parts, part = blockIdx.x - cell * job.parts;
    const KnProbeBox box = kn_probe_box(job, cell);
    if (box.points == 0) return;
    const int shares = job.parts * WAVES, share = part * WAVES + wave;
    const int t_lo = __builtin_amdgcn_readfirstlane((int)((int64_t)share * box.tiles / shares));
    const int t_hi = __builtin_amdgcn_readfirstlane((int)((int64_t)(share + 1) * box.tiles / shares));
    if (t_lo >= t_hi) return;

    u4 a1[2 * HT], a2[HT * HK], a_sig[HK];
    // (width 32: the density block restricted to the rows of sample tile u, made once per network; at width 64 the copies
    // would cost the third wavefront per SIMD, and the block is masked where it is used)
    constexpr bool MASKED_COPIES = H == 32;
    u4 a_sig_of[MASKED_COPIES ? 4 : 1][HK];
    f4 bias2[HT];
    float bias_sig = 0.0f;
    auto load_network = [&](int32_t net) {
        const u4 *__restrict__ wp = (const u4 *)(packed + (int64_t)net * L::HALFS);
#pragma unroll
        for (int b = 0; b < 2 * HT; ++b) a1[b] = wp[(L::L1 + b) * KN_WAVE + lane];
#pragma unroll
        for (int b = 0; b < HT * HK; ++b) a2[b] = wp[(L::L2 + b) * KN_WAVE + lane];
#pragma unroll
        for (int kb = 0; kb < HK; ++kb) a_sig[kb] = wp[(L::LS + kb) * KN_WAVE + lane];
        if constexpr (MASKED_COPIES) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int kb = 0; kb < HK; ++kb) a_sig_of[u][kb] = mrow == u ? a_sig[kb] : zero_u4;
        }
        const float *__restrict__ tail = (const float *)(wp + L::NBLK * KN_WAVE);
#pragma unroll
        for (int t = 0; t < HT; ++t) bias2[t] = *(const f4 *)(tail + 16 * t + 4 * g);
        bias_sig = tail[H + 3];
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
        {
            const float p3[3] = {x, y, z};
#pragma unroll
            for (int a = 0; a < 3; ++a)
                stage[wave][a][0][lane] = (f4){p3[a] * INV_2PI, p3[a] * (4.0f * INV_2PI), p3[a] * (16.0f * INV_2PI), 0.0f};
            stage[wave][3][0][lane] = (f4){x * (256.0f * INV_2PI), y * (256.0f * INV_2PI), z * (256.0f * INV_2PI), 0.0f};
            const u4 ident = {pk<BF>(x, y), pk<BF>(z, 1.0f), 0u, 0u};
            stage[wave][3][1][lane] = __builtin_bit_cast(f4, ident);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // One pass per network met in the tile: a single pass when the grids nest, a second one for the probes
        // of voxels that reach into a neighbouring cell otherwise.
        for (;;) {
            const unsigned long long pending = __ballot(todo);
            if (pending == 0ull) break;
            const int32_t nsel = __builtin_amdgcn_readlane(net, (int)__builtin_ctzll(pending));
            if (nsel != net_loaded) {
                load_network(nsel);
                net_loaded = nsel;
            }
            f4 out = {0.0f, 0.0f, 0.0f, bias_sig};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const f4 ang = stage[wave][g][0][16 * u + n];
                const u4 ident = __builtin_bit_cast(u4, stage[wave][g][1][16 * u + n]);
                u4 Bx[2];
                encode_position<BF, WRAP>(ang, ident, m3, Bx);
                f4 acc[HT];
                u4 Bh[HK];
#pragma unroll
                for (int t2 = 0; t2 < HT; ++t2) {
                    acc[t2] = mfma<BF>(a1[2 * t2], Bx[0], zero4);
                    acc[t2] = mfma<BF>(a1[2 * t2 + 1], Bx[1], acc[t2]);
                }
                pack_acts<H, BF, true>(acc, Bh);
#pragma unroll
                for (int t2 = 0; t2 < HT; ++t2) {
                    acc[t2] = bias2[t2];
#pragma unroll
                    for (int kb = 0; kb < HK; ++kb) acc[t2] = mfma<BF>(a2[t2 * HK + kb], Bh[kb], acc[t2]);
                }
                pack_acts<H, BF, true>(acc, Bh);
#pragma unroll
                for (int kb = 0; kb < HK; ++kb) {
                    if constexpr (MASKED_COPIES) out = mfma<BF>(a_sig_of[u][kb], Bh[kb], out);
                    else out = mfma<BF>(mrow == u ? a_sig[kb] : zero_u4, Bh[kb], out);
                }
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


// ---------------------------------------------------------------------------------------------
// Layer-at-a-time evaluation: the variable-batch grouped matrix products of Sec. 3.5 (one product per network and
// layer, batch sizes that differ per network), which the paper uses where the fused kernel does not apply.  Here it
// is the fused kernel cut at the layer boundaries, one launch per layer, with the same operands and the same
// order of operations, so both give the same bits; it exists as the comparison point for the fusion.
// Activations travel through HBM: row-major per sorted position, 16-bit, columns in slot order, so that the 16 bytes
// at column 32 kb + 8 g of a row are the B operand of lane group g for input block kb.
struct KnLayerBufs {
    uint16_t *x0; // M x 64: gamma(x)
    uint16_t *dd; // M x 32: gamma(d)
    uint16_t *ha; // M x H
    uint16_t *hb; // M x H
};

template <bool BF, int WAVES, bool WRAP>
__global__ void __launch_bounds__(WAVES *KN_WAVE)
    k_layer_encode(KnSampleSrc src, const int32_t *__restrict__ perm, const KnTile *__restrict__ tiles,
                   const int32_t *__restrict__ n_tiles, KnLayerBufs buf)
{
    __shared__ f4 stage[WAVES][4][2][KN_WAVE];
    const int wave = threadIdx.x / KN_WAVE, lane = threadIdx.x & (KN_WAVE - 1);
    const int n = lane & 15, g = lane >> 4;
    const unsigned m3 = (g == 3) ? 0xffffffffu : 0u;
    const int total_tiles = *n_tiles;
    for (int t = blockIdx.x * WAVES + wave; t < total_tiles; t += gridDim.x * WAVES) {
        const KnTile tl = tiles[t];
        const int32_t idx = perm[tl.start + min(lane, tl.len - 1)];
        float x, y, z, dx, dy, dz;
        float dscale; // (explicit points: always 1)
        int32_t out_idx; // (= idx: the layer-at-a-time path sorts indices)
        kn_load_sample(src, idx, x, y, z, dx, dy, dz, dscale, out_idx);
        {
            const float p3[3] = {x, y, z}, d3[3] = {dx, dy, dz};
#pragma unroll
            for (int a = 0; a < 3; ++a)
                stage[wave][a][0][lane] = (f4){p3[a] * INV_2PI, p3[a] * (4.0f * INV_2PI), p3[a] * (16.0f * INV_2PI), d3[a] * INV_2PI};
            stage[wave][3][0][lane] = (f4){x * (256.0f * INV_2PI), y * (256.0f * INV_2PI), z * (256.0f * INV_2PI), 0.0f};
            const u4 ident = {pk<BF>(x, y), pk<BF>(z, 1.0f), pk<BF>(dx, dy), pk<BF>(dz, 1.0f)};
            stage[wave][3][1][lane] = __builtin_bit_cast(f4, ident);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const f4 ang = stage[wave][g][0][16 * u + n];
            const u4 ident = __builtin_bit_cast(u4, stage[wave][g][1][16 * u + n]);
            u4 Bx[2];
            encode_position<BF, WRAP>(ang, ident, m3, Bx);
            const u4 Bd = encode_direction<BF>(ang[3], ident, m3);
            if (16 * u + n < tl.len) {
                const int64_t row = tl.start + 16 * u + n;
                *(u4 *)(buf.x0 + row * 64 + 8 * g) = Bx[0];
                *(u4 *)(buf.x0 + row * 64 + 32 + 8 * g) = Bx[1];
                *(u4 *)(buf.dd + row * 32 + 8 * g) = Bd;
            }
        }
        __builtin_amdgcn_wave_barrier(); // the staging buffer is rewritten by the next iteration
    }
}

// LAYER 1..5 of Sec. 3.2: 1: gamma(x) -> ha; 2: ha -> hb; 3: hb -> the density (its feature vector is folded into layer
// 4, as in the fused kernel); 4: [hb, gamma(d)] -> ha; 5: ha -> colour.  Tiles are dealt out as in k_mlp_mfma (a
// contiguous range per wavefront, weights re-fetched when the network changes).
template <int H, bool BF, int WAVES, int LAYER>
__global__ void __launch_bounds__(WAVES *KN_WAVE)
    k_layer(const uint16_t *__restrict__ packed, const int32_t *__restrict__ perm, const KnTile *__restrict__ tiles,
            const int32_t *__restrict__ n_tiles, KnLayerBufs buf, float *__restrict__ sigma, float *__restrict__ rgb)
{
    using L = Lay<H>;
    constexpr int HT = L::HT, HK = L::HK;
    constexpr int NB = LAYER == 1 ? 2 : (LAYER == 4 ? HK + 1 : HK); // input blocks
    constexpr int NT = (LAYER == 3 || LAYER == 5) ? 0 : HT;          // output tiles of the layer proper
    constexpr int W0 = LAYER == 1 ? L::L1 : (LAYER == 2 ? L::L2 : L::L4);
    constexpr bool HEAD = LAYER == 3 || LAYER == 5;                  // a density / colour head
    constexpr int WH = LAYER == 3 ? L::LS : L::L5;
    const uint16_t *__restrict__ in = LAYER == 1 ? buf.x0 : ((LAYER == 2 || LAYER == 5) ? buf.ha : buf.hb);
    uint16_t *__restrict__ out = (LAYER == 1 || LAYER == 4) ? buf.ha : buf.hb;
    constexpr int IN_COLS = LAYER == 1 ? 64 : H;

    const int wave = threadIdx.x / KN_WAVE, lane = threadIdx.x & (KN_WAVE - 1);
    const int n = lane & 15, g = lane >> 4;
    const f4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    const int total_tiles = *n_tiles;
    const int total_waves = gridDim.x * WAVES;
    const int wid = __builtin_amdgcn_readfirstlane(blockIdx.x * WAVES + wave);
    const int t_lo = __builtin_amdgcn_readfirstlane((int)((int64_t)wid * total_tiles / total_waves));
    const int t_hi = __builtin_amdgcn_readfirstlane((int)((int64_t)(wid + 1) * total_tiles / total_waves));
    if (t_lo >= t_hi) return;

    u4 aw[NT * NB > 0 ? NT * NB : 1], ah[HEAD ? HK : 1];
    f4 bias[NT > 0 ? NT : 1], bias_head = zero4;
    auto load_network = [&](int32_t net) {
        const u4 *__restrict__ wp = (const u4 *)(packed + (int64_t)net * L::HALFS);
#pragma unroll
        for (int b = 0; b < NT * NB; ++b) aw[b] = wp[(W0 + b) * KN_WAVE + lane];
        if constexpr (HEAD) {
#pragma unroll
            for (int kb = 0; kb < HK; ++kb) ah[kb] = wp[(WH + kb) * KN_WAVE + lane];
        }
        const float *__restrict__ tail = (const float *)(wp + L::NBLK * KN_WAVE);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if constexpr (LAYER == 2) bias[t] = *(const f4 *)(tail + 16 * t + 4 * g);
            else bias[t] = zero4; // layers 1 and 4: the bias rides in a constant-1 input slot
        }
        if constexpr (HEAD) bias_head = *(const f4 *)(tail + H); // (b5, density bias)
    };
    int32_t net_cur = -1;
    for (int t = t_lo; t < t_hi; ++t) {
        const KnTile tl = tiles[t];
        if (tl.net != net_cur) { // uniform
            load_network(tl.net);
            net_cur = tl.net;
        }
        f4 heads[4] = {bias_head, bias_head, bias_head, bias_head};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t row = tl.start + min(16 * u + n, tl.len - 1);
            u4 B[NB];
#pragma unroll
            for (int kb = 0; kb < NB; ++kb) {
                if (LAYER == 4 && kb == HK) B[kb] = *(const u4 *)(buf.dd + row * 32 + 8 * g);
                else B[kb] = *(const u4 *)(in + row * IN_COLS + 32 * kb + 8 * g);
            }
            if constexpr (NT > 0) {
                f4 acc[NT];
#pragma unroll
                for (int t2 = 0; t2 < NT; ++t2) {
                    if constexpr (LAYER == 4) { // same order as the fused kernel: gamma(d) block first
                        acc[t2] = mfma<BF>(aw[t2 * NB + HK], B[HK], zero4);
#pragma unroll
                        for (int kb = 0; kb < HK; ++kb) acc[t2] = mfma<BF>(aw[t2 * NB + kb], B[kb], acc[t2]);
                    } else {
                        acc[t2] = bias[t2];
#pragma unroll
                        for (int kb = 0; kb < NB; ++kb) acc[t2] = mfma<BF>(aw[t2 * NB + kb], B[kb], acc[t2]);
                    }
                }
                u4 Bh[HK];
                pack_acts<H, BF, true>(acc, Bh);
                if (16 * u + n < tl.len) {
                    const int64_t orow = tl.start + 16 * u + n;
#pragma unroll
                    for (int kb = 0; kb < HK; ++kb) *(u4 *)(out + orow * H + 32 * kb + 8 * g) = Bh[kb];
                }
            }
            if constexpr (HEAD) {
#pragma unroll
                for (int kb = 0; kb < HK; ++kb) heads[u] = mfma<BF>(ah[kb], B[kb], heads[u]);
            }
        }
        if constexpr (HEAD) {
            // the head blocks repeat their rows with period four: lane group g keeps tile g, lane l sample l
            const f4 o = g == 0 ? heads[0] : (g == 1 ? heads[1] : (g == 2 ? heads[2] : heads[3]));
            if (lane < tl.len) {
                const int32_t idx = perm[tl.start + lane];
                if constexpr (LAYER == 3) {
                    sigma[idx] = fmaxf(o[3], 0.0f);
                } else {
#pragma unroll
                    for (int c = 0; c < 3; ++c)
                        rgb[3 * (int64_t)idx + c] = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * o[c]));
                }
            }
        }
    }
}

template <int H, bool BF, int WAVES>
int launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t max_tiles, float *sigma,
           float *rgb, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    int64_t blocks = kn_div_up(max_tiles, WAVES);
    // one workgroup of 4 wavefronts per compute unit and resident wavefront (H = 32: four per SIMD, H = 64: two)
    const int fill = 256 * (H == 32 ? 4 : 2);
    if (blocks > fill) blocks = fill;
    // positions are only ever evaluated inside the grid's box: its largest coordinate bounds the encoding's
    // largest argument, 2^8 |p| / (2 pi) revolutions at the highest restart frequency
    float reach = 0.0f;
    for (int a = 0; a < 3; ++a)
        reach = fmaxf(reach, fmaxf(fabsf(sc->desc.aabb_min[a]), fabsf(sc->desc.aabb_max[a])));
    const bool wrap = !(reach * (256.0f * INV_2PI) < 250.0f);
    const bool rays = src.points == nullptr && src.records == nullptr;
    const bool strat = src.strat != 0 && rays;
    if (rays && !src.dir_table) return KN_E_INVALID_ARG;
    if ((src.out4 != nullptr) != (rays || src.records != nullptr)) return KN_E_INVALID_ARG; // where the results go is part of the kernel variant
    // render: the ray's encoded direction comes from the table, midpoint or stratified lattice; else explicit points,
    // through the index list or re-ordered
    auto kernel = src.records ? (wrap ? k_mlp_mfma<H, BF, WAVES, true, false, SRC_RECORDS> : k_mlp_mfma<H, BF, WAVES, false, false, SRC_RECORDS>)
                  : !rays     ? (wrap ? k_mlp_mfma<H, BF, WAVES, true, false, SRC_POINTS> : k_mlp_mfma<H, BF, WAVES, false, false, SRC_POINTS>)
                  : wrap      ? (strat ? k_mlp_mfma<H, BF, WAVES, true, true, SRC_RAYS> : k_mlp_mfma<H, BF, WAVES, true, false, SRC_RAYS>)
                              : (strat ? k_mlp_mfma<H, BF, WAVES, false, true, SRC_RAYS> : k_mlp_mfma<H, BF, WAVES, false, false, SRC_RAYS>);
    if (ev_start && ev_stop)
        hipExtLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(WAVES * KN_WAVE), 0, st, ev_start, ev_stop, 0,
                              (const uint16_t *)sc->packed_w, src, b.perm, b.tiles, b.n_tiles, sigma, rgb);
    else
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(WAVES * KN_WAVE), 0, st, (const uint16_t *)sc->packed_w, src, b.perm,
                           b.tiles, b.n_tiles, sigma, rgb);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

} // namespace

int kn_mlp_mfma_tile_len(const kn_scene *) { return MLP_TILE_LEN; }

// bytes of the slot-order weights of N networks of width H (0: no kernel for that width)
// (+ one status word behind the last network, for kn_mlp_pack_weights)
int64_t kn_mlp_packed_bytes(int32_t H, int64_t N)
{
    if (H != 32 && H != 64) return 0;
    return kn_align_up((int64_t)(H == 32 ? Lay<32>::HALFS : Lay<64>::HALFS) * 2 * N, 256) + 256;
}

// fills sc->packed_w (kn_mlp_packed_bytes bytes, assigned by the caller) and waits for it.  KN_E_UNSUPPORTED when the
// product of a network's feature layer and layer 4 leaves the range of the scene's 16-bit type (fp16 weights whose
// products sum beyond 65504: the folded layer cannot carry them).
int kn_mlp_pack_weights(kn_scene *sc, hipStream_t st)
{
    const int H = sc->desc.hidden;
    const bool bf = sc->desc.wdtype == KN_BF16;
    if (!sc->packed_w || (H != 32 && H != 64)) return KN_E_INVALID_ARG;
    const int64_t halfs = H == 32 ? Lay<32>::HALFS : Lay<64>::HALFS;
    const int64_t per = H == 32 ? Lay<32>::NBLK * 512 + Lay<32>::TAIL_FLOATS : Lay<64>::NBLK * 512 + Lay<64>::TAIL_FLOATS;
    sc->packed_halfs_per_net = halfs;
    const int64_t total = per * sc->N;
    const int64_t blocks = kn_div_up(total, 256);
    if (blocks > 0x7fffffffLL) return KN_E_UNSUPPORTED;
    const uint16_t *w = (const uint16_t *)sc->desc.weights;
    int32_t *flag = (int32_t *)((char *)sc->packed_w + kn_align_up(halfs * 2 * sc->N, 256));
    hipLaunchKernelGGL(k_clear_flag, dim3(1), dim3(1), 0, st, flag);
    KN_CHECK_LAUNCH();
    if (H == 32)
        hipLaunchKernelGGL(k_pack_weights<32>, dim3((unsigned)blocks), dim3(256), 0, st, w, sc->P, sc->N, bf,
                           (uint16_t *)sc->packed_w, flag);
    else
        hipLaunchKernelGGL(k_pack_weights<64>, dim3((unsigned)blocks), dim3(256), 0, st, w, sc->P, sc->N, bf,
                           (uint16_t *)sc->packed_w, flag);
    KN_CHECK_LAUNCH();
    int32_t overflow = 0;
    KN_HIP(hipMemcpyAsync(&overflow, flag, sizeof(overflow), hipMemcpyDeviceToHost, st));
    KN_HIP(hipStreamSynchronize(st));
    return overflow ? KN_E_UNSUPPORTED : KN_OK;
}

int kn_probe_mfma_launch(const kn_scene *sc, hipStream_t st, const KnProbeJob &job)
{
    const bool bf = sc->desc.wdtype == KN_BF16;
    const int H = sc->desc.hidden;
    float reach = 0.0f;
    for (int a = 0; a < 3; ++a)
        reach = fmaxf(reach, fmaxf(fabsf(sc->desc.aabb_min[a]), fabsf(sc->desc.aabb_max[a])));
    const bool wrap = !(reach * (256.0f * INV_2PI) < 250.0f);
    const dim3 grid((unsigned)(sc->cells * job.parts)), block(MLP_WAVES * KN_WAVE);
    const uint16_t *w = (const uint16_t *)sc->packed_w;
#define KN_PROBE_CASE(HH, BB, WW)                                                                          \
    if (H == HH && bf == BB && wrap == WW)                                                                  \
        hipLaunchKernelGGL((k_probe_mfma<HH, BB, MLP_WAVES, WW>), grid, block, 0, st, w, job);
    KN_PROBE_CASE(32, false, false)
    KN_PROBE_CASE(32, false, true)
    KN_PROBE_CASE(32, true, false)
    KN_PROBE_CASE(32, true, true)
    KN_PROBE_CASE(64, false, false)
    KN_PROBE_CASE(64, false, true)
    KN_PROBE_CASE(64, true, false)
    KN_PROBE_CASE(64, true, true)
#undef KN_PROBE_CASE
    if (H != 32 && H != 64) return KN_E_UNSUPPORTED;
    KN_CHECK_LAUNCH();
    return KN_OK;
}

int64_t kn_layered_act_bytes(const kn_scene *sc, int64_t M)
{
    const int64_t m = M > 0 ? M : 1;
    return kn_align_up(m * 64 * 2, 256) + kn_align_up(m * 32 * 2, 256) + 2 * kn_align_up(m * sc->desc.hidden * 2, 256);
}

template <int H, bool BF>
static int layered_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t max_tiles,
                          bool wrap, const KnLayerBufs &buf, float *sigma, float *rgb)
{
    constexpr int W = MLP_WAVES;
    int64_t blocks = kn_div_up(max_tiles, W);
    if (blocks > 256 * 4) blocks = 256 * 4;
    const dim3 grid((unsigned)blocks), block(W * KN_WAVE);
    const uint16_t *w = (const uint16_t *)sc->packed_w;
    if (wrap)
        hipLaunchKernelGGL((k_layer_encode<BF, W, true>), grid, block, 0, st, src, b.perm, b.tiles, b.n_tiles, buf);
    else
        hipLaunchKernelGGL((k_layer_encode<BF, W, false>), grid, block, 0, st, src, b.perm, b.tiles, b.n_tiles, buf);
    KN_CHECK_LAUNCH();
    hipLaunchKernelGGL((k_layer<H, BF, W, 1>), grid, block, 0, st, w, b.perm, b.tiles, b.n_tiles, buf, sigma, rgb);
    KN_CHECK_LAUNCH();
    hipLaunchKernelGGL((k_layer<H, BF, W, 2>), grid, block, 0, st, w, b.perm, b.tiles, b.n_tiles, buf, sigma, rgb);
    KN_CHECK_LAUNCH();
    hipLaunchKernelGGL((k_layer<H, BF, W, 3>), grid, block, 0, st, w, b.perm, b.tiles, b.n_tiles, buf, sigma, rgb);
    KN_CHECK_LAUNCH();
    hipLaunchKernelGGL((k_layer<H, BF, W, 4>), grid, block, 0, st, w, b.perm, b.tiles, b.n_tiles, buf, sigma, rgb);
    KN_CHECK_LAUNCH();
    hipLaunchKernelGGL((k_layer<H, BF, W, 5>), grid, block, 0, st, w, b.perm, b.tiles, b.n_tiles, buf, sigma, rgb);
    KN_CHECK_LAUNCH();
    return KN_OK;
}

// `acts`: kn_layered_act_bytes(sc, M) bytes of device memory, 256-byte aligned
int kn_mlp_layered_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t M,
                          int64_t max_tiles, void *acts, float *sigma, float *rgb)
{
    if (max_tiles <= 0 || M <= 0) return KN_OK;
    const int H = sc->desc.hidden;
    if (sc->desc.wdtype == KN_F32 || (H != 32 && H != 64)) return KN_E_UNSUPPORTED;
    KnCarver c(acts, kn_layered_act_bytes(sc, M));
    KnLayerBufs buf;
    buf.x0 = c.carve<uint16_t>(M * 64);
    buf.dd = c.carve<uint16_t>(M * 32);
    buf.ha = c.carve<uint16_t>(M * H);
    buf.hb = c.carve<uint16_t>(M * H);
    if (!c.ok()) return KN_E_WORKSPACE;
    float reach = 0.0f;
    for (int a = 0; a < 3; ++a)
        reach = fmaxf(reach, fmaxf(fabsf(sc->desc.aabb_min[a]), fabsf(sc->desc.aabb_max[a])));
    const bool wrap = !(reach * (256.0f * INV_2PI) < 250.0f);
    const bool bf = sc->desc.wdtype == KN_BF16;
    if (H == 32)
        return bf ? layered_launch<32, true>(sc, st, src, b, max_tiles, wrap, buf, sigma, rgb)
                  : layered_launch<32, false>(sc, st, src, b, max_tiles, wrap, buf, sigma, rgb);
    return bf ? layered_launch<64, true>(sc, st, src, b, max_tiles, wrap, buf, sigma, rgb)
              : layered_launch<64, false>(sc, st, src, b, max_tiles, wrap, buf, sigma, rgb);
}

int kn_mlp_mfma_launch(const kn_scene *sc, hipStream_t st, const KnSampleSrc &src, const KnBucketOut &b, int64_t max_tiles,
                       float *sigma, float *rgb, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (max_tiles <= 0) return KN_OK;
    const bool bf = sc->desc.wdtype == KN_BF16;
    if (sc->desc.hidden == 32)
        return bf ? launch<32, true, MLP_WAVES>(sc, st, src, b, max_tiles, sigma, rgb, ev_start, ev_stop)
                  : launch<32, false, MLP_WAVES>(sc, st, src, b, max_tiles, sigma, rgb, ev_start, ev_stop);
    if (sc->desc.hidden == 64)
        return bf ? launch<64, true, MLP_WAVES>(sc, st, src, b, max_tiles, sigma, rgb, ev_start, ev_stop)
                  : launch<64, false, MLP_WAVES>(sc, st, src, b, max_tiles, sigma, rgb, ev_start, ev_stop);
    return KN_E_UNSUPPORTED;
}
