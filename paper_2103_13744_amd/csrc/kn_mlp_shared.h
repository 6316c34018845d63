// Device helpers shared by the grouped-MLP kernels.
#pragma once

#include "kn_common.h"

// Fetch position and direction of sorted-list entry `idx`: from the re-ordered records (then idx is the position in
// the sorted list itself), from explicit arrays, or by rebuilding the lattice point of a render sample from its
// packed (ray, k) record with the same fused multiply-adds the marching kernel used.  dscale: the factor on the
// density that leaves the kernel (delta_k / step with stratified sampling, else 1).  out: the index the sample's
// result is written to.
__device__ __forceinline__ void kn_load_sample(const KnSampleSrc &s, int32_t idx, float &x, float &y, float &z,
                                               float &dx, float &dy, float &dz, float &dscale, int32_t &out)
{
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    dscale = 1.0f;
    out = idx;
    if (s.records) {
        const u4 h0 = *(const u4 *)(s.records + 4 * (int64_t)idx), h1 = *(const u4 *)(s.records_dir + 4 * (int64_t)idx);
        x = __uint_as_float(h0[0]); y = __uint_as_float(h0[1]); z = __uint_as_float(h0[2]);
        dx = __uint_as_float(h1[0]); dy = __uint_as_float(h1[1]); dz = __uint_as_float(h1[2]);
        out = (int32_t)h1[3];
    } else if (s.points) {
        const float *p = s.points + 3 * (int64_t)idx;
        const float *d = s.dirs + 3 * (int64_t)idx;
        x = p[0]; y = p[1]; z = p[2];
        dx = d[0]; dy = d[1]; dz = d[2];
    } else {
        const uint32_t r = s.rec[idx];
        const uint32_t ray = r >> s.kbits;
        const int32_t k = (int32_t)(r & ((1u << s.kbits) - 1u));
        const float *o = s.rays_o + 3 * (int64_t)ray;
        const float *d = s.rays_d + 3 * (int64_t)ray;
        dx = d[0]; dy = d[1]; dz = d[2];
        if (s.strat) {
            const uint32_t ray_key = kn_mix32(s.seed_key + ray);
            const float t0 = kn_lattice_t<true>(s.t_near, s.step, k, ray_key);
            const float t1 = kn_lattice_t<true>(s.t_near, s.step, k + 1, ray_key);
            x = fmaf(t0, dx, o[0]);
            y = fmaf(t0, dy, o[1]);
            z = fmaf(t0, dz, o[2]);
            dscale = (t1 - t0) / s.step;
        } else {
            kn_lattice_point(o[0], o[1], o[2], dx, dy, dz, s.t_near, s.step, k, x, y, z);
        }
    }
}
