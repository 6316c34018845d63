// Device helpers shared by the grouped-MLP kernels.
#pragma once

#include "kn_common.h"

// Fetch position and direction of sorted-list entry `idx`: either from explicit arrays, or by
// rebuilding the lattice point of a render sample from its packed (ray, k) record with the same
// fused multiply-adds the marching kernel used.
__device__ __forceinline__ void kn_load_sample(const KnSampleSrc &s, int32_t idx, float &x, float &y, float &z,
                                               float &dx, float &dy, float &dz)
{
    if (s.points) {
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
        kn_lattice_point(o[0], o[1], o[2], dx, dy, dz, s.t_near, s.step, k, x, y, z);
    }
}
