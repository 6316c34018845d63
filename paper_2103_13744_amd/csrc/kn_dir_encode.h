// Encoding helpers shared by the 16-bit grouped-MLP kernels and the render's set-up kernel: sine / cosine by the
// hardware's revolution-based instructions with the double-angle recurrence in between, packing to 16 bit, and
// gamma(d) of a direction in the operand order ("slot order") of the direction block of the last hidden layer.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kn_enc {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef __bf16 b2 __attribute__((ext_vector_type(2)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef unsigned u4 __attribute__((ext_vector_type(4)));

constexpr float INV_2PI = 0.15915494309189535f;

template <bool BF> __device__ __forceinline__ unsigned pk(float a, float b)
{
    f2 v = {a, b};
    if constexpr (BF)
        return __builtin_bit_cast(unsigned, __builtin_convertvector(v, b2));
    else
        return __builtin_bit_cast(unsigned, __builtin_convertvector(v, h2));
}

// s = sin, c = cos of 2*pi*rev.  The hardware takes revolutions and reduces the range itself for |rev| <= 256;
// WRAP adds an explicit reduction for arguments that may exceed that.
template <bool WRAP> __device__ __forceinline__ void sincos_rev(float rev, float &s, float &c)
{
    const float f = WRAP ? __builtin_amdgcn_fractf(rev) : rev;
    s = __builtin_amdgcn_sinf(f);
    c = __builtin_amdgcn_cosf(f);
}
// (sin a, cos a) -> (sin 2a, cos 2a) = (2 sin a cos a, 2 (1/2 - sin^2 a)).  Written so that each line is one
// VALU instruction with the "times two" output modifier where the file is compiled with flushed fp32 denormals
// and without IEEE mode (two instructions otherwise; the values are the same: doubling is exact).
__device__ __forceinline__ void double_angle(float s, float c, float &s2o, float &c2o)
{
    s2o = (s * c) * 2.0f;
    c2o = fmaf(-s, s, 0.5f) * 2.0f;
}

// The four packed pairs (sin, cos at frequencies 0..3) of one direction component given in revolutions.
template <bool BF> __device__ __forceinline__ u4 dir_axis_slots(float rev)
{
    float s[4], m[4];
    sincos_rev<false>(rev, s[0], m[0]); // directions: |d| far below 256 revolutions
    double_angle(s[0], m[0], s[1], m[1]);
    double_angle(s[1], m[1], s[2], m[2]);
    double_angle(s[2], m[2], s[3], m[3]);
    return (u4){pk<BF>(s[0], m[0]), pk<BF>(s[1], m[1]), pk<BF>(s[2], m[2]), pk<BF>(s[3], m[3])};
}

// gamma(d) of one direction as the B operands of the four lane groups (16 bytes each): groups 0..2 hold axis g at
// frequencies 0..3 (sin, cos pairs), group 3 holds (dx, dy), (dz, 1) and zeros (its other slots meet zero weights).
template <bool BF> __device__ __forceinline__ void dir_slots(float dx, float dy, float dz, u4 out[4])
{
    out[0] = dir_axis_slots<BF>(dx * INV_2PI);
    out[1] = dir_axis_slots<BF>(dy * INV_2PI);
    out[2] = dir_axis_slots<BF>(dz * INV_2PI);
    out[3] = (u4){pk<BF>(dx, dy), pk<BF>(dz, 1.0f), 0u, 0u};
}

} // namespace kn_enc
