// Device-side helpers shared by the kernel files: storage-type conversion and rotary angles.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float fc_to_float(float v) { return v; }
__device__ __forceinline__ float fc_to_float(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }

// float -> bfloat16, round to nearest even (the hardware conversion of gfx950); NaN stays NaN.
__device__ __forceinline__ uint16_t fc_bf16_bits(float f)
{
    union { __bf16 h; uint16_t u; } x;
    x.h = (__bf16)f;
    return x.u;
}

template <typename T>
__device__ __forceinline__ T fc_from_float(float f);
template <>
__device__ __forceinline__ float fc_from_float<float>(float f) { return f; }
template <>
__device__ __forceinline__ bf16_t fc_from_float<bf16_t>(float f)
{
    bf16_t r;
    r.bits = fc_bf16_bits(f);
    return r;
}

// cos and sin of pos * base^(-2 i / Dh).  The angle is formed and reduced to [-pi, pi] in double
// so that long contexts (pos ~ 1e5 and beyond) lose no accuracy; sin/cos themselves run in float.
__device__ __forceinline__ void fc_rope_cs(int pos, int i, int Dh, double log_base, float *c, float *s)
{
    const double theta = exp(-(2.0 * (double)i / (double)Dh) * log_base);
    double ang = (double)pos * theta;
    const double two_pi = 6.283185307179586476925286766559;
    ang -= two_pi * rint(ang / two_pi);
    sincosf((float)ang, s, c);
}
