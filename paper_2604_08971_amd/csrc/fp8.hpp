// E4M3 (OCP FP8, 1-4-3, bias 7, finite only) conversion shared by the kernels that quantise activations.
#pragma once

#include "common.hpp"

namespace sf {

// Four fp32 values (already multiplied by the reciprocal scale) -> four E4M3 codes, round to nearest even,
// saturating at +-448 (the conversion instruction alone would overflow to NaN), NaN -> 0x7F.
__device__ __forceinline__ uint32_t e4m3_pack4(float t0, float t1, float t2, float t3)
{
    const float c0 = __builtin_amdgcn_fmed3f(t0, -448.f, 448.f), c1 = __builtin_amdgcn_fmed3f(t1, -448.f, 448.f);
    const float c2 = __builtin_amdgcn_fmed3f(t2, -448.f, 448.f), c3 = __builtin_amdgcn_fmed3f(t3, -448.f, 448.f);
    int w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c0, c1, w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c2, c3, w, true);
    uint32_t u = (uint32_t)w;
    if (t0 != t0) u = (u & 0xffffff00u) | 0x0000007fu;
    if (t1 != t1) u = (u & 0xffff00ffu) | 0x00007f00u;
    if (t2 != t2) u = (u & 0xff00ffffu) | 0x007f0000u;
    if (t3 != t3) u = (u & 0x00ffffffu) | 0x7f000000u;
    return u;
}

// The value of one E4M3 code (exact in fp32): subnormals m * 2^-9, normals (1 + m/8) * 2^(e-7), 0x7F / 0xFF NaN.
__device__ __forceinline__ float e4m3_value(uint32_t code)
{
    const uint32_t e = (code >> 3) & 0xFu, m = code & 7u;
    float v = e ? __uint_as_float(((e + 120u) << 23) | (m << 20)) : (float)m * 0x1p-9f;
    if ((code & 0x7Fu) == 0x7Fu) v = __builtin_nanf("");
    return (code & 0x80u) ? -v : v;
}

}  // namespace sf
