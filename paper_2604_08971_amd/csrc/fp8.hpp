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

}  // namespace sf
