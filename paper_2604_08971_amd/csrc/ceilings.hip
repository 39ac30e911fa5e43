// Measurement aids: what this GPU reaches on a pure bf16 MFMA issue loop and on a plain device copy.
// The benchmark reports both next to the published peaks, measured in the same run on the same box, so that a
// kernel's fraction can be read against the published and against the reachable figure.  No part of the method.
#include "common.hpp"

namespace sf {

namespace {

constexpr int CEIL_WAVES = 8;          // 2 waves per SIMD
constexpr int CEIL_TILES = 8;          // independent 32x32 accumulator tiles per wave (128 registers)

// Every wave issues `iters` rounds of CEIL_TILES independent 32x32x16 MFMAs from operands held in registers: no
// memory traffic, no LDS.  random_operands = 0: the operands are one constant pattern (little switching in the
// multipliers); 1: four operand pairs of pseudo-random bf16 values in [-1, 1) rotate, zero-mean, so the sums stay
// small - the data-dependent power of a real GEMM without its data movement.
__global__ __launch_bounds__(64 * CEIL_WAVES) __attribute__((amdgpu_waves_per_eu(2, 2)))
void mfma_ceiling_kernel(int iters, int random_operands, float *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    h16x8 a[4], b[4];
    uint32_t s = (uint32_t)(blockIdx.x * 1024 + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float fa = 1.0f, fb = 0.5f;
            if (random_operands) {
                s = s * 1664525u + 1013904223u;
                fa = (float)(int)(s >> 8 & 0xFFFF) * (1.0f / 32768.0f) - 1.0f;
                s = s * 1664525u + 1013904223u;
                fb = (float)(int)(s >> 8 & 0xFFFF) * (1.0f / 32768.0f) - 1.0f;
            }
            a[r][e] = (h16)fa;
            b[r][e] = (h16)fb;
        }
    f32x16 acc[CEIL_TILES];
#pragma unroll
    for (int t = 0; t < CEIL_TILES; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int t = 0; t < CEIL_TILES; ++t) acc[t] = SF_MFMA16(a[r], b[(r + t) & 3], acc[t], 0, 0, 0);
    }
    float v = 0.f;
#pragma unroll
    for (int t = 0; t < CEIL_TILES; ++t) v += acc[t][lane & 15];
    if (v == 123.456f) sink[blockIdx.x] = v;      // keeps the loop alive; practically never true
}

// dst[i] = src[i], 16 bytes per lane, grid-stride, four independent loads in flight per lane; streamed (the data is
// touched once)
__global__ __launch_bounds__(256) void copy_ceiling_kernel(const f32x4 *__restrict__ src, f32x4 *__restrict__ dst,
                                                           int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        f32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

}  // namespace sf

using namespace sf;

extern "C" int64_t sf_ceiling_mfma_launch(int32_t workgroups, int32_t iters, int32_t random_operands, float *sink,
                                          void *stream)
{
    if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 24) || !sink) {
        fail(SF_ERR_INVALID_ARG, "ceiling_mfma: 1 <= workgroups <= 65536, 1 <= iters <= 2^24 and a sink of `workgroups` floats required");
        return SF_ERR_INVALID_ARG;
    }
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(workgroups), dim3(64 * CEIL_WAVES), 0, static_cast<hipStream_t>(stream),
                       iters, random_operands, sink);
    if (int32_t rc = check_launch("ceiling_mfma")) return rc;
    // flops of the launch: 2 * 32 * 32 * 16 per MFMA
    return (int64_t)workgroups * CEIL_WAVES * iters * 4 * CEIL_TILES * 32768;
}

extern "C" int32_t sf_ceiling_copy_launch(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst || bytes < 16 || bytes % 16 || (((uintptr_t)src | (uintptr_t)dst) & 15))
        return fail(SF_ERR_INVALID_ARG, "ceiling_copy: 16-byte aligned buffers and a multiple of 16 bytes required");
    const int64_t n16 = (int64_t)(bytes / 16);
    const int64_t want = (n16 + 255) / 256;
    const unsigned blocks = (unsigned)(want < 256 * 8 ? want : 256 * 8);
    hipLaunchKernelGGL(copy_ceiling_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const f32x4 *>(src), static_cast<f32x4 *>(dst), n16);
    return check_launch("ceiling_copy");
}
