// FP8 arithmetic for the attention projections (Sec. 6, "Compatibility with quantization": the FP8 models; which
// contractions run in FP8 is this build's reading).  The contractions are gemm_fp8() launches issued by the encoder;
// this file holds the argument checks and the V transposition that the bf16 GEMM does in its epilogue.
#include "fp8.hpp"
#include "gemm.hpp"

namespace sf {

namespace {

// 64 tokens x 64 features per block through LDS, 16 bytes per lane on both sides: 8 features of a token on the way
// in, 8 tokens of a feature on the way out (ld, col0, ncols, Lp multiples of 8).
__global__ __launch_bounds__(256) void transpose_v_kernel(const h16 *__restrict__ src, int64_t ld, int col0, int ncols,
                                                          int L, int Lp, h16 *__restrict__ vt,
                                                          const int32_t *__restrict__ row0)
{
    __shared__ uint16_t tile[64][66];                          // row stride 33 words: the column reads spread over the banks
    const int b = blockIdx.z, j0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    // row0: samples packed back to back (sample b starts at row row0[b]); the transposed copy stays b-strided
    const uint16_t *s = reinterpret_cast<const uint16_t *>(src) + (row0 ? (int64_t)row0[b] : (int64_t)b * L) * ld + col0;
    uint16_t *dst = reinterpret_cast<uint16_t *>(vt) + (int64_t)b * ncols * Lp;
    const int ch = threadIdx.x & 7, r = threadIdx.x >> 3;      // 8 chunks x 32 rows per pass
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int jj = r + pass * 32, j = j0 + jj, c = c0 + ch * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (j < L && c < ncols) v = *reinterpret_cast<const uint4 *>(s + (int64_t)j * ld + c);
        uint32_t *t = reinterpret_cast<uint32_t *>(&tile[jj][ch * 8]);
        t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int cc = r + pass * 32, c = c0 + cc, j = j0 + ch * 8;
        if (c >= ncols || j >= Lp) continue;
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            w[k] = (uint32_t)tile[ch * 8 + 2 * k][cc] | ((uint32_t)tile[ch * 8 + 2 * k + 1][cc] << 16);
        *reinterpret_cast<uint4 *>(dst + (int64_t)c * Lp + j) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// codes[r, c] = E4M3(x[r, c] * inv_scale) for c < K, 0 for K <= c < Kp: rows of a bf16 matrix into code rows padded to
// the FP8 GEMM's K granularity.  8 elements per thread (K, Kp, ld multiples of 8).
__global__ __launch_bounds__(256) void quantize_rows_fp8_kernel(const h16 *__restrict__ x, int64_t ld, int64_t rows, int K,
                                                                int Kp, float inv_scale, uint8_t *__restrict__ codes)
{
    const int per_row = Kp / 8;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= rows * per_row) return;
    const int64_t r = t / per_row;
    const int c = (int)(t % per_row) * 8;
    uint2 o = make_uint2(0, 0);
    if (c < K) {
        const h16x8 v = *reinterpret_cast<const h16x8 *>(x + r * ld + c);
        o.x = e4m3_pack4((float)v[0] * inv_scale, (float)v[1] * inv_scale, (float)v[2] * inv_scale, (float)v[3] * inv_scale);
        o.y = e4m3_pack4((float)v[4] * inv_scale, (float)v[5] * inv_scale, (float)v[6] * inv_scale, (float)v[7] * inv_scale);
    }
    *reinterpret_cast<uint2 *>(codes + r * Kp + c) = o;
}

}  // namespace

void quantize_rows_fp8(const void *x, int64_t ld, int64_t rows, int K, int Kp, float inv_scale, uint8_t *codes, hipStream_t st)
{
    const int64_t n = rows * (Kp / 8);
    if (n == 0) return;
    hipLaunchKernelGGL(quantize_rows_fp8_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const h16 *)x, ld,
                       rows, K, Kp, inv_scale, codes);
}

void transpose_v(const void *src, int64_t ld, int col0, int ncols, int B, int L, int Lp, void *vt, hipStream_t st,
                 const int32_t *row0)
{
    if (B == 0 || ncols == 0) return;
    dim3 grid((unsigned)ceil_div(Lp, 64), (unsigned)ceil_div(ncols, 64), (unsigned)B);
    hipLaunchKernelGGL(transpose_v_kernel, grid, dim3(256), 0, st, (const h16 *)src, ld, col0, ncols, L, Lp,
                       (h16 *)vt, row0);
}

int32_t proj_fp8_check(const char *who, const Dims &D, const sf_proj_fp8 *p, int k_head)
{
    if (!p) return fail(SF_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (D.dtype != SF_BF16) return fail(SF_ERR_UNSUPPORTED, "%s: the FP8 path takes 16-bit activations, not fp32", who);
    if (p->k_head != k_head) return fail(SF_ERR_INVALID_ARG, "%s: k_head differs from the compact layer's", who);
    if (!p->Wqkv8 || !p->WoT8) return fail(SF_ERR_INVALID_ARG, "%s: NULL weight pointer", who);
    if (((uintptr_t)p->Wqkv8 | (uintptr_t)p->WoT8) & 15)
        return fail(SF_ERR_INVALID_ARG, "%s: 16-byte aligned weight codes required", who);
    if (!(p->s_qkv > 0.f) || !(p->so > 0.f) || !(p->sx1 > 0.f) || !(p->sa > 0.f))
        return fail(SF_ERR_INVALID_ARG, "%s: the four scales must be positive", who);
    if (D.d % 128 || D.d < 256 || D.d > 4096)
        return fail(SF_ERR_SHAPE, "%s: d_model must be a multiple of 128 in [256, 4096]", who);
    if ((k_head + 2 * D.Hk) * D.dh < 192) return fail(SF_ERR_UNSUPPORTED, "%s: at least 192 Q/K/V features required", who);
    if (D.L < 192) return fail(SF_ERR_UNSUPPORTED, "%s: at least 192 tokens per sample required", who);
    return SF_OK;
}

}  // namespace sf

using namespace sf;

extern "C" int32_t sf_proj_fp8_padded(int32_t k_head, int32_t d_head)
{
    return k_head < 1 || d_head < 1 ? 0 : (int32_t)align_up((size_t)k_head * d_head, 128);
}
