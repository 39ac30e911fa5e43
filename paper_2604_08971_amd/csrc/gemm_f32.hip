// fp32 GEMM (plain FMA, LDS-tiled) and LayerNorm for both dtypes.
// The fp32 path exists for the 1e-5 parity bar of the fp32 workload; it is
// not the throughput path.
#include "gemm.hpp"

namespace sf {

int32_t gemm_bf16(const GemmArgs &a, hipStream_t st);

constexpr int FT = 32;      // output tile edge
constexpr int FK = 16;      // K step

__device__ __forceinline__ float act_f32(float z, int act)
{
    if (act == ACT_RELU) return z > 0.f ? z : 0.f;
    if (act == ACT_GELU) return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
    return z;
}

// 256 threads; thread (tx,ty) of a 16x16 grid owns a 2x2 patch of the 32x32 tile.
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs a)
{
    __shared__ float Xs[FT][FK + 1], Ws[FT][FK + 1];
    const int tiles_m = (a.L + FT - 1) / FT;
    const int b = blockIdx.x / tiles_m;
    const int m0 = (blockIdx.x % tiles_m) * FT;
    const int nt0 = blockIdx.y * FT;
    const int p = a.pattern_id ? a.pattern_id[b] : 0;
    if (p < 0) return;                                             // sample not in use
    if (a.n_lim) a.N = min(a.N, a.n_lim[p]);
    if (a.k_lim) a.K = min(a.K, a.k_lim[p]);
    if (nt0 >= a.N) return;
    const float *A = static_cast<const float *>(a.A) + ((int64_t)b * a.L) * a.lda;
    const float *W = static_cast<const float *>(a.W) + (int64_t)p * a.w_pstride + (int64_t)a.n0 * a.ldw;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};

    for (int k0 = 0; k0 < a.K; k0 += FK) {
        for (int e = threadIdx.x; e < FT * FK; e += 256) {
            const int r = e / FK, k = e % FK;
            const int i = m0 + r, n = nt0 + r;
            Xs[r][k] = (i < a.L && k0 + k < a.K) ? A[(int64_t)i * a.lda + k0 + k] : 0.f;
            Ws[r][k] = (n < a.N && k0 + k < a.K) ? W[(int64_t)n * a.ldw + k0 + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < FK; ++k) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int v = 0; v < 2; ++v)
                    acc[u][v] = fmaf(Xs[ty * 2 + u][k], Ws[tx * 2 + v][k], acc[u][v]);
        }
        __syncthreads();
    }
    const float *bias = a.bias ? static_cast<const float *>(a.bias) + (int64_t)p * a.bias_pstride + a.n0 : nullptr;
    const float *R = static_cast<const float *>(a.R);
    float *C = static_cast<float *>(a.C);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            const int i = m0 + ty * 2 + u, n = nt0 + tx * 2 + v;
            if (i >= a.L || n >= a.N) continue;
            const int64_t row = (int64_t)b * a.L + i;
            float z = acc[u][v] + (bias ? bias[n] : 0.f);
            z = act_f32(z, a.act);
            if (R) z += R[row * a.ldr + a.r0 + n];
            if (a.epi == EPI_VT) C[(int64_t)b * a.vt_b + (int64_t)n * a.vt_n + i] = z;
            else C[row * a.ldc + a.c0 + n] = z;
        }
}

int32_t gemm(int dtype, const GemmArgs &a, hipStream_t st)
{
    if (dtype == SF_BF16) return gemm_bf16(a, st);
    if (a.row_map || a.VT) return fail(SF_ERR_UNSUPPORTED, "gemm(f32): row_map / transposed column range are not supported");
    if (a.B <= 0 || a.N <= 0) return SF_OK;
    dim3 grid(ceil_div(a.L, FT) * a.B, ceil_div(a.N, FT));
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, a);
    return SF_OK;
}

// One 64-lane wave per row; statistics in fp32; biased variance.
// TI: stored type of x, TP: type of gamma/beta, TO: type of y.  y may alias x
// when TI == TO (each row is read completely before it is written).
template <class TI, class TP, class TO>
__global__ __launch_bounds__(256) void layernorm_kernel(const TI *x, const TP *__restrict__ gamma,
                                                        const TP *__restrict__ beta, float eps, int64_t rows,
                                                        int d, TO *y)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const TI *xr = x + row * d;
    TO *yr = y + row * d;
    float s = 0.f;
    for (int k = lane; k < d; k += 64) s += to_f32(xr[k]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    const float mean = s / d;
    float v = 0.f;
    for (int k = lane; k < d; k += 64) { const float c = to_f32(xr[k]) - mean; v += c * c; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    const float inv = 1.0f / sqrtf(v / d + eps);
    for (int k = lane; k < d; k += 64) {
        float z = (to_f32(xr[k]) - mean) * inv;
        if (gamma) z *= to_f32(gamma[k]);
        if (beta) z += to_f32(beta[k]);
        yr[k] = from_f32<TO>(z);
    }
}

// 8 consecutive parameters as floats (`fill` when the vector is absent); 16-byte aligned offsets
template <class TP>
__device__ __forceinline__ void load8(const TP *p, int off, float fill, float (&out)[8])
{
    if (!p) {
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = fill;
    } else if constexpr (sizeof(TP) == 2) {
        const h16x8 t = *reinterpret_cast<const h16x8 *>(p + off);
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = (float)t[e];
    } else {
        const f32x4 t0 = *reinterpret_cast<const f32x4 *>(p + off), t1 = *reinterpret_cast<const f32x4 *>(p + off + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { out[e] = t0[e]; out[4 + e] = t1[e]; }
    }
}

// Vector variant for d % 8 == 0 and d <= 64 * 8 * NCH: the row is read once with
// 16/32-byte loads, kept in registers for both statistics passes, and written
// with 16-byte stores.  One wave per row, 4 rows per block.
template <class TI, class TP, class TO, int NCH>
__global__ __launch_bounds__(256) void layernorm_vec_kernel(const TI *x, const TP *__restrict__ gamma,
                                                            const TP *__restrict__ beta, float eps, int64_t rows,
                                                            int d, TO *y)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const TI *xr = x + row * d;
    TO *yr = y + row * d;
    const int nch = d >> 3;                       // chunks of 8 elements
    float v[NCH][8];
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int ch = lane + c * 64;
        if (ch < nch) {
            if constexpr (sizeof(TI) == 2) {
                const h16x8 t = *reinterpret_cast<const h16x8 *>(xr + ch * 8);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[c][e] = (float)t[e];
            } else {
                const f32x4 t0 = *reinterpret_cast<const f32x4 *>(xr + ch * 8);
                const f32x4 t1 = *reinterpret_cast<const f32x4 *>(xr + ch * 8 + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) { v[c][e] = t0[e]; v[c][4 + e] = t1[e]; }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) s += v[c][e];
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[c][e] = 0.f;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    const float mean = s / d;
    float q = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c)
        if (lane + c * 64 < nch) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float t = v[c][e] - mean; q += t * t; }
        }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o);
    const float inv = 1.0f / sqrtf(q / d + eps);
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int ch = lane + c * 64;
        if (ch >= nch) continue;
        float z[8], gm[8], bt[8];
        load8(gamma, ch * 8, 1.f, gm);
        load8(beta, ch * 8, 0.f, bt);
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = (v[c][e] - mean) * inv * gm[e] + bt[e];
        if constexpr (sizeof(TO) == 2) {
            h16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (h16)z[e];
            *reinterpret_cast<h16x8 *>(yr + ch * 8) = o;
        } else {
            f32x4 o0, o1;
#pragma unroll
            for (int e = 0; e < 4; ++e) { o0[e] = z[e]; o1[e] = z[4 + e]; }
            *reinterpret_cast<f32x4 *>(yr + ch * 8) = o0;
            *reinterpret_cast<f32x4 *>(yr + ch * 8 + 4) = o1;
        }
    }
}

template <class TI, class TP, class TO>
static void launch_ln(const void *x, const void *gamma, const void *beta, float eps, int64_t rows, int d, void *y,
                      hipStream_t st)
{
    dim3 grid((unsigned)((rows + 3) / 4));
    const bool vec = d % 8 == 0 && ((uintptr_t)x % 16 == 0) && ((uintptr_t)y % 16 == 0) &&
                     ((uintptr_t)gamma % 16 == 0) && ((uintptr_t)beta % 16 == 0);
#define SF_LN_ARGS grid, dim3(256), 0, st, (const TI *)x, (const TP *)gamma, (const TP *)beta, eps, rows, d, (TO *)y
    if (vec && d <= 512) hipLaunchKernelGGL((layernorm_vec_kernel<TI, TP, TO, 1>), SF_LN_ARGS);
    else if (vec && d <= 1024) hipLaunchKernelGGL((layernorm_vec_kernel<TI, TP, TO, 2>), SF_LN_ARGS);
    else if (vec && d <= 2048) hipLaunchKernelGGL((layernorm_vec_kernel<TI, TP, TO, 4>), SF_LN_ARGS);
    else hipLaunchKernelGGL((layernorm_kernel<TI, TP, TO>), SF_LN_ARGS);
#undef SF_LN_ARGS
}

void layernorm(int dtype, int x_f32, const void *x, const void *gamma, const void *beta, float eps,
               int64_t rows, int d, void *y, hipStream_t st)
{
    if (rows <= 0) return;
    if (dtype == SF_BF16 && !x_f32) launch_ln<h16, h16, h16>(x, gamma, beta, eps, rows, d, y, st);
    else if (dtype == SF_BF16) launch_ln<float, h16, h16>(x, gamma, beta, eps, rows, d, y, st);
    else launch_ln<float, float, float>(x, gamma, beta, eps, rows, d, y, st);
}

}  // namespace sf
