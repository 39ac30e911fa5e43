// FP8 arithmetic for the pruned FFN (Sec. 6, "Compatibility with quantization": the paper reports FP8 models
// but not how they compute; here both operands of the two FFN contractions are OCP E4M3 codes with one fp32
// scale per tensor).  This file holds the quantisers (plain, and fused into LayerNorm) and the block's entry
// points; the contraction itself is gemm_fp8() in gemm_bf16_ws.hip.
#include "fp8.hpp"
#include "gemm.hpp"

namespace sf {

namespace {

// codes[i] = E4M3(x[i] * inv_scale), 8 elements per thread (n8 groups of 8), tail element-wise
template <class T>
__global__ __launch_bounds__(256) void quantize_fp8_kernel(const T *__restrict__ x, int64_t n, float inv_scale,
                                                           uint8_t *__restrict__ codes)
{
    const int64_t i8 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i8 >= n) return;
    float t[8];
    if (i8 + 8 <= n) {
        if constexpr (sizeof(T) == 2) {
            const h16x8 v = *reinterpret_cast<const h16x8 *>(x + i8);
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] = (float)v[e] * inv_scale;
        } else {
            const f32x4 a = *reinterpret_cast<const f32x4 *>(x + i8), b = *reinterpret_cast<const f32x4 *>(x + i8 + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { t[e] = a[e] * inv_scale; t[4 + e] = b[e] * inv_scale; }
        }
        uint2 o;
        o.x = e4m3_pack4(t[0], t[1], t[2], t[3]);
        o.y = e4m3_pack4(t[4], t[5], t[6], t[7]);
        *reinterpret_cast<uint2 *>(codes + i8) = o;
    } else {
        for (int64_t i = i8; i < n; ++i) {
            const float v = to_f32(x[i]) * inv_scale;
            codes[i] = (uint8_t)(e4m3_pack4(v, 0.f, 0.f, 0.f) & 0xffu);
        }
    }
}

// LayerNorm (statistics in fp32, biased variance) with the quantiser applied to the fp32 result: one wave per
// row, the row is read once and kept in registers (d % 8 == 0, d <= 512 * NCH), 8 codes per store.
template <class TI, int NCH>
__global__ __launch_bounds__(256) void layernorm_q8_kernel(const TI *__restrict__ x, const h16 *__restrict__ gamma,
                                                           const h16 *__restrict__ beta, float eps, int64_t rows,
                                                           int d, float inv_scale, uint8_t *__restrict__ y)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const TI *xr = x + row * d;
    const int nch = d >> 3;
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
        float z[8];
        h16x8 gm, bt;
        if (gamma) gm = *reinterpret_cast<const h16x8 *>(gamma + ch * 8);
        if (beta) bt = *reinterpret_cast<const h16x8 *>(beta + ch * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float t = (v[c][e] - mean) * inv;
            if (gamma) t *= (float)gm[e];
            if (beta) t += (float)bt[e];
            z[e] = t * inv_scale;
        }
        uint2 o;
        o.x = e4m3_pack4(z[0], z[1], z[2], z[3]);
        o.y = e4m3_pack4(z[4], z[5], z[6], z[7]);
        *reinterpret_cast<uint2 *>(y + row * d + ch * 8) = o;
    }
}

struct Fp8FfnWs { uint8_t *xq, *hq; size_t bytes; };
Fp8FfnWs fp8_ffn_ws(const Dims &D, int Fp8, void *ws)
{
    Carver c(ws);
    Fp8FfnWs w{};
    const size_t rows = (size_t)D.B * D.L;
    w.xq = c.take<uint8_t>(rows * D.d);
    w.hq = c.take<uint8_t>(rows * Fp8);
    w.bytes = c.off;
    return w;
}

int gemm_act(int act) { return act == SF_GELU_ERF ? ACT_GELU : ACT_RELU; }

}  // namespace

}  // namespace sf

using namespace sf;

extern "C" int32_t sf_ffn_fp8_padded(int32_t k_ffn)
{
    return k_ffn < 1 ? 0 : (int32_t)align_up((size_t)k_ffn, 128);
}

extern "C" int32_t sf_quantize_fp8(const void *x, int32_t dtype, int64_t n, float scale, uint8_t *codes, void *stream)
{
    if (n < 0 || (n > 0 && (!x || !codes))) return fail(SF_ERR_INVALID_ARG, "quantize_fp8: NULL argument");
    if (dtype != SF_BF16 && dtype != SF_F32)
        return fail(SF_ERR_INVALID_ARG, "quantize_fp8: dtype must be SF_F32 or SF_BF16");
    if (dtype == SF_BF16 && SF_DTYPE_16 != SF_BF16)
        return fail(SF_ERR_UNSUPPORTED, "quantize_fp8: bfloat16 input takes libsentryfuse.so");
    if (!(scale > 0.f) || !(scale < 3.0e38f)) return fail(SF_ERR_INVALID_ARG, "quantize_fp8: scale must be positive and finite");
    if (((uintptr_t)x & 15) || ((uintptr_t)codes & 7))
        return fail(SF_ERR_INVALID_ARG, "quantize_fp8: x must be 16-byte and codes 8-byte aligned");
    if (n == 0) return SF_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float inv = 1.0f / scale;
    const int64_t groups = (n + 7) / 8;
    const unsigned grid = (unsigned)((groups + 255) / 256);
    if (dtype == SF_BF16)
        hipLaunchKernelGGL(quantize_fp8_kernel<h16>, dim3(grid), dim3(256), 0, st, (const h16 *)x, n, inv, codes);
    else
        hipLaunchKernelGGL(quantize_fp8_kernel<float>, dim3(grid), dim3(256), 0, st, (const float *)x, n, inv, codes);
    return check_launch("quantize_fp8");
}

static int32_t check_ffn_fp8(const char *who, const Dims &D, const sf_ffn_fp8 *f)
{
    if (!f) return fail(SF_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (D.dtype != SF_BF16) return fail(SF_ERR_UNSUPPORTED, "%s: the FP8 path takes 16-bit activations, not fp32", who);
    if (f->k_ffn < 1 || f->k_ffn > D.F) return fail(SF_ERR_INVALID_ARG, "%s: k_ffn out of range", who);
    if (!f->W1q || !f->W2Tq) return fail(SF_ERR_INVALID_ARG, "%s: NULL weight pointer", who);
    if (!(f->s1 > 0.f) || !(f->s2 > 0.f) || !(f->sx > 0.f) || !(f->sh > 0.f))
        return fail(SF_ERR_INVALID_ARG, "%s: the four scales must be positive", who);
    if (D.d % 128 || D.d < 256) return fail(SF_ERR_SHAPE, "%s: d_model must be a multiple of 128, at least 256", who);
    if (D.L < 192) return fail(SF_ERR_UNSUPPORTED, "%s: at least 192 tokens per sample required", who);
    if (f->k_ffn <= 128) return fail(SF_ERR_UNSUPPORTED, "%s: more than 128 kept channels required", who);
    return SF_OK;
}

extern "C" size_t sf_pruned_ffn_fp8_workspace_bytes(const sf_desc *desc, int32_t k_ffn)
{
    Dims D;
    if (read_desc(desc, D) || k_ffn < 1) return 0;
    return fp8_ffn_ws(D, sf_ffn_fp8_padded(k_ffn), nullptr).bytes;
}

namespace sf {

void layernorm_q8(const void *X, bool x_f32, const void *gamma, const void *beta, float eps, int64_t rows, int d,
                  float inv_scale, uint8_t *y, hipStream_t st)
{
    if (rows == 0) return;
    dim3 grid((unsigned)((rows + 3) / 4));
#define SF_LNQ_ARGS(TI) grid, dim3(256), 0, st, (const TI *)X, (const h16 *)gamma, (const h16 *)beta, eps, rows, d, inv_scale, y
#define SF_LNQ(TI) \
    do { \
        if (d <= 512) hipLaunchKernelGGL((layernorm_q8_kernel<TI, 1>), SF_LNQ_ARGS(TI)); \
        else if (d <= 1024) hipLaunchKernelGGL((layernorm_q8_kernel<TI, 2>), SF_LNQ_ARGS(TI)); \
        else if (d <= 2048) hipLaunchKernelGGL((layernorm_q8_kernel<TI, 4>), SF_LNQ_ARGS(TI)); \
        else hipLaunchKernelGGL((layernorm_q8_kernel<TI, 8>), SF_LNQ_ARGS(TI)); \
    } while (0)
    if (x_f32) SF_LNQ(float);
    else SF_LNQ(h16);
#undef SF_LNQ
#undef SF_LNQ_ARGS
}

void quantize_fp8_bf16(const void *x, int64_t n, float inv_scale, uint8_t *codes, hipStream_t st)
{
    if (n == 0) return;
    hipLaunchKernelGGL(quantize_fp8_kernel<h16>, dim3((unsigned)(((n + 7) / 8 + 255) / 256)), dim3(256), 0, st,
                       (const h16 *)x, n, inv_scale, codes);
}

}  // namespace sf

namespace sf {

int32_t ffn_fp8_check(const char *who, const Dims &D, const sf_ffn_fp8 *f, bool pre_ln)
{
    if (int32_t rc = check_ffn_fp8(who, D, f)) return rc;
    if (pre_ln && D.d > 4096) return fail(SF_ERR_SHAPE, "%s: d_model <= 4096 required with the LayerNorm", who);
    if (((uintptr_t)f->ln2_g | (uintptr_t)f->ln2_b) & 15)
        return fail(SF_ERR_INVALID_ARG, "%s: 16-byte aligned LayerNorm vectors required", who);
    return SF_OK;
}

// x_f32 / y_f32: X / Y hold fp32 (the encoder's residual stream); with x_f32 the LayerNorm is required.
int32_t ffn_fp8_forward(const Dims &D, const sf_ffn_fp8 &f, const void *X, bool x_f32, const int32_t *pattern_id,
                        bool pre_ln, bool add_residual, void *Y, bool y_f32, uint8_t *xq, uint8_t *hq, hipStream_t st,
                        bool xq_ready)
{
    const int Fp8 = sf_ffn_fp8_padded(f.k_ffn);
    const int64_t rows = (int64_t)D.B * D.L;
    const float inv_sx = 1.0f / f.sx;
    if (xq_ready) {
        // the codes of LN2(X) were written together with X
    } else if (pre_ln) {
        layernorm_q8(X, x_f32, f.ln2_g, f.ln2_b, D.eps, rows, D.d, inv_sx, xq, st);
    } else {
        if (x_f32) return fail(SF_ERR_UNSUPPORTED, "ffn_fp8: an fp32 input needs the LayerNorm");
        quantize_fp8_bf16(X, rows * D.d, inv_sx, xq, st);
    }
    GemmArgs g{};
    g.f8 = 1; g.A = xq; g.lda = D.d; g.W = f.W1q; g.ldw = D.d; g.w_pstride = (int64_t)Fp8 * D.d;
    g.bias = f.b1; g.bias_pstride = Fp8; g.pattern_id = pattern_id;
    g.B = D.B; g.L = D.L; g.N = Fp8; g.K = D.d; g.epi = EPI_ROWMAJOR; g.act = gemm_act(D.act);
    g.out_scale = f.sx * f.s1;
    g.c_f8 = 1; g.c_scale = 1.0f / f.sh; g.C = hq; g.ldc = Fp8;
    if (int32_t rc = gemm_fp8(g, st)) return rc;

    GemmArgs h{};
    h.f8 = 1; h.A = hq; h.lda = Fp8; h.W = f.W2Tq; h.ldw = Fp8; h.w_pstride = (int64_t)D.d * Fp8;
    h.bias = f.b2; h.bias_pstride = 0; h.pattern_id = pattern_id;
    h.B = D.B; h.L = D.L; h.N = D.d; h.K = Fp8; h.epi = EPI_ROWMAJOR; h.act = ACT_NONE;
    h.out_scale = f.sh * f.s2;
    h.R = add_residual ? X : nullptr; h.ldr = D.d; h.r_f32 = x_f32;
    h.C = Y; h.ldc = D.d; h.c_f32 = y_f32;
    return gemm_fp8(h, st);
}

}  // namespace sf

extern "C" int32_t sf_pruned_ffn_fp8_forward(const sf_desc *desc, const sf_ffn_fp8 *f, const void *X,
                                             const int32_t *pattern_id, int32_t pre_ln, int32_t add_residual,
                                             void *Y, uint8_t *xq_out, uint8_t *hq_out, void *workspace,
                                             size_t workspace_bytes, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (SF_DTYPE_16 != SF_BF16)
        return fail(SF_ERR_UNSUPPORTED, "pruned_ffn_fp8: the stand-alone block is built for bfloat16 models (the FP16 build "
                                        "runs FP8 arithmetic inside sf_encoder_forward_fp8)");
    if (int32_t rc = ffn_fp8_check("pruned_ffn_fp8", D, f, pre_ln != 0)) return rc;
    if (!X || !Y) return fail(SF_ERR_INVALID_ARG, "pruned_ffn_fp8: NULL argument");
    if (X == Y) return fail(SF_ERR_INVALID_ARG, "pruned_ffn_fp8: Y may not alias X");
    if (D.P > 1 && !pattern_id) return fail(SF_ERR_INVALID_ARG, "pruned_ffn_fp8: pattern_id required when P > 1");
    if (((uintptr_t)X | (uintptr_t)Y | (uintptr_t)xq_out | (uintptr_t)hq_out) & 15)
        return fail(SF_ERR_INVALID_ARG, "pruned_ffn_fp8: 16-byte aligned pointers required");
    const int Fp8 = sf_ffn_fp8_padded(f->k_ffn);
    Fp8FfnWs w = fp8_ffn_ws(D, Fp8, workspace);
    if (!workspace || workspace_bytes < w.bytes || ((uintptr_t)workspace & 255))
        return fail(SF_ERR_WORKSPACE, "pruned_ffn_fp8: workspace of %zu bytes (256-byte aligned) required, got %zu",
                    w.bytes, workspace_bytes);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (int32_t rc = ffn_fp8_forward(D, *f, X, false, pattern_id, pre_ln != 0, add_residual != 0, Y, false,
                                     xq_out ? xq_out : w.xq, hq_out ? hq_out : w.hq, st, false))
        return rc;
    return check_launch("pruned_ffn_fp8_forward");
}
