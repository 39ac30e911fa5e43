// Output projection after SentryAttend when most rows are lazy (Sec. 4.4: rows outside a head's top-U set receive
// their group's mean-V context vector).  Every row that is lazy in ALL kept heads of its sample carries the
// same attention output - the concatenated group context vectors - so its projection is one vector per sample,
//     c_b = ctx_b Wo' + bo.
// Only the rows that are active in some head (at most Hq'*U per sample) go through the GEMM, from a compact buffer;
// one pass then forms the residual stream x1 = x + (projection of the row | c_b) and the LayerNorm that follows it.
// The arithmetic is that of fill + projection + residual + LayerNorm; only the summation order of c_b differs.
#include "attention.hpp"
#include "fp8.hpp"

namespace sf {

namespace {

// The rows with an active head, ascending, from the bitmap the selection leaves behind (bit i of sample b: some kept
// head selected row i): one block per sample, a thread per 32-row word.  arow[b, j] = row of compact position j,
// pos_of[b, i] = compact position of row i or -1, n_act[b] = their number (<= capA by construction: a head has at most
// U active rows and capA >= nH*U), and blk_pattern[b, k] = the sample's pattern for the 128-row blocks of the compact
// buffer that hold rows, -1 for the empty ones (the GEMM skips those).
constexpr int RA_NT = 512;          // one word per thread: L <= 16384 (lazy_cap() admits no longer sequence)

__global__ __launch_bounds__(RA_NT) void rows_active_kernel(const uint32_t *__restrict__ act_bits, int L, int capA,
                                                            const int32_t *__restrict__ pattern_id,
                                                            int32_t *__restrict__ arow, int32_t *__restrict__ pos_of,
                                                            int32_t *__restrict__ n_act, int32_t *__restrict__ blk_pattern)
{
    __shared__ int wsum[RA_NT / 64];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwords = (L + 31) / 32;
    uint32_t bits = tid < nwords ? act_bits[(int64_t)b * nwords + tid] : 0u;
    if (tid == nwords - 1 && (L & 31)) bits &= (1u << (L & 31)) - 1u;      // no row behind L
    const int cnt = __popc(bits);
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int pos = incl - cnt, total = 0;
#pragma unroll
    for (int w = 0; w < RA_NT / 64; ++w) {
        const int c = wsum[w];
        if (w < wave) pos += c;
        total += c;
    }
    if (tid < nwords) {
        const int i0 = tid * 32;
        for (int k = 0; k < 32 && i0 + k < L; ++k) {
            const bool act = (bits >> k) & 1u;
            const bool keep = act && pos < capA;
            pos_of[(int64_t)b * L + i0 + k] = keep ? pos : -1;
            if (keep) arow[(int64_t)b * capA + pos] = i0 + k;
            pos += act;
        }
    }
    total = min(total, capA);
    if (tid == 0) n_act[b] = total;
    const int p = pattern_id ? pattern_id[b] : 0;
    for (int k = tid; k < capA / 128; k += RA_NT) blk_pattern[(int64_t)b * (capA / 128) + k] = k * 128 < total ? p : -1;
}

// 8 consecutive context values of head h (group g of sample b), rounded to bf16 as the attention output stores them
__device__ __forceinline__ h16x8 ctx8(const float *__restrict__ stats, int b, int nG, int g, int dh, int e0)
{
    const float *c = stats + (((int64_t)b * nG + g) * 2 + 1) * dh + e0;
    h16x8 o;
#pragma unroll
    for (int t = 0; t < 8; ++t) o[t] = (h16)c[t];
    return o;
}

// One wave per compact row: the attention output of an active row - its active heads from `att`, its lazy heads from
// the context vectors - or a zero row behind n_act[b].  K = nH*dh, a multiple of 8; dh a multiple of 8.
__device__ __forceinline__ void att_compact_rows(int block, const h16 *__restrict__ att, int64_t ldo,
                                                          const int32_t *__restrict__ slot, const float *__restrict__ stats,
                                                          const int32_t *__restrict__ head_group, int hg_stride,
                                                          const int32_t *__restrict__ pattern_id,
                                                          const int32_t *__restrict__ arow, const int32_t *__restrict__ n_act,
                                                          int B, int nH, int nG, int L, int dh, int capA,
                                                          h16 *__restrict__ Ac)
{
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)block * 4 + (threadIdx.x >> 6);
    if (r >= (int64_t)B * capA) return;
    const int b = (int)(r / capA), j = (int)(r % capA);
    const int K = nH * dh;
    h16 *dst = Ac + r * K;
    if (j >= n_act[b]) {
        const h16x8 z = {};
        for (int c = lane; c < K / 8; c += 64) *reinterpret_cast<h16x8 *>(dst + c * 8) = z;
        return;
    }
    const int i = arow[r];
    const int p = pattern_id ? pattern_id[b] : 0;
    for (int c = lane; c < K / 8; c += 64) {
        const int h = (c * 8) / dh, e0 = (c * 8) % dh;
        h16x8 v;
        if (slot[((int64_t)b * nH + h) * L + i] >= 0)
            v = *reinterpret_cast<const h16x8 *>(att + ((int64_t)b * L + i) * ldo + c * 8);
        else
            v = ctx8(stats, b, nG, head_group[(int64_t)p * hg_stride + h], dh, e0);
        *reinterpret_cast<h16x8 *>(dst + c * 8) = v;
    }
}

// One wave per (sample, output feature n): c[b, n] = sum_k bf16(ctx_b[k]) WoT[p_b][n, k] + bo[n], fp32.
__device__ __forceinline__ void ctx_proj_rows(int block, const float *__restrict__ stats, const int32_t *__restrict__ head_group,
                                                       int hg_stride, const int32_t *__restrict__ pattern_id,
                                                       const h16 *__restrict__ WoT, int64_t w_pstride,
                                                       const h16 *__restrict__ bo, int B, int nH, int nG, int dh,
                                                       int d, float *__restrict__ cvec)
{
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)block * 4 + (threadIdx.x >> 6);
    if (r >= (int64_t)B * d) return;
    const int b = (int)(r / d), n = (int)(r % d);
    const int p = pattern_id ? pattern_id[b] : 0;
    const int K = nH * dh;
    const h16 *w = WoT + (int64_t)p * w_pstride + (int64_t)n * K;
    float acc = 0.f;
    for (int c = lane; c < K / 8; c += 64) {
        const int h = (c * 8) / dh, e0 = (c * 8) % dh;
        const h16x8 x = ctx8(stats, b, nG, head_group[(int64_t)p * hg_stride + h], dh, e0);
        const h16x8 wv = *reinterpret_cast<const h16x8 *>(w + c * 8);
#pragma unroll
        for (int t = 0; t < 8; ++t) acc = fmaf((float)x[t], (float)wv[t], acc);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) cvec[r] = acc + (bo ? (float)bo[n] : 0.f);
}

__global__ __launch_bounds__(256) void att_compact_kernel(const h16 *__restrict__ att, int64_t ldo,
                                                          const int32_t *__restrict__ slot, const float *__restrict__ stats,
                                                          const int32_t *__restrict__ head_group, int hg_stride,
                                                          const int32_t *__restrict__ pattern_id,
                                                          const int32_t *__restrict__ arow, const int32_t *__restrict__ n_act,
                                                          int B, int nH, int nG, int L, int dh, int capA,
                                                          h16 *__restrict__ Ac)
{
    att_compact_rows(blockIdx.x, att, ldo, slot, stats, head_group, hg_stride, pattern_id, arow, n_act, B, nH, nG, L, dh,
                     capA, Ac);
}

// Both in one launch (they are independent and small): the first n_compact blocks gather the compact rows, the rest
// project the context vectors.
__global__ __launch_bounds__(256) void att_compact_ctx_proj_kernel(
    int n_compact, const h16 *__restrict__ att, int64_t ldo, const int32_t *__restrict__ slot,
    const float *__restrict__ stats, const int32_t *__restrict__ head_group, int hg_stride,
    const int32_t *__restrict__ pattern_id, const int32_t *__restrict__ arow, const int32_t *__restrict__ n_act, int B,
    int nH, int nG, int L, int dh, int capA, h16 *__restrict__ Ac, const h16 *__restrict__ WoT, int64_t w_pstride,
    const h16 *__restrict__ bo, int d, float *__restrict__ cvec)
{
    if ((int)blockIdx.x < n_compact)
        att_compact_rows(blockIdx.x, att, ldo, slot, stats, head_group, hg_stride, pattern_id, arow, n_act, B, nH, nG, L,
                         dh, capA, Ac);
    else
        ctx_proj_rows(blockIdx.x - n_compact, stats, head_group, hg_stride, pattern_id, WoT, w_pstride, bo, B, nH, nG, dh,
                      d, cvec);
}

// The same in FP8 arithmetic: the context vector is quantised like every other row of the attention output,
// c[b, n] = (sum_k dec(E4M3(bf16(ctx_b[k]) * inv_sa)) dec(WoT8[p_b][n, k])) * out_scale + bo[n].
__global__ __launch_bounds__(256) void ctx_proj_q8_kernel(const float *__restrict__ stats, const int32_t *__restrict__ head_group,
                                                          int hg_stride, const int32_t *__restrict__ pattern_id,
                                                          const uint8_t *__restrict__ WoT8, int64_t w_pstride, int ldw,
                                                          const h16 *__restrict__ bo, int B, int nH, int nG, int dh,
                                                          int d, float inv_sa, float out_scale, float *__restrict__ cvec)
{
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= (int64_t)B * d) return;
    const int b = (int)(r / d), n = (int)(r % d);
    const int p = pattern_id ? pattern_id[b] : 0;
    const int K = nH * dh;
    const uint8_t *w = WoT8 + (int64_t)p * w_pstride + (int64_t)n * ldw;
    float acc = 0.f;
    for (int c = lane; c < K / 8; c += 64) {
        const int h = (c * 8) / dh, e0 = (c * 8) % dh;
        const h16x8 x = ctx8(stats, b, nG, head_group[(int64_t)p * hg_stride + h], dh, e0);
        const uint2 wv = *reinterpret_cast<const uint2 *>(w + c * 8);
        const uint32_t q0 = e4m3_pack4((float)x[0] * inv_sa, (float)x[1] * inv_sa, (float)x[2] * inv_sa, (float)x[3] * inv_sa);
        const uint32_t q1 = e4m3_pack4((float)x[4] * inv_sa, (float)x[5] * inv_sa, (float)x[6] * inv_sa, (float)x[7] * inv_sa);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            acc = fmaf(e4m3_value((q0 >> (8 * t)) & 0xFFu), e4m3_value((wv.x >> (8 * t)) & 0xFFu), acc);
            acc = fmaf(e4m3_value((q1 >> (8 * t)) & 0xFFu), e4m3_value((wv.y >> (8 * t)) & 0xFFu), acc);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) cvec[r] = acc * out_scale + (bo ? (float)bo[n] : 0.f);
}

// One wave per token row: x1 = x + (row active ? Cc[b, pos] + bo : c_b), written as fp32, then the LayerNorm of x1
// (statistics in fp32, biased variance) written as bf16, or (Q8) as E4M3 codes of LN(x1) * q_inv for an FFN in FP8
// arithmetic.  d % 8 == 0, d <= 512 * NCH.
template <class TI, int NCH, bool Q8>
__global__ __launch_bounds__(256) void combine_ln_kernel(const TI *__restrict__ x, const int32_t *__restrict__ pos_of,
                                                         const float *__restrict__ Cc, const h16 *__restrict__ bo,
                                                         const float *__restrict__ cvec, int L, int capA,
                                                         const h16 *__restrict__ gamma, const h16 *__restrict__ beta,
                                                         float eps, int64_t rows, int d, float *__restrict__ x1,
                                                         void *__restrict__ xn_out, float q_inv)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int64_t b = row / L;
    const int j = pos_of[row];
    const float *add = j >= 0 ? Cc + (b * capA + j) * d : cvec + b * d;
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
            const f32x4 a0 = *reinterpret_cast<const f32x4 *>(add + ch * 8);
            const f32x4 a1 = *reinterpret_cast<const f32x4 *>(add + ch * 8 + 4);
            float bb[8];
            if (j >= 0 && bo) {
                const h16x8 t = *reinterpret_cast<const h16x8 *>(bo + ch * 8);
#pragma unroll
                for (int e = 0; e < 8; ++e) bb[e] = (float)t[e];
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) bb[e] = 0.f;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[c][e] += a0[e] + bb[e];
                v[c][4 + e] += a1[e] + bb[4 + e];
            }
            f32x4 o0, o1;
#pragma unroll
            for (int e = 0; e < 4; ++e) { o0[e] = v[c][e]; o1[e] = v[c][4 + e]; }
            __builtin_nontemporal_store(o0, reinterpret_cast<f32x4 *>(x1 + row * d + ch * 8));
            __builtin_nontemporal_store(o1, reinterpret_cast<f32x4 *>(x1 + row * d + ch * 8 + 4));
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
        h16x8 gm, bt, o;
        float z[8];
        if (gamma) gm = *reinterpret_cast<const h16x8 *>(gamma + ch * 8);
        if (beta) bt = *reinterpret_cast<const h16x8 *>(beta + ch * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            z[e] = (v[c][e] - mean) * inv;
            if (gamma) z[e] *= (float)gm[e];
            if (beta) z[e] += (float)bt[e];
            o[e] = (h16)z[e];
        }
        if constexpr (Q8) {
            uint2 q;
            q.x = e4m3_pack4(z[0] * q_inv, z[1] * q_inv, z[2] * q_inv, z[3] * q_inv);
            q.y = e4m3_pack4(z[4] * q_inv, z[5] * q_inv, z[6] * q_inv, z[7] * q_inv);
            *reinterpret_cast<uint2 *>(static_cast<uint8_t *>(xn_out) + row * d + ch * 8) = q;
        } else {
            *reinterpret_cast<h16x8 *>(static_cast<h16 *>(xn_out) + row * d + ch * 8) = o;
        }
    }
}

}  // namespace

// Rows per sample of the compact buffers (a multiple of 128: the GEMM takes them as 128-row blocks), or 0 when the
// shortcut does not apply: it needs the sparse pattern, 16-byte rows, and at most a quarter of the rows can be active
// (measured: with half of the rows in the compact projection the extra passes cost more than the projection saves).
int lazy_cap(int L, int nH, int U, int dh, int d)
{
    if (U <= 0 || U >= L || L > 16384 || dh % 8 || d % 8 || d > 2048) return 0;
    const int64_t cap = (int64_t)align_up((size_t)nH * U, 128);
    if (cap * 4 > L) return 0;
    return (int)cap;
}

void lazy_rows_active(const uint32_t *act_bits, const int32_t *pattern_id, int B, int L, int capA, int32_t *arow,
                      int32_t *pos_of, int32_t *n_act, int32_t *blk_pattern, hipStream_t st)
{
    hipLaunchKernelGGL(rows_active_kernel, dim3(B), dim3(RA_NT), 0, st, act_bits, L, capA, pattern_id, arow, pos_of, n_act,
                       blk_pattern);
}

void lazy_att_compact(const void *att, int64_t ldo, const int32_t *slot, const float *stats, const int32_t *head_group,
                      int hg_stride, const int32_t *pattern_id, const int32_t *arow, const int32_t *n_act, int B, int nH,
                      int nG, int L, int dh, int capA, void *Ac, hipStream_t st)
{
    const int64_t rows = (int64_t)B * capA;
    hipLaunchKernelGGL(att_compact_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, (const h16 *)att, ldo,
                       slot, stats, head_group, hg_stride, pattern_id, arow, n_act, B, nH, nG, L, dh, capA, (h16 *)Ac);
}

void lazy_att_compact_ctx_proj(const void *att, int64_t ldo, const int32_t *slot, const float *stats,
                               const int32_t *head_group, int hg_stride, const int32_t *pattern_id, const int32_t *arow,
                               const int32_t *n_act, int B, int nH, int nG, int L, int dh, int capA, void *Ac,
                               const void *WoT, int64_t w_pstride, const void *bo, int d, float *cvec, hipStream_t st)
{
    const int64_t n_compact = ((int64_t)B * capA + 3) / 4, n_proj = ((int64_t)B * d + 3) / 4;
    hipLaunchKernelGGL(att_compact_ctx_proj_kernel, dim3((unsigned)(n_compact + n_proj)), dim3(256), 0, st, (int)n_compact,
                       (const h16 *)att, ldo, slot, stats, head_group, hg_stride, pattern_id, arow, n_act, B, nH, nG, L, dh,
                       capA, (h16 *)Ac, (const h16 *)WoT, w_pstride, (const h16 *)bo, d, cvec);
}

void lazy_ctx_proj_q8(const float *stats, const int32_t *head_group, int hg_stride, const int32_t *pattern_id,
                      const void *WoT8, int64_t w_pstride, int ldw, const void *bo, int B, int nH, int nG, int dh, int d,
                      float inv_sa, float out_scale, float *cvec, hipStream_t st)
{
    const int64_t rows = (int64_t)B * d;
    hipLaunchKernelGGL(ctx_proj_q8_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, stats, head_group, hg_stride,
                       pattern_id, (const uint8_t *)WoT8, w_pstride, ldw, (const h16 *)bo, B, nH, nG, dh, d, inv_sa, out_scale,
                       cvec);
}

void lazy_combine_ln(const void *x, bool x_f32, const int32_t *pos_of, const float *Cc, const void *bo, const float *cvec,
                     int B, int L, int capA, const void *gamma, const void *beta, float eps, int d, float *x1, void *xn,
                     float q_inv, hipStream_t st)
{
    // q_inv > 0: xn receives E4M3 codes of LN(x1) * q_inv (one byte per element) instead of bf16
    const int64_t rows = (int64_t)B * L;
    dim3 grid((unsigned)((rows + 3) / 4));
#define SF_CLN_ARGS(TI) grid, dim3(256), 0, st, (const TI *)x, pos_of, Cc, (const h16 *)bo, cvec, L, capA, \
                        (const h16 *)gamma, (const h16 *)beta, eps, rows, d, x1, xn, q_inv
#define SF_CLN_LAUNCH(TI, Q)                                                                            \
    do {                                                                                                \
        if (d <= 512) hipLaunchKernelGGL((combine_ln_kernel<TI, 1, Q>), SF_CLN_ARGS(TI));               \
        else if (d <= 1024) hipLaunchKernelGGL((combine_ln_kernel<TI, 2, Q>), SF_CLN_ARGS(TI));         \
        else hipLaunchKernelGGL((combine_ln_kernel<TI, 4, Q>), SF_CLN_ARGS(TI));                        \
    } while (0)
    if (q_inv > 0.f) {
        if (x_f32) SF_CLN_LAUNCH(float, true); else SF_CLN_LAUNCH(h16, true);
    } else {
        if (x_f32) SF_CLN_LAUNCH(float, false); else SF_CLN_LAUNCH(h16, false);
    }
#undef SF_CLN_LAUNCH
#undef SF_CLN_ARGS
}

}  // namespace sf
