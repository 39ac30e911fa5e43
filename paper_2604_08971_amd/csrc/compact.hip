// compact_heads_channels: gather the kept head blocks / FFN channels of the
// dense weights into padded dense buffers (Sec. 4.5: column blocks of W_Q for
// H_keep, the matching K/V group blocks, W1' = W1[:, N_keep],
// W2' = W2[N_keep, :]).  Pure data movement; HBM-bound.
#include "common.hpp"

namespace sf {

// One launch gathers up to 4 "regions".  Region g: dst_g[p, R, :] = src_g[idx_g[p, R / block] * block +
// R % block, :] for R < rows (zeros when the slot is unused); pattern p's rows start dst_pstride VECs
// after pattern p-1's (so a region can be part of a larger per-pattern buffer).  All regions of a
// launch share the row length.  One block per output row; VEC-typed copies.
struct GatherRegion {
    const void *src; void *dst; const int32_t *idx; const int32_t *n_dev;
    int idx_stride, block, n_static, rows; size_t dst_pstride;
};
struct GatherRegions { GatherRegion r[4]; int n; };

template <class VEC>
__global__ __launch_bounds__(256) void gather_rows_kernel(GatherRegions regs, int row_vecs)
{
    const int p = blockIdx.y;
    int R = blockIdx.x, g = 0;
    while (g + 1 < regs.n && R >= regs.r[g].rows) { R -= regs.r[g].rows; ++g; }
    const GatherRegion &rg = regs.r[g];
    const int slot = R / rg.block, r = R % rg.block;
    const int n_valid = rg.n_dev ? rg.n_dev[p] : rg.n_static;
    int src_unit = -1;
    if (slot < n_valid) src_unit = rg.idx[(size_t)p * rg.idx_stride + slot];
    VEC *d = static_cast<VEC *>(rg.dst) + (size_t)p * rg.dst_pstride + (size_t)R * row_vecs;
    if (src_unit < 0) {
        VEC z{};
        for (int i = threadIdx.x; i < row_vecs; i += blockDim.x) d[i] = z;
    } else {
        const VEC *s = static_cast<const VEC *>(rg.src) + ((size_t)src_unit * rg.block + r) * row_vecs;
        for (int i = threadIdx.x; i < row_vecs; i += blockDim.x) d[i] = s[i];
    }
}

// dstT[p * dst_pstride + n * cols_out + J] = src[idx[p, J / block] * block + J % block, n]  for n < d,
// J < cols_out (zeros when the slot is unused).  32x32 tiles through LDS so
// both the reads (along n) and the writes (along J) are contiguous.
template <class T>
__global__ __launch_bounds__(256) void gather_transpose_kernel(
    const T *__restrict__ src, T *__restrict__ dstT, const int32_t *__restrict__ idx,
    int idx_stride, int block, int n_valid, int cols_out, int d, size_t dst_pstride)
{
    __shared__ T tile[32][33];
    const int p = blockIdx.z;
    const int J0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    for (int jj = ty; jj < 32; jj += 8) {
        const int J = J0 + jj, n = n0 + tx;
        T v = T(0);
        if (J < cols_out && n < d) {
            const int slot = J / block;
            const int unit = slot < n_valid ? idx[(size_t)p * idx_stride + slot] : -1;
            if (unit >= 0) v = src[((size_t)unit * block + J % block) * d + n];
        }
        tile[jj][tx] = v;
    }
    __syncthreads();
    for (int nn = ty; nn < 32; nn += 8) {
        const int n = n0 + nn, J = J0 + tx;
        if (n < d && J < cols_out) dstT[(size_t)p * dst_pstride + (size_t)n * cols_out + J] = tile[tx][nn];
    }
}

// One launch for a whole layer when every weight row is a multiple of 16 bytes: blockIdx.x selects the job -
// blocks of CL_ROWS weight rows (regions of wr; a wave moves two rows, both loads in flight before the stores),
// then blocks of 256 bias elements (regions of br), then the tiles of the two transposed gathers; blockIdx.y is
// the pattern.  Four launches of a few microseconds each became one.
struct TransposeJob {
    const void *src; void *dst; const int32_t *idx;
    int idx_stride, block, n_valid, cols_out, tiles_j, tiles_n; size_t dst_pstride;
};
struct LayerJobs {
    GatherRegions wr; int n_rows, row_vecs, row_blocks;   // dst_pstride in uint4
    GatherRegions br; int n_bias, bias_blocks;            // dst_pstride in elements
    TransposeJob tr[2]; int d, tr_tile;                   // tr_tile: 64 (16-bit types, 16-byte accesses) or 32
};
constexpr int CL_ROWS = 8;

template <class T>
__global__ __launch_bounds__(256) void compact_layer_kernel(LayerJobs J)
{
    __shared__ T tile[sizeof(T) == 2 ? 64 : 32][sizeof(T) == 2 ? 66 : 33];
    const int p = blockIdx.y;
    int x = blockIdx.x;
    if (x < J.row_blocks) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const uint4 *sv[2] = {nullptr, nullptr};
        uint4 *dv[2] = {nullptr, nullptr};
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            int R = x * CL_ROWS + wave * 2 + k, g = 0;
            if (R >= J.n_rows) continue;
            while (g + 1 < J.wr.n && R >= J.wr.r[g].rows) { R -= J.wr.r[g].rows; ++g; }
            const GatherRegion &rg = J.wr.r[g];
            const int slot = R / rg.block, r = R % rg.block;
            const int n_valid = rg.n_dev ? rg.n_dev[p] : rg.n_static;
            int src_unit = -1;
            if (slot < n_valid) src_unit = rg.idx[(size_t)p * rg.idx_stride + slot];
            dv[k] = static_cast<uint4 *>(rg.dst) + (size_t)p * rg.dst_pstride + (size_t)R * J.row_vecs;
            if (src_unit >= 0) sv[k] = static_cast<const uint4 *>(rg.src) + ((size_t)src_unit * rg.block + r) * J.row_vecs;
        }
        for (int i = lane; i < J.row_vecs; i += 64) {
            uint4 v[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) v[k] = sv[k] ? sv[k][i] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int k = 0; k < 2; ++k)
                if (dv[k]) dv[k][i] = v[k];
        }
        return;
    }
    x -= J.row_blocks;
    if (x < J.bias_blocks) {
        int R = x * 256 + threadIdx.x;
        if (R >= J.n_bias) return;
        int g = 0;
        while (g + 1 < J.br.n && R >= J.br.r[g].rows) { R -= J.br.r[g].rows; ++g; }
        const GatherRegion &rg = J.br.r[g];
        const int slot = R / rg.block, r = R % rg.block;
        const int n_valid = rg.n_dev ? rg.n_dev[p] : rg.n_static;
        T v = T(0);
        if (slot < n_valid) {
            const int unit = rg.idx[(size_t)p * rg.idx_stride + slot];
            if (unit >= 0) v = static_cast<const T *>(rg.src)[(size_t)unit * rg.block + r];
        }
        static_cast<T *>(rg.dst)[(size_t)p * rg.dst_pstride + R] = v;
        return;
    }
    x -= J.bias_blocks;
    int t = 0;
    if (x >= J.tr[0].tiles_j * J.tr[0].tiles_n) { x -= J.tr[0].tiles_j * J.tr[0].tiles_n; t = 1; }
    const TransposeJob &tj = J.tr[t];
    const T *src = static_cast<const T *>(tj.src);
    T *dstT = static_cast<T *>(tj.dst);
    if constexpr (sizeof(T) == 2) {
        if (J.tr_tile == 64) {
            // 64 unit rows x 64 features through LDS, 16 bytes per lane on both sides: 8 features of a unit row on
            // the way in, 8 unit rows of a feature on the way out (d, cols_out multiples of 8, 16-byte aligned)
            const int J0 = (x % tj.tiles_j) * 64, n0 = (x / tj.tiles_j) * 64;
            const int ch = threadIdx.x & 7, r = threadIdx.x >> 3;      // 8 chunks x 32 rows per pass
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
                const int jj = r + pass * 32, Jc = J0 + jj, n = n0 + ch * 8;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (Jc < tj.cols_out && n < J.d) {
                    const int slot = Jc / tj.block;
                    const int unit = slot < tj.n_valid ? tj.idx[(size_t)p * tj.idx_stride + slot] : -1;
                    if (unit >= 0) v = *reinterpret_cast<const uint4 *>(src + ((size_t)unit * tj.block + Jc % tj.block) * J.d + n);
                }
                uint32_t *w = reinterpret_cast<uint32_t *>(&tile[jj][ch * 8]);
                w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
            }
            __syncthreads();
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
                const int nn = r + pass * 32, n = n0 + nn, Jc = J0 + ch * 8;
                if (n >= J.d || Jc >= tj.cols_out) continue;
                uint32_t w[4];
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    w[k] = (uint32_t)tile[ch * 8 + 2 * k][nn] | ((uint32_t)tile[ch * 8 + 2 * k + 1][nn] << 16);
                *reinterpret_cast<uint4 *>(dstT + (size_t)p * tj.dst_pstride + (size_t)n * tj.cols_out + Jc) =
                    make_uint4(w[0], w[1], w[2], w[3]);
            }
            return;
        }
    }
    const int J0 = (x % tj.tiles_j) * 32, n0 = (x / tj.tiles_j) * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    for (int jj = ty; jj < 32; jj += 8) {
        const int Jc = J0 + jj, n = n0 + tx;
        T v = T(0);
        if (Jc < tj.cols_out && n < J.d) {
            const int slot = Jc / tj.block;
            const int unit = slot < tj.n_valid ? tj.idx[(size_t)p * tj.idx_stride + slot] : -1;
            if (unit >= 0) v = src[((size_t)unit * tj.block + Jc % tj.block) * J.d + n];
        }
        tile[jj][tx] = v;
    }
    __syncthreads();
    for (int nn = ty; nn < 32; nn += 8) {
        const int n = n0 + nn, Jc = J0 + tx;
        if (n < J.d && Jc < tj.cols_out) dstT[(size_t)p * tj.dst_pstride + (size_t)n * tj.cols_out + Jc] = tile[tx][nn];
    }
}

// regs.r[g].dst_pstride is given in ROWS here and converted to VECs
static void gather_rows(hipStream_t st, GatherRegions regs, size_t row_bytes, int P)
{
    int rows = 0;
    bool a16 = row_bytes % 16 == 0;
    for (int g = 0; g < regs.n; ++g) {
        rows += regs.r[g].rows;
        a16 = a16 && ((uintptr_t)regs.r[g].src % 16 == 0) && ((uintptr_t)regs.r[g].dst % 16 == 0);
    }
    dim3 grid(rows, P);
    const size_t unit = a16 ? 16 : (row_bytes % 4 == 0 ? 4 : 2);
    for (int g = 0; g < regs.n; ++g) regs.r[g].dst_pstride = regs.r[g].dst_pstride * row_bytes / unit;
    const int rv = (int)(row_bytes / unit);
    if (unit == 16) {
        const int nt = rv >= 256 ? 256 : (rv >= 128 ? 128 : 64);
        hipLaunchKernelGGL(gather_rows_kernel<uint4>, grid, dim3(nt), 0, st, regs, rv);
    } else if (unit == 4) {
        hipLaunchKernelGGL(gather_rows_kernel<uint32_t>, grid, dim3(64), 0, st, regs, rv);
    } else {
        hipLaunchKernelGGL(gather_rows_kernel<uint16_t>, grid, dim3(64), 0, st, regs, rv);
    }
}

static void gather_transpose(hipStream_t st, int dtype, const void *src, void *dst,
                             const int32_t *idx, int idx_stride, int block, int n_valid,
                             int cols_out, int d, int P, size_t dst_pstride = 0)
{
    if (dst_pstride == 0) dst_pstride = (size_t)d * cols_out;
    dim3 grid(ceil_div(cols_out, 32), ceil_div(d, 32), P);
    if (dtype == SF_BF16)
        hipLaunchKernelGGL(gather_transpose_kernel<uint16_t>, grid, dim3(256), 0, st,
                           (const uint16_t *)src, (uint16_t *)dst, idx, idx_stride, block, n_valid,
                           cols_out, d, dst_pstride);
    else
        hipLaunchKernelGGL(gather_transpose_kernel<uint32_t>, grid, dim3(256), 0, st,
                           (const uint32_t *)src, (uint32_t *)dst, idx, idx_stride, block, n_valid,
                           cols_out, d, dst_pstride);
}

// ---- FP8 (OCP E4M3) weight storage: the same gathers, reading one byte per element and writing
// decode(byte) * scale rounded once to the model dtype (the product of a 4-bit and a 24-bit significand is
// exact in double).
__device__ inline double fp8_e4m3_value(uint32_t b)
{
    const uint32_t e = (b >> 3) & 15u, m = b & 7u;
    float v;
    if (e == 15u && m == 7u) v = __uint_as_float(0x7fc00000u);               // the only non-finite code
    else if (e == 0u) v = (float)m * 0x1p-9f;                                // subnormal
    else v = __uint_as_float(((e + 120u) << 23) | (m << 20));                // (1 + m/8) * 2^(e-7)
    return (b & 0x80u) ? -(double)v : (double)v;
}

// IEEE binary16 bit pattern -> value (every binary16 value is an fp32 value)
__device__ inline double f16_value(uint32_t bits)
{
    const uint16_t h = (uint16_t)bits;
    return (double)(float)__builtin_bit_cast(_Float16, h);
}

// value of one stored code: S = uint8_t is E4M3, S = uint16_t is binary16
template <class S> __device__ inline double code_value(uint32_t c)
{
    if constexpr (sizeof(S) == 1) return fp8_e4m3_value(c);
    else return f16_value(c);
}

template <class T> __device__ inline T round_from_double(double x);
template <> __device__ inline float round_from_double<float>(double x) { return (float)x; }
template <> __device__ inline uint16_t round_from_double<uint16_t>(double x)      // bf16 bits, ties to even
{
    // double -> fp32 towards zero with the lost bits folded into the last bit (round to odd) keeps every
    // tie / non-tie decision of the following 16-bit rounding
    float f = __double2float_rz(x);
    uint32_t u = __float_as_uint(f);
    if ((double)f != x && x == x) u |= 1u;
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

struct Fp8Region {
    const void *src; void *dst; const int32_t *idx; const int32_t *n_dev;
    int idx_stride, block, n_static, rows; size_t dst_pstride /* elements */; float scale;
};
struct Fp8Regions { Fp8Region r[4]; int n; };

// as gather_rows_kernel, rows of row_len elements (a multiple of 4); a thread converts 4 elements at a time
template <class T, class S>
__global__ __launch_bounds__(256) void gather_rows_fp8_kernel(Fp8Regions regs, int row_len)
{
    const int p = blockIdx.y;
    int R = blockIdx.x, g = 0;
    while (g + 1 < regs.n && R >= regs.r[g].rows) { R -= regs.r[g].rows; ++g; }
    const Fp8Region &rg = regs.r[g];
    const int slot = R / rg.block, r = R % rg.block;
    const int n_valid = rg.n_dev ? rg.n_dev[p] : rg.n_static;
    int src_unit = -1;
    if (slot < n_valid) src_unit = rg.idx[(size_t)p * rg.idx_stride + slot];
    T *d = static_cast<T *>(rg.dst) + (size_t)p * rg.dst_pstride + (size_t)R * row_len;
    const S *s = static_cast<const S *>(rg.src) + ((size_t)(src_unit < 0 ? 0 : src_unit) * rg.block + r) * row_len;
    const double sc = (double)rg.scale;
    constexpr int SB = 8 * sizeof(S);
    for (int i = threadIdx.x * 4; i < row_len; i += blockDim.x * 4) {
        uint64_t w = 0u;                                       // four codes
        if (src_unit >= 0) {
            if constexpr (sizeof(S) == 1) w = *reinterpret_cast<const uint32_t *>(s + i);
            else w = *reinterpret_cast<const uint64_t *>(s + i);
        }
        struct alignas(sizeof(T) * 4) Pack { T v[4]; } o;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o.v[e] = src_unit < 0 ? T(0)
                                  : round_from_double<T>(code_value<S>((uint32_t)(w >> (SB * e)) & ((1u << SB) - 1u)) * sc);
        *reinterpret_cast<Pack *>(d + i) = o;
    }
}

// as gather_transpose_kernel with an FP8 source
template <class T, class S>
__global__ __launch_bounds__(256) void gather_transpose_fp8_kernel(
    const S *__restrict__ src, T *__restrict__ dstT, const int32_t *__restrict__ idx,
    int idx_stride, int block, int n_valid, int cols_out, int d, size_t dst_pstride, float scale)
{
    __shared__ T tile[32][33];
    const int p = blockIdx.z;
    const int J0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    for (int jj = ty; jj < 32; jj += 8) {
        const int J = J0 + jj, n = n0 + tx;
        T v = T(0);
        if (J < cols_out && n < d) {
            const int slot = J / block;
            const int unit = slot < n_valid ? idx[(size_t)p * idx_stride + slot] : -1;
            if (unit >= 0)
                v = round_from_double<T>(code_value<S>(src[((size_t)unit * block + J % block) * d + n]) * (double)scale);
        }
        tile[jj][tx] = v;
    }
    __syncthreads();
    for (int nn = ty; nn < 32; nn += 8) {
        const int n = n0 + nn, J = J0 + tx;
        if (n < d && J < cols_out) dstT[(size_t)p * dst_pstride + (size_t)n * cols_out + J] = tile[tx][nn];
    }
}

struct ExpertCounts { int32_t k[64]; };
__global__ void store_expert_counts_kernel(ExpertCounts ec, int E, int32_t *__restrict__ out)
{
    if ((int)threadIdx.x < E) out[threadIdx.x] = ec.k[threadIdx.x];
}

}  // namespace sf

using namespace sf;

extern "C" int32_t sf_compact_heads_channels(const sf_desc *desc, int32_t layer,
                                             const sf_dense_layer *dense,
                                             const int32_t *head_idx, const int32_t *group_idx,
                                             const int32_t *n_groups, const int32_t *ffn_idx,
                                             const sf_compact_layer *c, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!dense || !c || !head_idx || !group_idx || !n_groups || !ffn_idx)
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels: NULL argument");
    if (layer < 0 || layer >= D.nl)
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels: layer %d out of range", layer);
    if (c->k_head < 1 || c->k_head > D.Hq || c->k_ffn < 1 || c->k_ffn > D.F)
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels: keep counts out of range");
    if (!dense->Wq || !dense->Wk || !dense->Wv || !dense->Wo || !dense->W1 || !dense->W2 ||
        !c->Wqkv || !c->WoT || !c->W1 || !c->W2T)
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels: NULL weight pointer");
    const bool qkv_bias = dense->bq || dense->bk || dense->bv;
    if (qkv_bias && !(dense->bq && dense->bk && dense->bv))
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels: bq, bk, bv must be all set or all NULL");
    if ((qkv_bias && !c->bqkv) || (dense->b1 && !c->b1))
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels: compact bias buffer missing");

    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t es = elem_size(D.dtype);
    const int P = D.P, dh = D.dh, d = D.d, kh = c->k_head, kf = c->k_ffn;
    const int Fp = (int)align_up(kf, D.ffn_pad);
    const int Nqkv = (kh + 2 * D.Hk) * dh;
    const int32_t *hi = head_idx + (size_t)layer * P * D.Hq;
    const int32_t *gi = group_idx + (size_t)layer * P * D.Hk;
    const int32_t *ng = n_groups + (size_t)layer * P;
    const int32_t *fi = ffn_idx + (size_t)layer * P * D.F;

    // One launch for all weight rows and one for all bias entries: the three row regions of
    // Wqkv [P, Nqkv, d] (kept Q heads, K group slots, V group slots) and W1' (+ zero pad rows).
    auto region = [&](const void *src, void *dst, size_t elem_off, const int32_t *idx, int idx_stride, int block,
                      int n_static, const int32_t *n_dev, int rows, size_t rows_per_pattern, size_t row_bytes) {
        GatherRegion r{};
        r.src = src; r.dst = (char *)dst + elem_off * row_bytes; r.idx = idx; r.n_dev = n_dev;
        r.idx_stride = idx_stride; r.block = block; r.n_static = n_static; r.rows = rows;
        r.dst_pstride = rows_per_pattern;
        return r;
    };
    const size_t rowW = (size_t)d * es;
    GatherRegions wr{};
    wr.r[0] = region(dense->Wq, c->Wqkv, 0, hi, D.Hq, dh, kh, nullptr, kh * dh, Nqkv, rowW);
    wr.r[1] = region(dense->Wk, c->Wqkv, (size_t)kh * dh, gi, D.Hk, dh, 0, ng, D.Hk * dh, Nqkv, rowW);
    wr.r[2] = region(dense->Wv, c->Wqkv, (size_t)(kh + D.Hk) * dh, gi, D.Hk, dh, 0, ng, D.Hk * dh, Nqkv, rowW);
    wr.r[3] = region(dense->W1, c->W1, 0, fi, D.F, 1, kf, nullptr, Fp, Fp, rowW);
    wr.n = 4;
    GatherRegions br{};
    if (qkv_bias) {
        br.r[br.n++] = region(dense->bq, c->bqkv, 0, hi, D.Hq, dh, kh, nullptr, kh * dh, Nqkv, es);
        br.r[br.n++] = region(dense->bk, c->bqkv, (size_t)kh * dh, gi, D.Hk, dh, 0, ng, D.Hk * dh, Nqkv, es);
        br.r[br.n++] = region(dense->bv, c->bqkv, (size_t)(kh + D.Hk) * dh, gi, D.Hk, dh, 0, ng, D.Hk * dh, Nqkv, es);
    }
    if (dense->b1) br.r[br.n++] = region(dense->b1, c->b1, 0, fi, D.F, 1, kf, nullptr, Fp, Fp, es);
    bool aligned = rowW % 16 == 0 && P <= 65535;
    for (int g = 0; g < wr.n; ++g)
        aligned = aligned && ((uintptr_t)wr.r[g].src % 16 == 0) && ((uintptr_t)wr.r[g].dst % 16 == 0);
    if (aligned) {
        // everything in one launch (weight rows, bias elements, the two transposed gathers)
        LayerJobs J{};
        J.wr = wr; J.row_vecs = (int)(rowW / 16);
        for (int g = 0; g < wr.n; ++g) { J.n_rows += wr.r[g].rows; J.wr.r[g].dst_pstride = wr.r[g].dst_pstride * J.row_vecs; }
        J.br = br;
        for (int g = 0; g < br.n; ++g) J.n_bias += br.r[g].rows;
        J.bias_blocks = ceil_div(J.n_bias, 256);
        J.row_blocks = ceil_div(J.n_rows, CL_ROWS);
        J.d = d;
        // W2'^T and Wo'^T: unit rows become columns so the GEMMs read K-contiguous operands
        const bool wide = D.dtype == SF_BF16 && d % 8 == 0 && Fp % 8 == 0 && (kh * dh) % 8 == 0 &&
                          !(((uintptr_t)dense->W2 | (uintptr_t)dense->Wo | (uintptr_t)c->W2T | (uintptr_t)c->WoT) & 15);
        const int tt = wide ? 64 : 32;
        J.tr_tile = tt;
        J.tr[0] = TransposeJob{dense->W2, c->W2T, fi, D.F, 1, kf, Fp, ceil_div(Fp, tt), ceil_div(d, tt), (size_t)d * Fp};
        J.tr[1] = TransposeJob{dense->Wo, c->WoT, hi, D.Hq, dh, kh, kh * dh, ceil_div(kh * dh, tt), ceil_div(d, tt),
                               (size_t)d * kh * dh};
        dim3 grid(J.row_blocks + J.bias_blocks + J.tr[0].tiles_j * J.tr[0].tiles_n + J.tr[1].tiles_j * J.tr[1].tiles_n, P);
        if (D.dtype == SF_BF16) hipLaunchKernelGGL(compact_layer_kernel<uint16_t>, grid, dim3(256), 0, st, J);
        else hipLaunchKernelGGL(compact_layer_kernel<uint32_t>, grid, dim3(256), 0, st, J);
        return check_launch("compact_heads_channels");
    }
    gather_rows(st, wr, rowW, P);
    if (br.n) gather_rows(st, br, es, P);
    gather_transpose(st, D.dtype, dense->W2, c->W2T, fi, D.F, 1, kf, Fp, d, P);
    gather_transpose(st, D.dtype, dense->Wo, c->WoT, hi, D.Hq, dh, kh, kh * dh, d, P);
    return check_launch("compact_heads_channels");
}

// Sparse-MoE FFN pruning (Sec. 4.5): every expert keeps its own channel set; the compact buffers are padded
// to the widest expert (zero channels contribute exactly zero).
extern "C" int32_t sf_compact_moe_experts(const sf_desc *desc, const sf_moe_dense *dense,
                                          const int32_t *ffn_idx, const int32_t *k_ffn_host,
                                          const sf_moe_compact *c, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!dense || !c || !ffn_idx || !k_ffn_host) return fail(SF_ERR_INVALID_ARG, "compact_moe_experts: NULL argument");
    const int E = c->n_experts;
    if (E < 1 || E > 64 || c->top_k < 1 || c->top_k > E || c->top_k > 8)
        return fail(SF_ERR_INVALID_ARG, "compact_moe_experts: needs 1 <= top_k <= min(8, n_experts), n_experts <= 64");
    int kmax = 0;
    for (int e = 0; e < E; ++e) {
        if (k_ffn_host[e] < 1 || k_ffn_host[e] > D.F)
            return fail(SF_ERR_INVALID_ARG, "compact_moe_experts: keep count of expert %d out of range", e);
        if (k_ffn_host[e] > kmax) kmax = k_ffn_host[e];
    }
    if (c->k_ffn_max != kmax) return fail(SF_ERR_INVALID_ARG, "compact_moe_experts: k_ffn_max must be %d", kmax);
    if (!dense->W1 || !dense->W2 || !c->W1 || !c->W2T || !c->k_ffn || (dense->b1 && !c->b1) || (dense->b2 && !c->b2x))
        return fail(SF_ERR_INVALID_ARG, "compact_moe_experts: NULL weight pointer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t es = elem_size(D.dtype);
    const int P = D.P, d = D.d, F = D.F;
    const int Fp = (int)align_up(kmax, D.ffn_pad);
    const size_t rowW = (size_t)d * es;
    for (int e0 = 0; e0 < E; e0 += 4) {          // up to four experts per launch
        GatherRegions wr{}, br{};
        for (int e = e0; e < E && e < e0 + 4; ++e) {
            const int32_t *fi = ffn_idx + (size_t)e * P * F;
            GatherRegion r{};
            r.src = (const char *)dense->W1 + (size_t)e * F * rowW; r.dst = (char *)c->W1 + (size_t)e * Fp * rowW;
            r.idx = fi; r.idx_stride = F; r.block = 1; r.n_static = k_ffn_host[e]; r.rows = Fp;
            r.dst_pstride = (size_t)E * Fp;
            wr.r[wr.n++] = r;
            if (dense->b1) {
                GatherRegion q = r;
                q.src = (const char *)dense->b1 + (size_t)e * F * es; q.dst = (char *)c->b1 + (size_t)e * Fp * es;
                br.r[br.n++] = q;
            }
        }
        gather_rows(st, wr, rowW, P);
        if (br.n) gather_rows(st, br, es, P);
    }
    for (int e = 0; e < E; ++e)
        gather_transpose(st, D.dtype, (const char *)dense->W2 + (size_t)e * F * rowW,
                         (char *)c->W2T + (size_t)e * d * Fp * es, ffn_idx + (size_t)e * P * F, F, 1, k_ffn_host[e],
                         Fp, d, P, (size_t)E * d * Fp);
    {                                              // keep counts to the device as kernel arguments (no host copy)
        ExpertCounts ec{};
        for (int e = 0; e < E; ++e) ec.k[e] = k_ffn_host[e];
        hipLaunchKernelGGL(store_expert_counts_kernel, dim3(1), dim3(64), 0, st, ec, E, c->k_ffn);
    }
    if (dense->b2)                                 // b2x[p, e, :] = b2[e, :]
        for (int p = 0; p < P; ++p)
            if (hipMemcpyAsync((char *)c->b2x + (size_t)p * E * rowW, dense->b2, (size_t)E * rowW,
                               hipMemcpyDeviceToDevice, st) != hipSuccess)
                return fail(SF_ERR_HIP, "compact_moe_experts: copy of b2 failed");
    return check_launch("compact_moe_experts");
}

// Dense weights stored as codes - S = uint8_t: OCP E4M3 bytes + one fp32 scale per matrix, S = uint16_t: IEEE
// binary16, scale 1: gather and dequantise in one pass.
template <class S>
static int32_t compact_coded(const sf_desc *desc, int32_t layer, const sf_dense_layer_fp8 *dense,
                             const int32_t *head_idx, const int32_t *group_idx,
                             const int32_t *n_groups, const int32_t *ffn_idx,
                             const sf_compact_layer *c, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!dense || !c || !head_idx || !group_idx || !n_groups || !ffn_idx)
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels_fp8: NULL argument");
    if (layer < 0 || layer >= D.nl)
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels_fp8: layer %d out of range", layer);
    if (c->k_head < 1 || c->k_head > D.Hq || c->k_ffn < 1 || c->k_ffn > D.F)
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels_fp8: keep counts out of range");
    if (!dense->Wq || !dense->Wk || !dense->Wv || !dense->Wo || !dense->W1 || !dense->W2 ||
        !c->Wqkv || !c->WoT || !c->W1 || !c->W2T)
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels_fp8: NULL weight pointer");
    if (D.d % 4) return fail(SF_ERR_SHAPE, "compact_heads_channels_fp8: d_model must be a multiple of 4");
    if (((uintptr_t)dense->Wq | (uintptr_t)dense->Wk | (uintptr_t)dense->Wv | (uintptr_t)dense->W1) & (4 * sizeof(S) - 1))
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels_fp8: weight matrices must be %zu-byte aligned", 4 * sizeof(S));
    const bool qkv_bias = dense->bq || dense->bk || dense->bv;
    if (qkv_bias && !(dense->bq && dense->bk && dense->bv))
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels_fp8: bq, bk, bv must be all set or all NULL");
    if ((qkv_bias && !c->bqkv) || (dense->b1 && !c->b1))
        return fail(SF_ERR_INVALID_ARG, "compact_heads_channels_fp8: compact bias buffer missing");

    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t es = elem_size(D.dtype);
    const bool bf = D.dtype == SF_BF16;
    const int P = D.P, dh = D.dh, d = D.d, kh = c->k_head, kf = c->k_ffn;
    const int Fp = (int)align_up(kf, D.ffn_pad);
    const int Nqkv = (kh + 2 * D.Hk) * dh;
    const int32_t *hi = head_idx + (size_t)layer * P * D.Hq;
    const int32_t *gi = group_idx + (size_t)layer * P * D.Hk;
    const int32_t *ng = n_groups + (size_t)layer * P;
    const int32_t *fi = ffn_idx + (size_t)layer * P * D.F;

    auto wreg = [&](const void *src, void *dst, size_t row_off, const int32_t *idx, int idx_stride, int block, int n_static,
                    const int32_t *n_dev, int rows, size_t rows_per_pattern, float scale) {
        Fp8Region r{};
        r.src = src; r.dst = (char *)dst + row_off * d * es; r.idx = idx; r.n_dev = n_dev;
        r.idx_stride = idx_stride; r.block = block; r.n_static = n_static; r.rows = rows;
        r.dst_pstride = rows_per_pattern * d; r.scale = scale;
        return r;
    };
    Fp8Regions wr{};
    wr.r[0] = wreg(dense->Wq, c->Wqkv, 0, hi, D.Hq, dh, kh, nullptr, kh * dh, Nqkv, dense->sq);
    wr.r[1] = wreg(dense->Wk, c->Wqkv, (size_t)kh * dh, gi, D.Hk, dh, 0, ng, D.Hk * dh, Nqkv, dense->sk);
    wr.r[2] = wreg(dense->Wv, c->Wqkv, (size_t)(kh + D.Hk) * dh, gi, D.Hk, dh, 0, ng, D.Hk * dh, Nqkv, dense->sv);
    wr.r[3] = wreg(dense->W1, c->W1, 0, fi, D.F, 1, kf, nullptr, Fp, Fp, dense->s1);
    wr.n = 4;
    {
        dim3 grid(kh * dh + 2 * D.Hk * dh + Fp, P);
        const int nt = d >= 1024 ? 256 : (d >= 512 ? 128 : 64);
        if (bf) hipLaunchKernelGGL((gather_rows_fp8_kernel<uint16_t, S>), grid, dim3(nt), 0, st, wr, d);
        else hipLaunchKernelGGL((gather_rows_fp8_kernel<float, S>), grid, dim3(nt), 0, st, wr, d);
    }
    // biases are stored in the model dtype: the plain gathers
    auto region = [&](const void *src, void *dst, size_t elem_off, const int32_t *idx, int idx_stride, int block,
                      int n_static, const int32_t *n_dev, int rows, size_t rows_per_pattern, size_t row_bytes) {
        GatherRegion r{};
        r.src = src; r.dst = (char *)dst + elem_off * row_bytes; r.idx = idx; r.n_dev = n_dev;
        r.idx_stride = idx_stride; r.block = block; r.n_static = n_static; r.rows = rows;
        r.dst_pstride = rows_per_pattern;
        return r;
    };
    GatherRegions br{};
    if (qkv_bias) {
        br.r[br.n++] = region(dense->bq, c->bqkv, 0, hi, D.Hq, dh, kh, nullptr, kh * dh, Nqkv, es);
        br.r[br.n++] = region(dense->bk, c->bqkv, (size_t)kh * dh, gi, D.Hk, dh, 0, ng, D.Hk * dh, Nqkv, es);
        br.r[br.n++] = region(dense->bv, c->bqkv, (size_t)(kh + D.Hk) * dh, gi, D.Hk, dh, 0, ng, D.Hk * dh, Nqkv, es);
    }
    if (dense->b1) br.r[br.n++] = region(dense->b1, c->b1, 0, fi, D.F, 1, kf, nullptr, Fp, Fp, es);
    if (br.n) gather_rows(st, br, es, P);
    auto transpose8 = [&](const void *src, void *dst, const int32_t *idx, int idx_stride, int block, int n_valid, int cols_out,
                          float scale) {
        dim3 grid(ceil_div(cols_out, 32), ceil_div(d, 32), P);
        const size_t ps = (size_t)d * cols_out;
        if (bf)
            hipLaunchKernelGGL((gather_transpose_fp8_kernel<uint16_t, S>), grid, dim3(256), 0, st, (const S *)src,
                               (uint16_t *)dst, idx, idx_stride, block, n_valid, cols_out, d, ps, scale);
        else
            hipLaunchKernelGGL((gather_transpose_fp8_kernel<float, S>), grid, dim3(256), 0, st, (const S *)src,
                               (float *)dst, idx, idx_stride, block, n_valid, cols_out, d, ps, scale);
    };
    transpose8(dense->W2, c->W2T, fi, D.F, 1, kf, Fp, dense->s2);
    transpose8(dense->Wo, c->WoT, hi, D.Hq, dh, kh, kh * dh, dense->so);
    return check_launch("compact_heads_channels_fp8");
}

extern "C" int32_t sf_compact_heads_channels_fp8(const sf_desc *desc, int32_t layer, const sf_dense_layer_fp8 *dense,
                                                 const int32_t *head_idx, const int32_t *group_idx,
                                                 const int32_t *n_groups, const int32_t *ffn_idx,
                                                 const sf_compact_layer *c, void *stream)
{
    // the single rounding from the exact product to a 16-bit model type is written for bfloat16
    if (SF_DTYPE_16 == SF_F16 && desc && desc->dtype == SF_F16)
        return fail(SF_ERR_UNSUPPORTED, "compact_heads_channels_fp8: E4M3-stored weights are built for fp32 and bfloat16 models");
    return compact_coded<uint8_t>(desc, layer, dense, head_idx, group_idx, n_groups, ffn_idx, c, stream);
}

// FP16-stored dense weights: the six matrices of `dense` hold IEEE binary16, everything else is in the model dtype.
extern "C" int32_t sf_compact_heads_channels_f16(const sf_desc *desc, int32_t layer, const sf_dense_layer *dense,
                                                 const int32_t *head_idx, const int32_t *group_idx,
                                                 const int32_t *n_groups, const int32_t *ffn_idx,
                                                 const sf_compact_layer *c, void *stream)
{
    if (!dense) return fail(SF_ERR_INVALID_ARG, "compact_heads_channels_f16: NULL argument");
    // a binary16 model stores these very bits: the plain gathers
    if (SF_DTYPE_16 == SF_F16 && desc && desc->dtype == SF_F16)
        return sf_compact_heads_channels(desc, layer, dense, head_idx, group_idx, n_groups, ffn_idx, c, stream);
    sf_dense_layer_fp8 q{};
    q.Wq = dense->Wq; q.Wk = dense->Wk; q.Wv = dense->Wv; q.Wo = dense->Wo; q.W1 = dense->W1; q.W2 = dense->W2;
    q.sq = q.sk = q.sv = q.so = q.s1 = q.s2 = 1.0f;
    q.bq = dense->bq; q.bk = dense->bk; q.bv = dense->bv; q.bo = dense->bo; q.b1 = dense->b1; q.b2 = dense->b2;
    q.ln1_g = dense->ln1_g; q.ln1_b = dense->ln1_b; q.ln2_g = dense->ln2_g; q.ln2_b = dense->ln2_b;
    return compact_coded<uint16_t>(desc, layer, &q, head_idx, group_idx, n_groups, ffn_idx, c, stream);
}

// FFN weights kept as E4M3 codes for the FP8 arithmetic path: the same gathers on bytes, nothing is decoded.
extern "C" int32_t sf_compact_ffn_fp8(const sf_desc *desc, int32_t layer, const sf_dense_layer_fp8 *dense,
                                      const int32_t *ffn_idx, const sf_ffn_fp8 *f, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!dense || !f || !ffn_idx) return fail(SF_ERR_INVALID_ARG, "compact_ffn_fp8: NULL argument");
    if (layer < 0 || layer >= D.nl) return fail(SF_ERR_INVALID_ARG, "compact_ffn_fp8: layer %d out of range", layer);
    if (f->k_ffn < 1 || f->k_ffn > D.F) return fail(SF_ERR_INVALID_ARG, "compact_ffn_fp8: k_ffn out of range");
    if (!dense->W1 || !dense->W2 || !f->W1q || !f->W2Tq)
        return fail(SF_ERR_INVALID_ARG, "compact_ffn_fp8: NULL weight pointer");
    if (dense->b1 && !f->b1) return fail(SF_ERR_INVALID_ARG, "compact_ffn_fp8: compact bias buffer missing");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t es = elem_size(D.dtype);
    const int P = D.P, d = D.d, kf = f->k_ffn;
    const int Fp8 = (int)align_up((size_t)kf, 128);
    const int32_t *fi = ffn_idx + (size_t)layer * P * D.F;
    auto region = [&](const void *src, void *dst) {
        GatherRegion r{};
        r.src = src; r.dst = dst; r.idx = fi; r.n_dev = nullptr;
        r.idx_stride = D.F; r.block = 1; r.n_static = kf; r.rows = Fp8;
        r.dst_pstride = (size_t)Fp8;
        return r;
    };
    GatherRegions wr{};
    wr.r[wr.n++] = region(dense->W1, f->W1q);
    gather_rows(st, wr, (size_t)d, P);
    if (dense->b1) {
        GatherRegions br{};
        br.r[br.n++] = region(dense->b1, f->b1);
        gather_rows(st, br, es, P);
    }
    dim3 grid(ceil_div(Fp8, 32), ceil_div(d, 32), P);
    hipLaunchKernelGGL(gather_transpose_kernel<uint8_t>, grid, dim3(256), 0, st, (const uint8_t *)dense->W2,
                       (uint8_t *)f->W2Tq, fi, D.F, 1, kf, Fp8, d, (size_t)d * Fp8);
    return check_launch("compact_ffn_fp8");
}

// Attention projection weights kept as E4M3 codes for the FP8 arithmetic path: Wqkv8 [P, (k_head + 2 Hk) dh, d]
// (kept Q heads, then the K and the V rows of the used groups, zero rows for unused group slots) and
// WoT8 [P, d, Kp] with Kp = k_head dh rounded up to 128 (zero columns: the FP8 GEMM contracts over multiples of 128),
// the same gathers as for the 16-bit weights on bytes.
extern "C" int32_t sf_compact_proj_fp8(const sf_desc *desc, int32_t layer, const sf_dense_layer_fp8 *dense,
                                       const int32_t *head_idx, const int32_t *group_idx, const int32_t *n_groups,
                                       const sf_proj_fp8 *pj, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!dense || !pj || !head_idx || !group_idx || !n_groups)
        return fail(SF_ERR_INVALID_ARG, "compact_proj_fp8: NULL argument");
    if (layer < 0 || layer >= D.nl) return fail(SF_ERR_INVALID_ARG, "compact_proj_fp8: layer %d out of range", layer);
    if (pj->k_head < 1 || pj->k_head > D.Hq) return fail(SF_ERR_INVALID_ARG, "compact_proj_fp8: k_head out of range");
    if (!dense->Wq || !dense->Wk || !dense->Wv || !dense->Wo || !pj->Wqkv8 || !pj->WoT8)
        return fail(SF_ERR_INVALID_ARG, "compact_proj_fp8: NULL weight pointer");
    if (!(dense->sq == dense->sk && dense->sk == dense->sv))
        return fail(SF_ERR_INVALID_ARG, "compact_proj_fp8: Wq, Wk, Wv must share one scale (they form one GEMM operand)");
    if (pj->s_qkv != dense->sq || pj->so != dense->so)
        return fail(SF_ERR_INVALID_ARG, "compact_proj_fp8: s_qkv / so differ from the scales of the dense codes");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int P = D.P, dh = D.dh, d = D.d, kh = pj->k_head;
    const int Nqkv = (kh + 2 * D.Hk) * dh;
    const int32_t *hi = head_idx + (size_t)layer * P * D.Hq;
    const int32_t *gi = group_idx + (size_t)layer * P * D.Hk;
    const int32_t *ng = n_groups + (size_t)layer * P;
    auto region = [&](const void *src, size_t row_off, const int32_t *idx, int idx_stride, int n_static,
                      const int32_t *n_dev, int rows) {
        GatherRegion r{};
        r.src = src; r.dst = (char *)pj->Wqkv8 + row_off * d; r.idx = idx; r.n_dev = n_dev;
        r.idx_stride = idx_stride; r.block = dh; r.n_static = n_static; r.rows = rows;
        r.dst_pstride = (size_t)Nqkv;
        return r;
    };
    GatherRegions wr{};
    wr.r[wr.n++] = region(dense->Wq, 0, hi, D.Hq, kh, nullptr, kh * dh);
    wr.r[wr.n++] = region(dense->Wk, (size_t)kh * dh, gi, D.Hk, 0, ng, D.Hk * dh);
    wr.r[wr.n++] = region(dense->Wv, (size_t)(kh + D.Hk) * dh, gi, D.Hk, 0, ng, D.Hk * dh);
    if (d % 2) return fail(SF_ERR_SHAPE, "compact_proj_fp8: d_model must be even");
    gather_rows(st, wr, (size_t)d, P);
    const int Kp = (int)align_up((size_t)kh * dh, 128);
    dim3 grid(ceil_div(Kp, 32), ceil_div(d, 32), P);
    hipLaunchKernelGGL(gather_transpose_kernel<uint8_t>, grid, dim3(256), 0, st, (const uint8_t *)dense->Wo,
                       (uint8_t *)pj->WoT8, hi, D.Hq, dh, kh, Kp, d, (size_t)d * Kp);
    return check_launch("compact_proj_fp8");
}
