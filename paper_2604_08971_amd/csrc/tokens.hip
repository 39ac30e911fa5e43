// Token compaction: the tokens of absent modalities are dropped (Sec. 4.2 / 4.4: the encoder runs over the
// concatenated tokens of the sensors that are present), each sample keeps its valid tokens in order at the front of
// a shorter padded sequence, and its number of active queries follows its own length, U_b = min(c*ceil(ln T_b), T_b)
// (Sec. 4.4).  Index work only: bit-exact.
#include "common.hpp"

namespace sf {

namespace {

// ceil(ln n) for n >= 1 from the integer parts of e^k: ceil(ln n) is the smallest k with n <= floor(e^k)
__device__ __forceinline__ int ceil_ln(int n)
{
    const int fl_exp[] = {1, 2, 7, 20, 54, 148, 403, 1096, 2980, 8103, 22026, 59874, 162754, 442413, 1202604,
                          3269017, 8886110, 24154952, 65659969, 178482300, 485165195, 1318815734};
    int k = 0;
    while (k < 21 && n > fl_exp[k]) ++k;
    return k;
}

// One block per sample.  slot_of[b,i] = position of token i in the compacted sample or -1; row_index[b,j] = token at
// position j or -1; valid_c[b,j] = j < T_b; len[b] = T_b (not clamped: T_b > Lc tells the caller its Lc was too
// small, positions >= Lc are dropped); u_active[b] = min(c*ceil(ln T_b), T_b).
__global__ __launch_bounds__(256) void token_index_kernel(const uint8_t *__restrict__ token_valid, int L, int Lc,
                                                          int c_factor, int32_t *__restrict__ slot_of,
                                                          int32_t *__restrict__ row_index, uint8_t *__restrict__ valid_c,
                                                          int32_t *__restrict__ len, int32_t *__restrict__ u_active)
{
    __shared__ int wsum[4];
    __shared__ int base_s;
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint8_t *tv = token_valid + (int64_t)b * L;
    if (threadIdx.x == 0) base_s = 0;
    __syncthreads();
    for (int i0 = 0; i0 < L; i0 += 256) {
        const int i = i0 + threadIdx.x;
        const bool ok = i < L && tv[i];
        const uint64_t m = __ballot(ok);
        const int before = __popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) wsum[wave] = __popcll(m);
        __syncthreads();
        int off = base_s;
        for (int w = 0; w < wave; ++w) off += wsum[w];
        const int pos = off + before;
        if (i < L) slot_of[(int64_t)b * L + i] = ok && pos < Lc ? pos : -1;
        if (ok && pos < Lc) row_index[(int64_t)b * Lc + pos] = i;
        __syncthreads();
        if (threadIdx.x == 0) base_s += wsum[0] + wsum[1] + wsum[2] + wsum[3];
        __syncthreads();
    }
    const int T = base_s;
    for (int j = threadIdx.x; j < Lc; j += 256) {
        valid_c[(int64_t)b * Lc + j] = j < T;
        if (j >= T) row_index[(int64_t)b * Lc + j] = -1;
    }
    if (threadIdx.x == 0) {
        len[b] = T;
        const long long u = T >= 1 ? (long long)c_factor * ceil_ln(T) : 0;
        u_active[b] = (int32_t)(u < T ? u : T);
    }
}

// dst[b, j, :] = src[b, index[b, j], :] (zeros where index < 0): one wave per destination row, rows of `units`
// elements of VEC bytes.  Serves both directions (gather with row_index, scatter back with slot_of).
template <class VEC>
__global__ __launch_bounds__(256) void rows_by_index_kernel(const VEC *__restrict__ src, int64_t src_rows,
                                                            const int32_t *__restrict__ index, int64_t dst_rows,
                                                            int64_t n_rows_total, int units, VEC *__restrict__ dst)
{
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);       // destination row over all samples
    if (r >= n_rows_total) return;
    const int64_t b = r / dst_rows;
    const int32_t s = index[r];
    VEC *d = dst + r * units;
    if (s < 0) {
        VEC z{};
        for (int u = lane; u < units; u += 64) d[u] = z;
    } else {
        const VEC *p = src + (b * src_rows + s) * units;
        for (int u = lane; u < units; u += 64) d[u] = p[u];
    }
}

int32_t move_rows(const char *who, const void *src, int64_t src_rows, const int32_t *index, int64_t dst_rows, int B,
                  size_t row_bytes, void *dst, hipStream_t st)
{
    const int64_t total = (int64_t)B * dst_rows;
    if (total == 0) return SF_OK;
    const unsigned grid = (unsigned)((total + 3) / 4);
    if (row_bytes % 16 == 0 && !(((uintptr_t)src | (uintptr_t)dst) & 15))
        hipLaunchKernelGGL(rows_by_index_kernel<uint4>, dim3(grid), dim3(256), 0, st, (const uint4 *)src, src_rows, index,
                           dst_rows, total, (int)(row_bytes / 16), (uint4 *)dst);
    else if (row_bytes % 4 == 0 && !(((uintptr_t)src | (uintptr_t)dst) & 3))
        hipLaunchKernelGGL(rows_by_index_kernel<uint32_t>, dim3(grid), dim3(256), 0, st, (const uint32_t *)src, src_rows,
                           index, dst_rows, total, (int)(row_bytes / 4), (uint32_t *)dst);
    else
        return fail(SF_ERR_SHAPE, "%s: rows must be a multiple of 4 bytes and 4-byte aligned", who);
    return check_launch(who);
}

}  // namespace

}  // namespace sf

using namespace sf;

extern "C" int32_t sf_token_compact(const sf_desc *desc, const void *X, const uint8_t *token_valid, int32_t Lc,
                                    void *Xc, uint8_t *valid_c, int32_t *row_index, int32_t *slot_of, int32_t *len,
                                    int32_t *u_active, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!X || !token_valid || !Xc || !valid_c || !row_index || !slot_of || !len || !u_active)
        return fail(SF_ERR_INVALID_ARG, "token_compact: NULL argument");
    if (Lc < 1 || Lc > D.L) return fail(SF_ERR_INVALID_ARG, "token_compact: Lc must be in [1, L]");
    if (X == Xc) return fail(SF_ERR_INVALID_ARG, "token_compact: Xc may not alias X");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int c = desc->c_factor > 0 ? desc->c_factor : 5;
    hipLaunchKernelGGL(token_index_kernel, dim3(D.B), dim3(256), 0, st, token_valid, D.L, Lc, c, slot_of, row_index,
                       valid_c, len, u_active);
    return move_rows("token_compact", X, D.L, row_index, Lc, D.B, (size_t)D.d * elem_size(D.dtype), Xc, st);
}

extern "C" int32_t sf_token_scatter(const sf_desc *desc, const void *Yc, const int32_t *slot_of, int32_t Lc, void *Y,
                                    void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!Yc || !slot_of || !Y) return fail(SF_ERR_INVALID_ARG, "token_scatter: NULL argument");
    if (Lc < 1 || Lc > D.L) return fail(SF_ERR_INVALID_ARG, "token_scatter: Lc must be in [1, L]");
    if (Y == Yc) return fail(SF_ERR_INVALID_ARG, "token_scatter: Y may not alias Yc");
    return move_rows("token_scatter", Yc, Lc, slot_of, D.L, D.B, (size_t)D.d * elem_size(D.dtype), Y,
                     static_cast<hipStream_t>(stream));
}
