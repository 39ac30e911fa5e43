// Token compaction: the tokens of absent modalities are dropped (Sec. 4.2 / 4.4: the encoder runs over the
// concatenated tokens of the sensors that are present), each sample keeps its valid tokens in order at the front of
// a shorter padded sequence, and its number of active queries follows its own length, U_b = min(c*ceil(ln T_b), T_b)
// (Sec. 4.4).  Index work only: bit-exact.
#include <algorithm>

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

// ---- packed layout: no padding to a common length ------------------------------------------------------------
// The valid tokens of all samples back to back in one [Tc, d] buffer, the samples ordered by presence pattern (then
// by sample number) and every pattern's run of rows starting on a multiple of 256, so that a 256-row block of the
// buffer holds rows of one pattern only (it may straddle samples): the row-wise work of the encoder (LayerNorm, the
// four GEMMs) runs over the blocks in use, with each block's pattern in blk_pattern, and only the attention kernels
// see samples (first row row0[b], allowed positions valid_c[b, :]).  Behind the last run come align(L, 256) rows of
// slack with the last run's pattern: an attention kernel reads up to L rows from a sample's first row whatever the
// sample's own length (what lies behind its tokens is masked), so those rows must exist and hold finite numbers.
// ext[b] >= len[b] is the number of rows sample b answers for in the attention output: its tokens, and for the last
// sample of a run the padding up to the next run (for the last run: and the slack).

// Pass 1, one block per sample: rank[b, i] = number of valid tokens before i (for a valid token: its position in
// the compacted sample) and len[b].
__global__ __launch_bounds__(256) void token_rank_kernel(const uint8_t *__restrict__ token_valid, int L,
                                                         int32_t *__restrict__ rank, int32_t *__restrict__ len)
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
        if (lane == 0) wsum[wave] = __popcll(m);
        __syncthreads();
        int off = base_s + __popcll(m & ((1ull << lane) - 1ull));
        for (int w = 0; w < wave; ++w) off += wsum[w];
        if (i < L) rank[(int64_t)b * L + i] = off;
        __syncthreads();
        if (threadIdx.x == 0) base_s += wsum[0] + wsum[1] + wsum[2] + wsum[3];
        __syncthreads();
    }
    if (threadIdx.x == 0) len[b] = base_s;
}

// Pass 2, one block: the layout.  n_rows[0] = rows in use (runs + slack, a multiple of 256; 0 when no sample has a
// token), n_rows[1] = the same before the comparison with Tc.  When the rows do not fit (n_rows[1] > Tc) the plan is
// the empty one - every sample at row 0 with no rows, every block unused - so that whatever runs on it touches
// nothing; the caller reads n_rows[1] and comes back with a larger buffer.  A pattern number outside [0, P) gives the
// empty plan too, with n_rows[1] = -1.
// Per pattern (LDS, P <= PACK_MAX_P): the rows of its run (integer atomics: order-free), its last sample, then the
// first row of its run from one scan over the patterns.  Per sample: the samples are walked in order, PACK_NT at a
// time; a sample's row is its pattern's running position plus the rows of the earlier samples of the same pattern
// in its chunk.  Three barriers per PACK_NT patterns and per PACK_NT samples.
constexpr int PACK_MAX_P = 4096, PACK_NT = 256;

__global__ __launch_bounds__(PACK_NT) void pack_layout_kernel(const int32_t *__restrict__ len,
                                                              const int32_t *__restrict__ pattern_id, int B, int P, int L,
                                                              int Tc, int32_t *__restrict__ row0, int32_t *__restrict__ ext,
                                                              int32_t *__restrict__ blk_pattern, int32_t *__restrict__ n_rows)
{
    extern __shared__ int32_t psm[];
    int32_t *seg = psm, *base = psm + P, *lastb = psm + 2 * P, *cur = psm + 3 * P;      // [P] each
    __shared__ int wsum[PACK_NT / 64];
    __shared__ __attribute__((aligned(16))) int p_s[PACK_NT], l_s[PACK_NT];
    __shared__ int carry_s, tail_p_s, bad_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nblk = Tc / 256;
    for (int p = tid; p < P; p += PACK_NT) { seg[p] = 0; lastb[p] = -1; }
    for (int k = tid; k < nblk; k += PACK_NT) blk_pattern[k] = -1;
    if (tid == 0) { carry_s = 0; tail_p_s = -1; bad_s = 0; }
    __syncthreads();
    for (int b = tid; b < B; b += PACK_NT) {
        const int p = pattern_id ? pattern_id[b] : 0;
        if (p < 0 || p >= P) { bad_s = 1; continue; }
        atomicAdd(&seg[p], len[b]);
        atomicMax(&lastb[p], b);
    }
    __syncthreads();
    // first row of every run: exclusive scan of the padded run lengths, PACK_NT patterns at a time
    for (int p0 = 0; p0 < P; p0 += PACK_NT) {
        const int p = p0 + tid;
        const int v = p < P ? (seg[p] + 255) & ~255 : 0;
        int incl = v;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        int off = carry_s + incl - v;
        for (int w = 0; w < wave; ++w) off += wsum[w];
        if (p < P) { base[p] = off; cur[p] = off; }
        if (p < P && seg[p] > 0) atomicMax(&tail_p_s, p);           // the last run that has rows
        __syncthreads();
        if (tid == 0) { int t = 0; for (int w = 0; w < PACK_NT / 64; ++w) t += wsum[w]; carry_s += t; }
        __syncthreads();
    }
    const bool bad = bad_s != 0;
    const int used = carry_s, slack = (L + 255) & ~255;
    const int need = bad ? -1 : used > 0 ? used + slack : 0;
    const bool fits = !bad && need <= Tc;
    const int tail_p = tail_p_s;
    for (int c0 = 0; c0 < B; c0 += PACK_NT) {
        const int b = c0 + tid;
        int p = b < B ? (pattern_id ? pattern_id[b] : 0) : -1;
        if (p >= P) p = -1;
        const int lb = b < B && p >= 0 ? len[b] : 0;
        p_s[tid] = p;
        l_s[tid] = lb;
        __syncthreads();
        int before = 0;                                 // four entries per LDS read, no branch: the reads pipeline
#pragma unroll 4
        for (int t4 = 0; t4 * 4 < tid; ++t4) {
            const int4 pp = reinterpret_cast<const int4 *>(p_s)[t4], ll = reinterpret_cast<const int4 *>(l_s)[t4];
            before += (pp.x == p && t4 * 4 + 0 < tid ? ll.x : 0) + (pp.y == p && t4 * 4 + 1 < tid ? ll.y : 0) +
                      (pp.z == p && t4 * 4 + 2 < tid ? ll.z : 0) + (pp.w == p && t4 * 4 + 3 < tid ? ll.w : 0);
        }
        const int row = p >= 0 ? cur[p] + before : 0;
        __syncthreads();
        if (p >= 0) atomicAdd(&cur[p], lb);
        if (b < B) {
            int e = lb;
            if (p >= 0 && b == lastb[p] && seg[p] > 0) {            // the last sample of a run answers for its padding
                e = base[p] + ((seg[p] + 255) & ~255) - row;
                if (p == tail_p) e += slack;                        // ... and the last run's for the slack
            }
            row0[b] = fits ? row : 0;
            ext[b] = fits ? e : 0;
        }
        __syncthreads();
    }
    if (fits) {
        for (int p = wave; p < P; p += PACK_NT / 64) {        // a wave per run, a lane per block
            if (seg[p] <= 0) continue;
            const int k1 = (base[p] + ((seg[p] + 255) & ~255) + (p == tail_p ? slack : 0)) / 256;
            for (int k = base[p] / 256 + lane; k < k1; k += 64) blk_pattern[k] = p;
        }
    }
    if (tid == 0) { n_rows[0] = fits ? need : 0; n_rows[1] = need; }
}

// Pass 3, grid (row chunks of 256, B + 1).  Samples: dst_row[b, i] (on entry the rank of token i) becomes the packed
// row of a valid token or -1, src_row[r] the source row b*L + i of a packed row or -1 for the padding the sample
// answers for, valid_c[b, j] = j < len[b], u_active[b] = min(c*ceil(ln T_b), T_b).  The extra grid row marks the
// rows behind the ones in use as empty.
__global__ __launch_bounds__(256) void pack_rows_kernel(const uint8_t *__restrict__ token_valid,
                                                        const int32_t *__restrict__ len, const int32_t *__restrict__ row0,
                                                        const int32_t *__restrict__ ext, const int32_t *__restrict__ n_rows,
                                                        int B, int L, int Tc, int c_factor, int32_t *__restrict__ dst_row,
                                                        int32_t *__restrict__ src_row, uint8_t *__restrict__ valid_c,
                                                        int32_t *__restrict__ u_active)
{
    const int b = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
    const int used = n_rows[0];
    if (b == B) {
        for (int64_t r = (int64_t)used + j; r < Tc; r += (int64_t)gridDim.x * 256) src_row[r] = -1;
        return;
    }
    const bool ok = used > 0;                              // else: the empty plan
    const int T = ok ? len[b] : 0, r0 = row0[b], e = ext[b];
    if (j < L) {
        const int64_t t = (int64_t)b * L + j;
        const bool tok = ok && token_valid[t];
        const int r = r0 + dst_row[t];
        dst_row[t] = tok ? r : -1;
        if (tok) src_row[r] = (int32_t)t;
        valid_c[t] = j < T;
    }
    if (j >= T && j < e) src_row[r0 + j] = -1;
    if (j == 0) {
        const long long u = T >= 1 ? (long long)c_factor * ceil_ln(T) : 0;
        u_active[b] = (int32_t)(u < T ? u : T);
    }
}

}  // namespace

}  // namespace sf

using namespace sf;

static int32_t check_pack_plan(const char *who, const Dims &D, const sf_token_pack_plan *plan)
{
    if (!plan) return fail(SF_ERR_INVALID_ARG, "%s: plan is NULL", who);
    if (plan->Tc < 256 || plan->Tc % 256) return fail(SF_ERR_INVALID_ARG, "%s: Tc must be a positive multiple of 256", who);
    if (!plan->len || !plan->u_active || !plan->row0 || !plan->ext || !plan->valid_c || !plan->blk_pattern ||
        !plan->src_row || !plan->dst_row || !plan->n_rows)
        return fail(SF_ERR_INVALID_ARG, "%s: NULL pointer in the plan", who);
    if ((int64_t)plan->Tc > ((int64_t)1 << 30)) return fail(SF_ERR_SHAPE, "%s: Tc too large", who);
    (void)D;
    return SF_OK;
}

extern "C" int32_t sf_token_pack_rows_max(const sf_desc *desc)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    const int64_t runs = D.P < D.B ? D.P : D.B;
    const int64_t need = (int64_t)align_up((size_t)D.B * D.L, 256) + 256 * runs + (int64_t)align_up((size_t)D.L, 256);
    if (need > ((int64_t)1 << 30)) return fail(SF_ERR_SHAPE, "token_pack_rows_max: B*L too large");
    return (int32_t)need;
}

extern "C" int32_t sf_token_pack(const sf_desc *desc, const void *X, const uint8_t *token_valid,
                                 const int32_t *pattern_id, const sf_token_pack_plan *plan, void *Xp, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (int32_t rc = check_pack_plan("token_pack", D, plan)) return rc;
    if (!X || !token_valid || !Xp) return fail(SF_ERR_INVALID_ARG, "token_pack: NULL argument");
    if (X == Xp) return fail(SF_ERR_INVALID_ARG, "token_pack: Xp may not alias X");
    if (D.P > 1 && !pattern_id) return fail(SF_ERR_INVALID_ARG, "token_pack: pattern_id required when P > 1");
    if (D.P > PACK_MAX_P) return fail(SF_ERR_SHAPE, "token_pack: at most %d presence patterns", PACK_MAX_P);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int c = desc->c_factor > 0 ? desc->c_factor : 5;
    hipLaunchKernelGGL(token_rank_kernel, dim3(D.B), dim3(256), 0, st, token_valid, D.L, plan->dst_row, plan->len);
    hipLaunchKernelGGL(pack_layout_kernel, dim3(1), dim3(PACK_NT), (size_t)4 * D.P * sizeof(int32_t), st, plan->len,
                       pattern_id, D.B, D.P, D.L, plan->Tc, plan->row0, plan->ext, plan->blk_pattern, plan->n_rows);
    // a sample answers for at most its L tokens, 255 rows of padding and the slack
    dim3 grid((unsigned)ceil_div(2 * D.L + 512, 256), (unsigned)D.B + 1);
    hipLaunchKernelGGL(pack_rows_kernel, grid, dim3(256), 0, st, token_valid, plan->len, plan->row0, plan->ext,
                       plan->n_rows, D.B, D.L, plan->Tc, c, plan->dst_row, plan->src_row, plan->valid_c, plan->u_active);
    // rows by global source row: one "sample" of Tc rows
    return move_rows("token_pack", X, 0, plan->src_row, plan->Tc, 1, (size_t)D.d * elem_size(D.dtype), Xp, st);
}

extern "C" int32_t sf_token_unpack(const sf_desc *desc, const void *Yp, const sf_token_pack_plan *plan, void *Y,
                                   void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (int32_t rc = check_pack_plan("token_unpack", D, plan)) return rc;
    if (!Yp || !Y) return fail(SF_ERR_INVALID_ARG, "token_unpack: NULL argument");
    if (Y == Yp) return fail(SF_ERR_INVALID_ARG, "token_unpack: Y may not alias Yp");
    return move_rows("token_unpack", Yp, 0, plan->dst_row, (int64_t)D.B * D.L, 1, (size_t)D.d * elem_size(D.dtype), Y,
                     static_cast<hipStream_t>(stream));
}

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
