// Sparse-MoE FFN with pruned experts (Sec. 4.5 of the paper, "Sparse-MoE FFN
// pruning"): fixed number of experts and Top-k routing, every expert's FFN
// pruned to its own channel set.
//
// Data flow on the GPU (everything stream-ordered, no host round trip):
//   LayerNorm -> router (logits, Top-k, softmax over the chosen logits)
//   -> counting sort of the (token, slot) pairs by segment = (pattern, expert),
//      every segment padded to a multiple of 256 rows
//   -> gather of the normalised rows into that order
//   -> the two GEMMs of the encoder's FFN, run over 256-row blocks: the GEMM's
//      per-sample "pattern" index is the block's segment, so each block uses
//      its expert's (and pattern's) compacted weights without any change to
//      the GEMM kernels; rows of padding produce values nobody reads
//   -> weighted combination of each token's top_k rows (+ residual).
// The order of rows inside a segment depends on integer atomics and may vary
// from run to run; no result depends on it (every row is computed on its own).
#include "gemm.hpp"

namespace sf {

namespace {

constexpr int SEG_ROWS = 256;           // rows per GEMM block (one "sample" of the grouped GEMM)

// One wave per token: lane e ends up holding logit_e (E <= 64).
template <class T>
__global__ __launch_bounds__(256) void moe_router_kernel(
    const T *__restrict__ xn, const T *__restrict__ Wr, const T *__restrict__ br, int64_t rows, int d, int E,
    int top_k, const int32_t *__restrict__ forced_route, int32_t *__restrict__ route, float *__restrict__ weight,
    float *__restrict__ logit_out)
{
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= rows) return;
    const T *x = xn + t * d;
    float mine = -INFINITY;                                 // logit of expert `lane`
    for (int e = 0; e < E; ++e) {
        const T *w = Wr + (int64_t)e * d;
        float acc = 0.f;
        for (int c = lane; c < d; c += 64) acc = fmaf(to_f32(x[c]), to_f32(w[c]), acc);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
        if (br) acc += to_f32(br[e]);
        if (lane == e) mine = acc;
    }
    if (logit_out && lane < E) logit_out[t * E + lane] = mine;
    // Top-k by repeated wave argmax over the experts not taken yet (ties: lower expert index; a NaN logit
    // ranks below every number), or the caller's experts.  Lane s < top_k remembers the expert of slot s.
    const float val = mine == mine ? mine : -INFINITY;
    bool avail = lane < E;
    int my_slot = -1, slot_expert = 0;
    float my_logit = 0.f;
    for (int s = 0; s < top_k; ++s) {
        int pick;
        if (forced_route) {
            pick = min(max(forced_route[t * top_k + s], 0), E - 1);
        } else {
            float v = val;
            int idx = lane;
            bool a = avail;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float ov = __shfl_xor(v, o);
                const int oi = __shfl_xor(idx, o);
                const bool oa = __shfl_xor((int)a, o) != 0;
                const bool better = (oa && !a) || (oa == a && (ov > v || (ov == v && oi < idx)));
                if (better) { v = ov; idx = oi; a = oa; }
            }
            pick = idx;                                     // the order is total: every lane agrees
        }
        if (lane == pick) { my_slot = s; my_logit = val; avail = false; }
        if (lane == s) slot_expert = pick;
    }
    // softmax over the chosen logits (an expert listed twice by the caller counts once, in its last slot)
    float mx = my_slot >= 0 ? my_logit : -INFINITY;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    const float ex = my_slot >= 0 ? expf(my_logit - mx) : 0.f;
    float den = ex;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) den += __shfl_xor(den, o);
    const float w_e = ex / den;
    const float w_s = __shfl(w_e, slot_expert);
    const int owner = __shfl(my_slot, slot_expert);
    if (lane < top_k) {
        route[t * top_k + lane] = slot_expert;
        weight[t * top_k + lane] = owner == lane ? w_s : 0.f;
    }
}

__global__ void moe_zero_kernel(int32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// counts[seg] += 1 for every (token, slot); seg = pattern(token) * E + expert
__global__ __launch_bounds__(256) void moe_count_kernel(const int32_t *__restrict__ route, const int32_t *__restrict__ pattern_id,
                                                        int64_t rows, int L, int P, int E, int top_k,
                                                        int32_t *__restrict__ counts)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= rows * top_k) return;
    const int64_t t = i / top_k;
    const int p = pattern_id ? min(max(pattern_id[t / L], 0), P - 1) : 0;
    atomicAdd(&counts[p * E + route[i]], 1);
}

// Segment bases (each segment padded to a multiple of SEG_ROWS), the segment of every 256-row block
// (unused blocks: segment 0) and the fill cursors.  One block; n_seg <= MAX_SEG, staged in LDS.
constexpr int MAX_SEG = 4096;

__global__ __launch_bounds__(256) void moe_layout_kernel(const int32_t *__restrict__ counts, int n_seg, int n_blocks_max,
                                                         int32_t *__restrict__ seg_base, int32_t *__restrict__ cursor,
                                                         int32_t *__restrict__ blk_seg)
{
    __shared__ int first_blk[MAX_SEG + 1];                  // first 256-row block of every segment
    for (int s = threadIdx.x; s < n_seg; s += 256) first_blk[s] = (counts[s] + SEG_ROWS - 1) / SEG_ROWS;
    __syncthreads();
    if (threadIdx.x == 0) {
        int base = 0;
        for (int s = 0; s < n_seg; ++s) {
            const int nb = first_blk[s];
            first_blk[s] = base;
            base += nb;
        }
        first_blk[n_seg] = base;
    }
    __syncthreads();
    for (int s = threadIdx.x; s <= n_seg; s += 256) {
        seg_base[s] = first_blk[s] * SEG_ROWS;
        if (s < n_seg) cursor[s] = 0;
    }
    const int total_blocks = first_blk[n_seg];
    for (int j = threadIdx.x; j < n_blocks_max; j += 256) {
        int s = 0;
        if (j < total_blocks) {
            // the last segment that starts at or before block j (empty segments share their successor's start)
            int lo = 0, hi = n_seg - 1;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (first_blk[mid] <= j) lo = mid; else hi = mid - 1;
            }
            s = lo;
        }
        blk_seg[j] = s;
    }
}

// pos[token, slot] = row of the pair in the gathered order
__global__ __launch_bounds__(256) void moe_place_kernel(const int32_t *__restrict__ route, const int32_t *__restrict__ pattern_id,
                                                        int64_t rows, int L, int P, int E, int top_k,
                                                        const int32_t *__restrict__ seg_base, int32_t *__restrict__ cursor,
                                                        int32_t *__restrict__ pos)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= rows * top_k) return;
    const int64_t t = i / top_k;
    const int p = pattern_id ? min(max(pattern_id[t / L], 0), P - 1) : 0;
    const int seg = p * E + route[i];
    pos[i] = seg_base[seg] + atomicAdd(&cursor[seg], 1);
}

// Xg[pos[token, slot], :] = xn[token, :]; one wave per (token, slot), 16-byte copies when possible
template <class VEC>
__global__ __launch_bounds__(256) void moe_gather_kernel(const VEC *__restrict__ xn, const int32_t *__restrict__ pos,
                                                         int64_t pairs, int top_k, int row_vecs, VEC *__restrict__ xg)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= pairs) return;
    const VEC *s = xn + (i / top_k) * row_vecs;
    VEC *d = xg + (int64_t)pos[i] * row_vecs;
    for (int c = lane; c < row_vecs; c += 64) d[c] = s[c];
}

// Y[t, :] = [X[t, :] +] sum_s weight[t, s] * Yg[pos[t, s], :]; one wave per token
template <class T>
__global__ __launch_bounds__(256) void moe_combine_kernel(const T *__restrict__ X, const float *__restrict__ yg,
                                                          const int32_t *__restrict__ pos, const float *__restrict__ weight,
                                                          int64_t rows, int d, int top_k, int add_residual, T *__restrict__ Y)
{
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= rows) return;
    for (int c = lane * 4; c < d; c += 256) {               // d % 4 == 0 checked on the host
        float acc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = add_residual ? to_f32(X[t * d + c + e]) : 0.f;
        for (int s = 0; s < top_k; ++s) {
            const float w = weight[t * top_k + s];
            const f32x4 v = *reinterpret_cast<const f32x4 *>(yg + (int64_t)pos[t * top_k + s] * d + c);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = fmaf(w, v[e], acc[e]);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) Y[t * d + c + e] = from_f32<T>(acc[e]);
    }
}

struct MoeWs {
    void *xn, *xg, *hg; float *yg, *weight; int32_t *route, *pos, *counts, *seg_base, *cursor, *blk_seg;
    int n_blocks_max, Fp; size_t bytes;
};

MoeWs moe_ws(const Dims &D, const sf_moe_compact &m, void *ws)
{
    MoeWs w{};
    const size_t es = elem_size(D.dtype), rows = (size_t)D.B * D.L;
    const int n_seg = D.P * m.n_experts;
    w.Fp = (int)align_up(m.k_ffn_max, D.ffn_pad);
    w.n_blocks_max = (int)((rows * m.top_k + SEG_ROWS - 1) / SEG_ROWS) + n_seg;
    const size_t grows = (size_t)w.n_blocks_max * SEG_ROWS;
    Carver c(ws);
    w.xn = c.take<char>(rows * D.d * es);
    w.route = c.take<int32_t>(rows * m.top_k);
    w.weight = c.take<float>(rows * m.top_k);
    w.pos = c.take<int32_t>(rows * m.top_k);
    w.counts = c.take<int32_t>(n_seg);
    w.seg_base = c.take<int32_t>(n_seg + 1);
    w.cursor = c.take<int32_t>(n_seg);
    w.blk_seg = c.take<int32_t>(w.n_blocks_max);
    w.xg = c.take<char>(grows * D.d * es);
    w.hg = c.take<char>(grows * (size_t)w.Fp * es);
    w.yg = c.take<float>(grows * D.d);
    w.bytes = c.off;
    return w;
}

int32_t check_moe(const Dims &D, const sf_moe_compact *m)
{
    if (!m) return fail(SF_ERR_INVALID_ARG, "moe_ffn: NULL argument");
    if (m->n_experts < 1 || m->n_experts > 64 || m->top_k < 1 || m->top_k > m->n_experts || m->top_k > 8)
        return fail(SF_ERR_INVALID_ARG, "moe_ffn: needs 1 <= top_k <= min(8, n_experts), n_experts <= 64");
    if (m->k_ffn_max < 1 || m->k_ffn_max > D.F) return fail(SF_ERR_INVALID_ARG, "moe_ffn: k_ffn_max out of range");
    if ((int64_t)D.P * m->n_experts > MAX_SEG) return fail(SF_ERR_SHAPE, "moe_ffn: more than %d (pattern, expert) pairs", MAX_SEG);
    if (D.d % 4) return fail(SF_ERR_SHAPE, "moe_ffn: d_model must be a multiple of 4");
    if ((int64_t)D.B * D.L * m->top_k > ((int64_t)1 << 30)) return fail(SF_ERR_SHAPE, "moe_ffn: too many (token, slot) pairs");
    return SF_OK;
}

}  // namespace

}  // namespace sf

using namespace sf;

extern "C" size_t sf_moe_ffn_workspace_bytes(const sf_desc *desc, const sf_moe_compact *m)
{
    Dims D;
    if (read_desc(desc, D) || check_moe(D, m)) return 0;
    return moe_ws(D, *m, nullptr).bytes;
}

extern "C" int32_t sf_moe_ffn_forward(const sf_desc *desc, const sf_moe_compact *m, const void *X,
                                      const int32_t *pattern_id, int32_t pre_ln, int32_t add_residual,
                                      const int32_t *forced_route, void *Y, int32_t *route_out,
                                      float *weight_out, float *logit_out, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (int32_t rc = check_moe(D, m)) return rc;
    if (!X || !Y) return fail(SF_ERR_INVALID_ARG, "moe_ffn: NULL argument");
    if (X == Y) return fail(SF_ERR_INVALID_ARG, "moe_ffn: Y may not alias X");
    if (!m->Wr || !m->W1 || !m->W2T || (pre_ln && (!m->ln_g || !m->ln_b)))
        return fail(SF_ERR_INVALID_ARG, "moe_ffn: NULL parameter pointer");
    if (D.P > 1 && !pattern_id) return fail(SF_ERR_INVALID_ARG, "moe_ffn: pattern_id required when P > 1");
    MoeWs w = moe_ws(D, *m, workspace);
    if (!workspace || workspace_bytes < w.bytes || ((uintptr_t)workspace & 255))
        return fail(SF_ERR_WORKSPACE, "moe_ffn: workspace of %zu bytes (256-byte aligned) required, got %zu", w.bytes,
                    workspace_bytes);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t rows = (int64_t)D.B * D.L, pairs = rows * m->top_k;
    const int E = m->n_experts, k = m->top_k, n_seg = D.P * E;
    const size_t es = elem_size(D.dtype);
    const bool bf = D.dtype == SF_BF16;

    const void *xin = X;
    if (pre_ln) {
        layernorm(D.dtype, 0, X, m->ln_g, m->ln_b, D.eps, rows, D.d, w.xn, st);
        xin = w.xn;
    }
    // router
    {
        dim3 grid((unsigned)((rows + 3) / 4));
        if (bf)
            hipLaunchKernelGGL(moe_router_kernel<__bf16>, grid, dim3(256), 0, st, (const __bf16 *)xin,
                               (const __bf16 *)m->Wr, (const __bf16 *)m->br, rows, D.d, E, k, forced_route, w.route,
                               w.weight, logit_out);
        else
            hipLaunchKernelGGL(moe_router_kernel<float>, grid, dim3(256), 0, st, (const float *)xin,
                               (const float *)m->Wr, (const float *)m->br, rows, D.d, E, k, forced_route, w.route,
                               w.weight, logit_out);
    }
    // counting sort of the (token, slot) pairs by (pattern, expert)
    hipLaunchKernelGGL(moe_zero_kernel, dim3(ceil_div(n_seg, 256)), dim3(256), 0, st, w.counts, n_seg);
    hipLaunchKernelGGL(moe_count_kernel, dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, st, w.route, pattern_id,
                       rows, D.L, D.P, E, k, w.counts);
    hipLaunchKernelGGL(moe_layout_kernel, dim3(1), dim3(256), 0, st, w.counts, n_seg, w.n_blocks_max, w.seg_base,
                       w.cursor, w.blk_seg);
    hipLaunchKernelGGL(moe_place_kernel, dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, st, w.route, pattern_id,
                       rows, D.L, D.P, E, k, w.seg_base, w.cursor, w.pos);
    {
        const size_t row_bytes = (size_t)D.d * es;
        dim3 grid((unsigned)((pairs + 3) / 4));
        if (row_bytes % 16 == 0 && ((uintptr_t)xin % 16 == 0))
            hipLaunchKernelGGL(moe_gather_kernel<uint4>, grid, dim3(256), 0, st, (const uint4 *)xin, w.pos, pairs, k,
                               (int)(row_bytes / 16), (uint4 *)w.xg);
        else
            hipLaunchKernelGGL(moe_gather_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t *)xin, w.pos, pairs,
                               k, (int)(row_bytes / 2), (uint16_t *)w.xg);
    }
    // the two GEMMs over 256-row blocks; the block's segment selects the weights
    GemmArgs g{};
    g.A = w.xg; g.lda = D.d; g.W = m->W1; g.ldw = D.d; g.w_pstride = (int64_t)w.Fp * D.d;
    g.bias = m->b1; g.bias_pstride = w.Fp; g.pattern_id = w.blk_seg;
    g.B = w.n_blocks_max; g.L = SEG_ROWS; g.N = w.Fp; g.K = D.d; g.epi = EPI_ROWMAJOR;
    g.act = D.act == SF_GELU_ERF ? ACT_GELU : ACT_RELU;
    g.C = w.hg; g.ldc = w.Fp;
    if (int32_t rc = gemm(D.dtype, g, st)) return rc;
    GemmArgs h{};
    h.A = w.hg; h.lda = w.Fp; h.W = m->W2T; h.ldw = w.Fp; h.w_pstride = (int64_t)D.d * w.Fp;
    h.bias = m->b2x; h.bias_pstride = D.d; h.pattern_id = w.blk_seg;
    h.B = w.n_blocks_max; h.L = SEG_ROWS; h.N = D.d; h.K = w.Fp; h.epi = EPI_ROWMAJOR; h.act = ACT_NONE;
    h.C = w.yg; h.ldc = D.d; h.c_f32 = 1;
    if (int32_t rc = gemm(D.dtype, h, st)) return rc;
    {
        dim3 grid((unsigned)((rows + 3) / 4));
        if (bf)
            hipLaunchKernelGGL(moe_combine_kernel<__bf16>, grid, dim3(256), 0, st, (const __bf16 *)X, w.yg, w.pos,
                               w.weight, rows, D.d, k, add_residual, (__bf16 *)Y);
        else
            hipLaunchKernelGGL(moe_combine_kernel<float>, grid, dim3(256), 0, st, (const float *)X, w.yg, w.pos,
                               w.weight, rows, D.d, k, add_residual, (float *)Y);
    }
    if (route_out &&
        hipMemcpyAsync(route_out, w.route, (size_t)pairs * 4, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(SF_ERR_HIP, "moe_ffn: copy of the routing failed");
    if (weight_out &&
        hipMemcpyAsync(weight_out, w.weight, (size_t)pairs * 4, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(SF_ERR_HIP, "moe_ffn: copy of the weights failed");
    return check_launch("moe_ffn_forward");
}
