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
//      its expert's (and pattern's) compacted weights; the per-pattern width
//      limits of the GEMM stop at the expert's own padded channel count and
//      blocks beyond the last segment are skipped; rows of padding produce
//      values nobody reads
//   -> weighted combination of each token's top_k rows (+ residual).
// The order of rows inside a segment depends on integer atomics and may vary
// from run to run; no result depends on it (every row is computed on its own).
#include "gemm.hpp"

namespace sf {

namespace {

constexpr int SEG_ROWS = 256;           // rows per GEMM block (one "sample" of the grouped GEMM)

// 16 bytes of a row as floats
template <class T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    static __device__ void load(const float *p, float (&v)[4]) {
        const f32x4 q = *reinterpret_cast<const f32x4 *>(p);
        v[0] = q[0]; v[1] = q[1]; v[2] = q[2]; v[3] = q[3];
    }
};
template <> struct Vec16<h16> {
    static constexpr int N = 8;
    static __device__ void load(const h16 *p, float (&v)[8]) {
        const h16x8 q = *reinterpret_cast<const h16x8 *>(p);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (float)q[i];
    }
};

// Router.  Phase 1, one wave per token (TOK_PER_BLOCK tokens per block): the token's row is read once
// (16 bytes per lane and step, d % Vec16<T>::N == 0) against the router rows, which are staged in LDS once
// per block when they fit (WLDS) and come through the cache otherwise; the E logits go to LDS.  Phase 2, one
// lane per token: Top-k and the softmax over the chosen logits.
constexpr int TOK_PER_BLOCK = 64;

template <class T, int EB, bool WLDS>
__global__ __launch_bounds__(256) void moe_router_kernel(
    const T *__restrict__ xn, const T *__restrict__ Wr, const T *__restrict__ br, int64_t rows, int d, int E,
    int top_k, const int32_t *__restrict__ forced_route, int32_t *__restrict__ route, float *__restrict__ weight,
    float *__restrict__ logit_out)
{
    constexpr int VN = Vec16<T>::N;
    extern __shared__ __attribute__((aligned(16))) char router_lds[];
    float *lg = reinterpret_cast<float *>(router_lds);      // [TOK_PER_BLOCK][E + 1]
    const int lgs = E + 1;
    const T *Wl = Wr;
    if constexpr (WLDS) {
        char *wbase = router_lds + (((size_t)TOK_PER_BLOCK * lgs * sizeof(float) + 15) & ~(size_t)15);
        uint4 *dst = reinterpret_cast<uint4 *>(wbase);
        const uint4 *src = reinterpret_cast<const uint4 *>(Wr);
        const int n16 = E * d / VN;
        for (int i = threadIdx.x; i < n16; i += 256) dst[i] = src[i];
        __syncthreads();
        Wl = reinterpret_cast<const T *>(wbase);
    }
    const int lane = threadIdx.x & 63;
    for (int tt = threadIdx.x >> 6; tt < TOK_PER_BLOCK; tt += 4) {
        const int64_t t = (int64_t)blockIdx.x * TOK_PER_BLOCK + tt;
        if (t >= rows) break;
        const T *x = xn + t * d;
        float acc[EB];
#pragma unroll
        for (int e = 0; e < EB; ++e) acc[e] = 0.f;
        for (int c = lane * VN; c < d; c += 64 * VN) {
            if constexpr (VN == 8) {
                // 16-bit: two products per instruction, fp32 accumulate, no unpacking
                const uint4 xq = *reinterpret_cast<const uint4 *>(x + c);
                const uint32_t xw[4] = {xq.x, xq.y, xq.z, xq.w};
#pragma unroll
                for (int e = 0; e < EB; ++e) {
                    if (e < E) {
                        const uint4 wq = *reinterpret_cast<const uint4 *>(Wl + e * d + c);
                        const uint32_t ww[4] = {wq.x, wq.y, wq.z, wq.w};
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            acc[e] = SF_FDOT2(__builtin_bit_cast(h16x2, xw[i]), __builtin_bit_cast(h16x2, ww[i]), acc[e], false);
                    }
                }
            } else {
                float xv[VN];
                Vec16<T>::load(x + c, xv);
#pragma unroll
                for (int e = 0; e < EB; ++e) {
                    if (e < E) {
                        float wv[VN];
                        Vec16<T>::load(Wl + e * d + c, wv);
#pragma unroll
                        for (int i = 0; i < VN; ++i) acc[e] = fmaf(xv[i], wv[i], acc[e]);
                    }
                }
            }
        }
        // Transposing reduction: every step halves the number of partial sums a lane carries (the lanes whose
        // bit `o` is set keep the upper half) until one is left, which the remaining steps sum up; lane l then
        // holds the logit of expert l >> SH.  EB - 1 + log2(64 / EB) exchanges instead of 6 * EB.
        constexpr int SH = EB == 64 ? 0 : (EB == 16 ? 2 : 3);
        int n = EB;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            if (n > 1) {
                n >>= 1;
                const bool up = (lane & o) != 0;
#pragma unroll
                for (int i = 0; i < EB / 2; ++i) {
                    if (i < n) {
                        const float send = up ? acc[i] : acc[i + n];
                        const float keep = up ? acc[i + n] : acc[i];
                        acc[i] = keep + __shfl_xor(send, o);
                    }
                }
            } else {
                acc[0] += __shfl_xor(acc[0], o);
            }
        }
        const int e = lane >> SH;
        if ((lane & ((1 << SH) - 1)) == 0 && e < E) lg[tt * lgs + e] = acc[0] + (br ? to_f32(br[e]) : 0.f);
    }
    __syncthreads();
    // Phase 2: lane tt of the first wave owns token tt.  Top-k by repeated scan over the experts not taken yet
    // (ties: lower expert index; a NaN logit ranks below every number), or the caller's experts.
    if (threadIdx.x >= TOK_PER_BLOCK) return;
    const int64_t t = (int64_t)blockIdx.x * TOK_PER_BLOCK + threadIdx.x;
    if (t >= rows) return;
    const float *my = lg + threadIdx.x * lgs;
    if (logit_out)
        for (int e = 0; e < E; ++e) logit_out[t * E + e] = my[e];
    int pick[8];
    float pv[8];
    unsigned long long taken = 0;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        pick[s] = 0;
        pv[s] = -INFINITY;
        if (s < top_k) {
            int be = -1;
            float bv = -INFINITY;
            if (forced_route) {
                be = min(max(forced_route[t * top_k + s], 0), E - 1);
                bv = my[be];
                bv = bv == bv ? bv : -INFINITY;
            } else {
                for (int e = 0; e < E; ++e) {
                    float v = my[e];
                    v = v == v ? v : -INFINITY;
                    if (!((taken >> e) & 1) && (be < 0 || v > bv)) { be = e; bv = v; }
                }
                taken |= 1ull << be;                        // be >= 0: top_k <= E
            }
            pick[s] = be;
            pv[s] = bv;
        }
    }
    // softmax over the chosen logits (an expert listed twice by the caller counts once, in its last slot)
    float mx = -INFINITY, den = 0.f, ex[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        bool again = false;
#pragma unroll
        for (int q = s + 1; q < 8; ++q) again = again || (q < top_k && pick[q] == pick[s]);
        ex[s] = (s >= top_k || again) ? -1.f : 0.f;         // < 0: not part of the softmax
        if (ex[s] < 0.f) pv[s] = -INFINITY;
        mx = fmaxf(mx, pv[s]);
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        ex[s] = ex[s] < 0.f ? 0.f : expf(pv[s] - mx);
        den += ex[s];
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if (s < top_k) {
            route[t * top_k + s] = pick[s];
            weight[t * top_k + s] = ex[s] / den;
        }
    }
}

__global__ void moe_zero_kernel(int32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

constexpr int MAX_SEG = 4096;           // (pattern, expert) pairs: their counters fit in LDS
constexpr int PAIRS_PER_BLOCK = 1024;   // (token, slot) pairs per block of the two sorting passes

__device__ inline int pair_segment(const int32_t *route, const int32_t *pattern_id, int64_t i, int L, int P, int E,
                                   int top_k)
{
    const int64_t t = i / top_k;
    const int p = pattern_id ? min(max(pattern_id[t / L], 0), P - 1) : 0;
    return p * E + route[i];
}

// counts[seg] += 1 for every (token, slot); seg = pattern(token) * E + expert.  Counted in LDS first so that
// the global counters see one atomic per (block, segment).
__global__ __launch_bounds__(256) void moe_count_kernel(const int32_t *__restrict__ route, const int32_t *__restrict__ pattern_id,
                                                        int64_t pairs, int L, int P, int E, int top_k,
                                                        int32_t *__restrict__ counts)
{
    __shared__ int hist[MAX_SEG];
    const int n_seg = P * E;
    for (int s = threadIdx.x; s < n_seg; s += 256) hist[s] = 0;
    __syncthreads();
    const int64_t i0 = (int64_t)blockIdx.x * PAIRS_PER_BLOCK;
    for (int j = threadIdx.x; j < PAIRS_PER_BLOCK; j += 256) {
        const int64_t i = i0 + j;
        if (i < pairs) atomicAdd(&hist[pair_segment(route, pattern_id, i, L, P, E, top_k)], 1);
    }
    __syncthreads();
    for (int s = threadIdx.x; s < n_seg; s += 256)
        if (hist[s]) atomicAdd(&counts[s], hist[s]);
}

// Segment bases (each segment padded to a multiple of SEG_ROWS), the segment of every 256-row block
// (unused blocks: -1, which the GEMMs skip), the fill cursors and the padded width of every segment's
// expert.  One block; n_seg <= MAX_SEG, staged in LDS.
__global__ __launch_bounds__(256) void moe_layout_kernel(const int32_t *__restrict__ counts, int n_seg, int n_blocks_max,
                                                         const int32_t *__restrict__ k_ffn, int E, int ffn_pad, int Fp,
                                                         int32_t *__restrict__ seg_base, int32_t *__restrict__ cursor,
                                                         int32_t *__restrict__ blk_seg, int32_t *__restrict__ seg_width)
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
        if (s < n_seg) {
            cursor[s] = 0;
            const int k = min(max(k_ffn[s % E], 1), Fp);
            seg_width[s] = min((k + ffn_pad - 1) / ffn_pad * ffn_pad, Fp);
        }
    }
    const int total_blocks = first_blk[n_seg];
    for (int j = threadIdx.x; j < n_blocks_max; j += 256) {
        int s = -1;
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

// pos[token, slot] = row of the pair in the gathered order: rank inside the block from LDS atomics, the
// block's range inside the segment from one global atomic per (block, segment).
__global__ __launch_bounds__(256) void moe_place_kernel(const int32_t *__restrict__ route, const int32_t *__restrict__ pattern_id,
                                                        int64_t pairs, int L, int P, int E, int top_k,
                                                        const int32_t *__restrict__ seg_base, int32_t *__restrict__ cursor,
                                                        int32_t *__restrict__ pos, int32_t *__restrict__ src_row)
{
    __shared__ int hist[MAX_SEG];
    constexpr int PER = PAIRS_PER_BLOCK / 256;
    const int n_seg = P * E;
    for (int s = threadIdx.x; s < n_seg; s += 256) hist[s] = 0;
    __syncthreads();
    const int64_t i0 = (int64_t)blockIdx.x * PAIRS_PER_BLOCK;
    int seg[PER], rank[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int64_t i = i0 + q * 256 + threadIdx.x;
        seg[q] = -1;
        rank[q] = 0;
        if (i < pairs) {
            seg[q] = pair_segment(route, pattern_id, i, L, P, E, top_k);
            rank[q] = atomicAdd(&hist[seg[q]], 1);
        }
    }
    __syncthreads();
    for (int s = threadIdx.x; s < n_seg; s += 256) {
        const int n = hist[s];
        hist[s] = seg_base[s] + (n ? atomicAdd(&cursor[s], n) : 0);
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PER; ++q)
        if (seg[q] >= 0) {
            const int64_t i = i0 + q * 256 + threadIdx.x;
            const int at = hist[seg[q]] + rank[q];
            pos[i] = at;
            src_row[at] = (int32_t)(i / top_k);             // the token whose row the GEMM reads for gathered row `at`
        }
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

// Y[t, :] = [X[t, :] +] sum_s weight[t, s] * Yg[pos[t, s], :]; one wave per token, 16 bytes of X and Y per lane
template <class T>
__global__ __launch_bounds__(256) void moe_combine_kernel(const T *__restrict__ X, const float *__restrict__ yg,
                                                          const int32_t *__restrict__ pos, const float *__restrict__ weight,
                                                          int64_t rows, int d, int top_k, int add_residual, T *__restrict__ Y)
{
    constexpr int VN = Vec16<T>::N;
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= rows) return;
    float w[8];
    int64_t src[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        w[s] = s < top_k ? weight[t * top_k + s] : 0.f;
        src[s] = s < top_k ? (int64_t)pos[t * top_k + s] * d : 0;
    }
    for (int c = lane * VN; c < d; c += 64 * VN) {          // d % VN == 0 checked on the host
        float acc[VN];
        if (add_residual) Vec16<T>::load(X + t * d + c, acc);
        else {
#pragma unroll
            for (int e = 0; e < VN; ++e) acc[e] = 0.f;
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            if (s < top_k) {
#pragma unroll
                for (int h = 0; h < VN / 4; ++h) {
                    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(yg + src[s] + c) + h);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[h * 4 + e] = fmaf(w[s], v[e], acc[h * 4 + e]);
                }
            }
        }
        if constexpr (VN == 8) {
            uint4 o;
            uint32_t *ow = reinterpret_cast<uint32_t *>(&o);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const h16 lo = from_f32<h16>(acc[2 * e]), hi = from_f32<h16>(acc[2 * e + 1]);
                ow[e] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
            }
            *reinterpret_cast<uint4 *>(Y + t * d + c) = o;
        } else {
            f32x4 o = {acc[0], acc[1], acc[2], acc[3]};
            *reinterpret_cast<f32x4 *>(Y + t * d + c) = o;
        }
    }
}

struct MoeWs {
    void *xn, *xg, *hg; float *yg, *weight; int32_t *route, *pos, *counts, *seg_base, *cursor, *blk_seg, *seg_width, *src_row;
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
    w.seg_width = c.take<int32_t>(n_seg);
    w.src_row = c.take<int32_t>(grows);
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
    if (!m->k_ffn) return fail(SF_ERR_INVALID_ARG, "moe_ffn: k_ffn (device keep counts) missing");
    if ((int64_t)D.P * m->n_experts > MAX_SEG) return fail(SF_ERR_SHAPE, "moe_ffn: more than %d (pattern, expert) pairs", MAX_SEG);
    if (D.d % (D.dtype == SF_BF16 ? 8 : 4)) return fail(SF_ERR_SHAPE, "moe_ffn: rows of d_model elements must be a multiple of 16 bytes");
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
    if (((uintptr_t)X | (uintptr_t)Y | (uintptr_t)m->Wr) & 15)
        return fail(SF_ERR_INVALID_ARG, "moe_ffn: X, Y and Wr must be 16-byte aligned");
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
        dim3 grid((unsigned)((rows + TOK_PER_BLOCK - 1) / TOK_PER_BLOCK));
        const size_t wbytes = (size_t)E * D.d * es;
        const size_t lgbytes = ((size_t)TOK_PER_BLOCK * (E + 1) * sizeof(float) + 15) & ~(size_t)15;
        const bool wlds = lgbytes + wbytes <= 64 * 1024;
#define SF_ROUTER(T, EB)                                                                                              \
    do {                                                                                                              \
        if (wlds)                                                                                                     \
            hipLaunchKernelGGL((moe_router_kernel<T, EB, true>), grid, dim3(256), lgbytes + wbytes, st, (const T *)xin,         \
                               (const T *)m->Wr, (const T *)m->br, rows, D.d, E, k, forced_route, w.route, w.weight,  \
                               logit_out);                                                                            \
        else                                                                                                          \
            hipLaunchKernelGGL((moe_router_kernel<T, EB, false>), grid, dim3(256), lgbytes, st, (const T *)xin,             \
                               (const T *)m->Wr, (const T *)m->br, rows, D.d, E, k, forced_route, w.route, w.weight,  \
                               logit_out);                                                                            \
    } while (0)
        if (bf) {
            if (E <= 8) SF_ROUTER(h16, 8);
            else if (E <= 16) SF_ROUTER(h16, 16);
            else SF_ROUTER(h16, 64);
        } else {
            if (E <= 8) SF_ROUTER(float, 8);
            else if (E <= 16) SF_ROUTER(float, 16);
            else SF_ROUTER(float, 64);
        }
#undef SF_ROUTER
    }
    // counting sort of the (token, slot) pairs by (pattern, expert)
    const unsigned sort_blocks = (unsigned)((pairs + PAIRS_PER_BLOCK - 1) / PAIRS_PER_BLOCK);
    hipLaunchKernelGGL(moe_zero_kernel, dim3(ceil_div(n_seg, 256)), dim3(256), 0, st, w.counts, n_seg);
    // rows of padding read token 0 (their results are never used)
    hipLaunchKernelGGL(moe_zero_kernel, dim3(ceil_div(w.n_blocks_max * SEG_ROWS, 256)), dim3(256), 0, st, w.src_row,
                       w.n_blocks_max * SEG_ROWS);
    hipLaunchKernelGGL(moe_count_kernel, dim3(sort_blocks), dim3(256), 0, st, w.route, pattern_id, pairs, D.L, D.P, E, k,
                       w.counts);
    hipLaunchKernelGGL(moe_layout_kernel, dim3(1), dim3(256), 0, st, w.counts, n_seg, w.n_blocks_max, m->k_ffn, E,
                       D.ffn_pad, w.Fp, w.seg_base, w.cursor, w.blk_seg, w.seg_width);
    hipLaunchKernelGGL(moe_place_kernel, dim3(sort_blocks), dim3(256), 0, st, w.route, pattern_id, pairs, D.L, D.P, E, k,
                       w.seg_base, w.cursor, w.pos, w.src_row);
    // first GEMM over 256-row blocks; the block's segment selects the weights.  Large bf16 problems read the
    // token rows through the row map, the others from a gathered copy.
    GemmArgs g{};
    g.A = xin; g.lda = D.d; g.W = m->W1; g.ldw = D.d; g.w_pstride = (int64_t)w.Fp * D.d;
    g.bias = m->b1; g.bias_pstride = w.Fp; g.pattern_id = w.blk_seg; g.n_lim = w.seg_width; g.xcd_rows = 1;
    g.B = w.n_blocks_max; g.L = SEG_ROWS; g.N = w.Fp; g.K = D.d; g.epi = EPI_ROWMAJOR;
    g.act = D.act == SF_GELU_ERF ? ACT_GELU : ACT_RELU;
    g.C = w.hg; g.ldc = w.Fp;
    g.row_map = w.src_row;
    if (!(rows * D.d * 2 < ((int64_t)1 << 32) && gemm_takes_row_map(D.dtype, g))) {
        const size_t row_bytes = (size_t)D.d * es;
        dim3 grid((unsigned)((pairs + 3) / 4));
        if (row_bytes % 16 == 0 && ((uintptr_t)xin % 16 == 0))
            hipLaunchKernelGGL(moe_gather_kernel<uint4>, grid, dim3(256), 0, st, (const uint4 *)xin, w.pos, pairs, k,
                               (int)(row_bytes / 16), (uint4 *)w.xg);
        else
            hipLaunchKernelGGL(moe_gather_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t *)xin, w.pos, pairs,
                               k, (int)(row_bytes / 2), (uint16_t *)w.xg);
        g.A = w.xg;
        g.row_map = nullptr;
    }
    if (int32_t rc = gemm(D.dtype, g, st)) return rc;
    GemmArgs h{};
    h.A = w.hg; h.lda = w.Fp; h.W = m->W2T; h.ldw = w.Fp; h.w_pstride = (int64_t)D.d * w.Fp;
    h.bias = m->b2x; h.bias_pstride = D.d; h.pattern_id = w.blk_seg; h.k_lim = w.seg_width; h.xcd_rows = 1;
    h.B = w.n_blocks_max; h.L = SEG_ROWS; h.N = D.d; h.K = w.Fp; h.epi = EPI_ROWMAJOR; h.act = ACT_NONE;
    h.C = w.yg; h.ldc = D.d; h.c_f32 = 1;
    if (int32_t rc = gemm(D.dtype, h, st)) return rc;
    {
        dim3 grid((unsigned)((rows + 3) / 4));
        if (bf)
            hipLaunchKernelGGL(moe_combine_kernel<h16>, grid, dim3(256), 0, st, (const h16 *)X, w.yg, w.pos,
                               w.weight, rows, D.d, k, add_residual, (h16 *)Y);
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
