// SentryGate on the device: the importance scores of Eq. (1) for every layer and presence pattern, and
// the global threshold that meets a cost budget (Sec. 4.5, the paragraph that introduces the three pruning
// locations; Sec. 4.2 names the FLOPs / energy budget).  Both are plan-construction steps: tiny next to the
// encoder forward, so the kernels aim at being exact and launch-cheap, not at a roofline.
#include "common.hpp"

namespace sf {

namespace {

constexpr int MAX_HIDDEN = 1024;
constexpr int MAX_LAYERS_BUDGET = 64;

// g[l, p, i] = sigmoid(zeta[l, i] + gamma[l] * (Wb[l, i, :] . h + cb[l, i])),  h = nonlin(Wa[l] m_p + ba[l]).
// grid (ceil(n_units / 256), P, nl).  Eight lanes share one unit's output row (one 128-byte line per step).
__global__ __launch_bounds__(256) void gate_eval_kernel(
    const float *__restrict__ Wa, const float *__restrict__ ba, const float *__restrict__ Wb,
    const float *__restrict__ cb, const float *__restrict__ zeta, const float *__restrict__ gamma,
    const int32_t *__restrict__ pattern_bits, int M, int Hd, int n_units, int Hq, int nonlin, int P,
    float *__restrict__ g_head, float *__restrict__ g_ffn)
{
    __shared__ float h[MAX_HIDDEN];
    const int l = blockIdx.z, p = blockIdx.y;
    const uint32_t bits = (uint32_t)pattern_bits[p];
    for (int r = threadIdx.x; r < Hd; r += 256) {
        float a = ba ? ba[(int64_t)l * Hd + r] : 0.f;
        for (int j = 0; j < M; ++j)
            if ((bits >> j) & 1u) a += Wa[((int64_t)l * Hd + r) * M + j];
        h[r] = nonlin == 0 ? fmaxf(a, 0.f) : tanhf(a);
    }
    __syncthreads();
    const int sub = threadIdx.x & 7;
    const int F = n_units - Hq;
    const float gm = gamma[l];
    for (int u0 = 0; u0 < 256; u0 += 32) {
        const int i = blockIdx.x * 256 + u0 + (threadIdx.x >> 3);       // uniform over the 8 lanes of a unit
        float acc = 0.f;
        if (i < n_units) {
            const float *w = Wb + ((int64_t)l * n_units + i) * Hd;
            if ((Hd & 3) == 0) {
                for (int r = sub * 4; r < Hd; r += 32) {
                    const f32x4 q = *reinterpret_cast<const f32x4 *>(w + r);
                    acc = fmaf(q[0], h[r], acc);
                    acc = fmaf(q[1], h[r + 1], acc);
                    acc = fmaf(q[2], h[r + 2], acc);
                    acc = fmaf(q[3], h[r + 3], acc);
                }
            } else {
                for (int r = sub; r < Hd; r += 8) acc = fmaf(w[r], h[r], acc);
            }
        }
        acc += __shfl_xor(acc, 1);
        acc += __shfl_xor(acc, 2);
        acc += __shfl_xor(acc, 4);
        if (i < n_units && sub == 0) {
            const float f = acc + (cb ? cb[(int64_t)l * n_units + i] : 0.f);
            const float z = zeta[(int64_t)l * n_units + i] + gm * f;
            const float g = 1.f / (1.f + expf(-z));
            if (i < Hq) g_head[((int64_t)l * P + p) * Hq + i] = g;
            else g_ffn[((int64_t)l * P + p) * F + (i - Hq)] = g;
        }
    }
}

// Order-preserving map float -> uint32 (a >= b  <=>  key(a) >= key(b) for non-NaN; -0 and +0 share a key)
__device__ inline uint32_t score_key(float f)
{
    if (f == 0.f) f = 0.f;
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float key_score(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

struct BudgetCosts { int64_t head[MAX_LAYERS_BUDGET], group[MAX_LAYERS_BUDGET], ffn[MAX_LAYERS_BUDGET]; };

// One block.  Sizes of the keep set { key(score) >= K } per layer (before the one-unit floor), into LDS.
// `none` keeps nothing (the one-unit-per-layer network).
__device__ void count_keep(const float *__restrict__ gh, const float *__restrict__ gf, int64_t lstride_h,
                           int64_t lstride_f, int nl, int Hq, int Hk, int F, uint32_t K, bool none, int *kh, int *kg,
                           int *kf, unsigned long long *gmask)
{
    const int tid = threadIdx.x, lane = tid & 63;
    for (int l = tid; l < nl; l += blockDim.x) { kh[l] = 0; kf[l] = 0; gmask[l] = 0ull; }
    __syncthreads();
    if (!none) {
        const int per_group = Hq / Hk;
        for (int l = 0; l < nl; ++l) {
            int c = 0;
            for (int i = tid; i < F; i += blockDim.x) c += score_key(gf[l * lstride_f + i]) >= K;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);
            if (lane == 0 && c) atomicAdd(&kf[l], c);
            for (int hd = tid; hd < Hq; hd += blockDim.x)
                if (score_key(gh[l * lstride_h + hd]) >= K) {
                    atomicAdd(&kh[l], 1);
                    atomicOr(&gmask[l], 1ull << (hd / per_group));
                }
        }
    }
    __syncthreads();
    for (int l = tid; l < nl; l += blockDim.x) {
        kg[l] = __popcll(gmask[l]);
        if (kh[l] == 0) { kh[l] = 1; kg[l] = 1; }                   // the best head stays, with its group
        if (kf[l] == 0) kf[l] = 1;                                  // the best channel stays
    }
    __syncthreads();
}

__global__ __launch_bounds__(1024) void budget_search_kernel(
    const float *__restrict__ gh, const float *__restrict__ gf, int64_t lstride_h, int64_t lstride_f, int nl, int Hq,
    int Hk, int F, BudgetCosts costs, int64_t c_fixed, int64_t budget, float *__restrict__ tau_out,
    int32_t *__restrict__ k_head_out, int32_t *__restrict__ k_ffn_out, int64_t *__restrict__ cost_out,
    int32_t *__restrict__ feasible_out)
{
    __shared__ int kh[MAX_LAYERS_BUDGET], kg[MAX_LAYERS_BUDGET], kf[MAX_LAYERS_BUDGET];
    __shared__ unsigned long long gmask[MAX_LAYERS_BUDGET];
    __shared__ uint32_t s_key;
    __shared__ int s_ok;
    const int tid = threadIdx.x;

    auto cost_now = [&]() {                                          // thread 0, after count_keep
        int64_t c = c_fixed;
        for (int l = 0; l < nl; ++l) c += kh[l] * costs.head[l] + kg[l] * costs.group[l] + kf[l] * costs.ffn[l];
        return c;
    };

    // the largest score present: the strictest threshold that is a candidate
    if (tid == 0) s_key = 0u;
    __syncthreads();
    {
        uint32_t mk = 0u;
        for (int l = 0; l < nl; ++l) {
            for (int i = tid; i < F; i += blockDim.x) mk = max(mk, score_key(gf[l * lstride_f + i]));
            for (int i = tid; i < Hq; i += blockDim.x) mk = max(mk, score_key(gh[l * lstride_h + i]));
        }
        atomicMax(&s_key, mk);
    }
    __syncthreads();
    const uint32_t max_key = s_key;
    __syncthreads();

    count_keep(gh, gf, lstride_h, lstride_f, nl, Hq, Hk, F, max_key, false, kh, kg, kf, gmask);
    if (tid == 0) s_ok = cost_now() <= budget;
    __syncthreads();
    const bool feasible = s_ok != 0;
    __syncthreads();

    uint32_t lo = 0u, hi = max_key;                                  // smallest K in [lo, hi] whose keep set fits
    if (feasible) {
        while (lo < hi) {                                            // uniform over the block
            const uint32_t mid = lo + (hi - lo) / 2;
            count_keep(gh, gf, lstride_h, lstride_f, nl, Hq, Hk, F, mid, false, kh, kg, kf, gmask);
            if (tid == 0) s_ok = cost_now() <= budget;
            __syncthreads();
            if (s_ok) hi = mid; else lo = mid + 1;
            __syncthreads();
        }
    }
    // final keep set, its cost, and the threshold as a score value: the smallest score >= K
    count_keep(gh, gf, lstride_h, lstride_f, nl, Hq, Hk, F, lo, !feasible, kh, kg, kf, gmask);
    if (tid == 0) s_key = 0xffffffffu;
    __syncthreads();
    if (feasible) {
        uint32_t mk = 0xffffffffu;
        for (int l = 0; l < nl; ++l) {
            for (int i = tid; i < F; i += blockDim.x) {
                const uint32_t k = score_key(gf[l * lstride_f + i]);
                if (k >= lo) mk = min(mk, k);
            }
            for (int i = tid; i < Hq; i += blockDim.x) {
                const uint32_t k = score_key(gh[l * lstride_h + i]);
                if (k >= lo) mk = min(mk, k);
            }
        }
        atomicMin(&s_key, mk);
    }
    __syncthreads();
    for (int l = tid; l < nl; l += blockDim.x) { k_head_out[l] = kh[l]; k_ffn_out[l] = kf[l]; }
    if (tid == 0) {
        *tau_out = feasible ? key_score(s_key) : INFINITY;
        *cost_out = cost_now();
        *feasible_out = feasible ? 1 : 0;
    }
}

}  // namespace

}  // namespace sf

using namespace sf;

extern "C" int32_t sf_gate_eval(const sf_desc *desc, const sf_gate_params *gp, const int32_t *pattern_bits,
                                float *g_head, float *g_ffn, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!gp || !pattern_bits || !g_head || !g_ffn) return fail(SF_ERR_INVALID_ARG, "gate_eval: NULL argument");
    if (gp->n_modalities < 1 || gp->n_modalities > 32 || gp->hidden < 1 || gp->hidden > MAX_HIDDEN)
        return fail(SF_ERR_INVALID_ARG, "gate_eval: needs 1 <= n_modalities <= 32 and 1 <= hidden <= %d", MAX_HIDDEN);
    if (gp->nonlin != SF_GATE_RELU && gp->nonlin != SF_GATE_TANH)
        return fail(SF_ERR_UNSUPPORTED, "gate_eval: unknown nonlinearity");
    if (!gp->Wa || !gp->Wb || !gp->zeta || !gp->gamma) return fail(SF_ERR_INVALID_ARG, "gate_eval: NULL parameter pointer");
    if ((uintptr_t)gp->Wb & 15) return fail(SF_ERR_INVALID_ARG, "gate_eval: Wb must be 16-byte aligned");
    if (D.P > 65535 || D.nl > 65535) return fail(SF_ERR_SHAPE, "gate_eval: too many patterns or layers");
    const int n_units = D.Hq + D.F;
    dim3 grid(ceil_div(n_units, 256), D.P, D.nl);
    hipLaunchKernelGGL(gate_eval_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), (const float *)gp->Wa,
                       (const float *)gp->ba, (const float *)gp->Wb, (const float *)gp->cb, (const float *)gp->zeta,
                       (const float *)gp->gamma, pattern_bits, gp->n_modalities, gp->hidden, n_units, D.Hq, gp->nonlin,
                       D.P, g_head, g_ffn);
    return check_launch("gate_eval");
}

extern "C" int32_t sf_budget_search(const sf_desc *desc, const float *g_head, const float *g_ffn, int32_t pattern,
                                    const int64_t *c_head_host, const int64_t *c_group_host,
                                    const int64_t *c_ffn_host, int64_t c_fixed, int64_t budget, float *tau,
                                    int32_t *k_head, int32_t *k_ffn, int64_t *cost, int32_t *feasible, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!g_head || !g_ffn || !c_head_host || !c_group_host || !c_ffn_host || !tau || !k_head || !k_ffn || !cost ||
        !feasible)
        return fail(SF_ERR_INVALID_ARG, "budget_search: NULL argument");
    if (pattern < 0 || pattern >= D.P) return fail(SF_ERR_INVALID_ARG, "budget_search: pattern %d out of range", pattern);
    if (D.nl > MAX_LAYERS_BUDGET) return fail(SF_ERR_SHAPE, "budget_search: at most %d layers", MAX_LAYERS_BUDGET);
    if (D.Hk > 64) return fail(SF_ERR_SHAPE, "budget_search: at most 64 K/V groups");
    BudgetCosts bc{};
    for (int l = 0; l < D.nl; ++l) {
        if (c_head_host[l] < 0 || c_group_host[l] < 0 || c_ffn_host[l] < 0)
            return fail(SF_ERR_INVALID_ARG, "budget_search: negative cost in layer %d", l);
        bc.head[l] = c_head_host[l]; bc.group[l] = c_group_host[l]; bc.ffn[l] = c_ffn_host[l];
    }
    hipLaunchKernelGGL(budget_search_kernel, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(stream),
                       g_head + (int64_t)pattern * D.Hq, g_ffn + (int64_t)pattern * D.F, (int64_t)D.P * D.Hq,
                       (int64_t)D.P * D.F, D.nl, D.Hq, D.Hk, D.F, bc, c_fixed, budget, tau, k_head, k_ffn, cost, feasible);
    return check_launch("budget_search");
}
