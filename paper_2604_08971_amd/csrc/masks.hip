// gate_scores_to_masks: SentryGate scores -> keep masks, kept-index lists and
// the GQA-consistent K/V group keep set (Sec. 4.5 of the paper).
// Integer / fp32-compare work only: results are exact.
#include "common.hpp"
#include "topk.hpp"

namespace sf {

constexpr int MASK_NT = 256;
constexpr int MAX_LAYERS = 128;
struct KeepCounts { int k[MAX_LAYERS]; };

// Top-k of n scores of one (layer, pattern); called by every thread of the block.
// GROUPS: additionally derive the kept K/V groups of the kept heads.
template <bool GROUPS, int NT>
__device__ void keep_topk_block(const float *__restrict__ g, int n, int lp, int k, uint8_t *__restrict__ mask,
                                int32_t *__restrict__ idx, int Hk, int32_t *__restrict__ group_idx,
                                int32_t *__restrict__ n_groups, int32_t *__restrict__ head_group, uint32_t *keys,
                                int *scratch)
{
    const float *gs = g + (size_t)lp * n;
    uint8_t *m = mask + (size_t)lp * n;
    int32_t *ix = idx + (size_t)lp * n;

    for (int i = threadIdx.x; i < n; i += NT) keys[i] = sortable_key(gs[i]);
    __syncthreads();
    block_topk<NT>(keys, n, k, scratch, [&](int i, bool kept, int pos) {
        m[i] = kept ? 1 : 0;
        if (kept) ix[pos] = i;
    });
    for (int i = k + threadIdx.x; i < n; i += NT) ix[i] = -1;

    if (GROUPS) {
        // K_keep = floor(H_keep / (Hq/Hk)); groups no kept head refers to are dropped.
        __syncthreads();                     // ix[] written by other threads (global, same block)
        __threadfence_block();
        if (threadIdx.x == 0) {
            const int per = n / Hk;
            int32_t *gi = group_idx + (size_t)lp * Hk;
            int32_t *hg = head_group + (size_t)lp * n;
            int ng = 0;
            for (int i = 0; i < k; ++i) {    // ix ascending => groups ascending
                const int grp = ix[i] / per;
                if (ng == 0 || gi[ng - 1] != grp) gi[ng++] = grp;
                hg[i] = ng - 1;
            }
            for (int i = k; i < n; ++i) hg[i] = -1;
            for (int r = ng; r < Hk; ++r) gi[r] = -1;
            n_groups[lp] = ng;
        }
    }
}

// One launch for both unit types: blocks [0, nl*P) take the FFN channels of one (layer, pattern) - the long
// rows, scheduled first -, blocks [nl*P, 2*nl*P) its heads and K/V groups.  There are few blocks, so wide
// layers get NT = 1024 threads (2-4 keys per thread and radix pass).
template <int NT>
__global__ __launch_bounds__(NT) void keep_masks_kernel(
    const float *__restrict__ g_head, const float *__restrict__ g_ffn, int Hq, int Hk, int F, int P, int n_lp,
    KeepCounts kh, KeepCounts kf, uint8_t *__restrict__ head_mask, uint8_t *__restrict__ ffn_mask,
    int32_t *__restrict__ head_idx, int32_t *__restrict__ ffn_idx, int32_t *__restrict__ group_idx,
    int32_t *__restrict__ n_groups, int32_t *__restrict__ head_group)
{
    extern __shared__ uint32_t keys[];
    __shared__ int scratch[TOPK_SCRATCH];
    if ((int)blockIdx.x < n_lp) {
        const int lp = blockIdx.x;
        keep_topk_block<false, NT>(g_ffn, F, lp, kf.k[lp / P], ffn_mask, ffn_idx, 0, nullptr, nullptr, nullptr, keys, scratch);
    } else {
        const int lp = blockIdx.x - n_lp;
        keep_topk_block<true, NT>(g_head, Hq, lp, kh.k[lp / P], head_mask, head_idx, Hk, group_idx, n_groups, head_group,
                                  keys, scratch);
    }
}

// Sec. 4.2 / 4.4: position j of the concatenated token sequence is an allowed key of sample b iff it belongs to
// no modality (tok_modality < 0: fusion tokens) or to one that sample b has.  One thread per 4 positions.
__global__ __launch_bounds__(256) void presence_to_key_valid_kernel(const uint8_t *__restrict__ presence,
                                                                    const int32_t *__restrict__ tok_modality, int B,
                                                                    int M, int L, uint8_t *__restrict__ key_valid)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;     // over B * ceil(L/4)
    const int L4 = (L + 3) >> 2;
    if (i >= (int64_t)B * L4) return;
    const int b = (int)(i / L4), j0 = (int)(i % L4) * 4;
    const uint8_t *pr = presence + (int64_t)b * M;
    uint8_t *out = key_valid + (int64_t)b * L;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int j = j0 + e;
        if (j < L) {
            const int m = tok_modality[j];
            out[j] = (m < 0 || (m < M && pr[m] != 0)) ? 1 : 0;     // an id >= M is refused by the host when it can see it
        }
    }
}

}  // namespace sf

using namespace sf;

extern "C" int32_t sf_presence_to_key_valid(const uint8_t *presence, const int32_t *tok_modality, int32_t B,
                                            int32_t M, int32_t L, uint8_t *key_valid, void *stream)
{
    if (B < 1 || L < 1 || M < 0 || M > 64) return fail(SF_ERR_INVALID_ARG, "presence_to_key_valid: B, L >= 1 and 0 <= M <= 64 required");
    if (!tok_modality || !key_valid || (M > 0 && !presence))
        return fail(SF_ERR_INVALID_ARG, "presence_to_key_valid: NULL argument");
    if ((int64_t)B * L > (int64_t)1 << 31) return fail(SF_ERR_SHAPE, "presence_to_key_valid: B*L too large");
    const int64_t n = (int64_t)B * ((L + 3) / 4);
    hipLaunchKernelGGL(presence_to_key_valid_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), presence, tok_modality, B, M, L, key_valid);
    return check_launch("presence_to_key_valid");
}

extern "C" int32_t sf_gate_scores_to_masks(const sf_desc *desc, const float *g_head,
                                           const float *g_ffn, const int32_t *k_head_host,
                                           const int32_t *k_ffn_host, uint8_t *head_mask,
                                           uint8_t *ffn_mask, int32_t *head_idx, int32_t *ffn_idx,
                                           int32_t *group_idx, int32_t *n_groups,
                                           int32_t *head_group, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!g_head || !g_ffn || !k_head_host || !k_ffn_host || !head_mask || !ffn_mask || !head_idx ||
        !ffn_idx || !group_idx || !n_groups || !head_group)
        return fail(SF_ERR_INVALID_ARG, "gate_scores_to_masks: NULL argument");
    if (D.Hq > 64 || D.F > 16384 || D.nl > MAX_LAYERS)
        return fail(SF_ERR_SHAPE, "gate_scores_to_masks: needs Hq <= 64, d_ff <= 16384, n_layers <= %d",
                    MAX_LAYERS);
    KeepCounts kh{}, kf{};
    for (int l = 0; l < D.nl; ++l) {
        if (k_head_host[l] < 1 || k_head_host[l] > D.Hq || k_ffn_host[l] < 1 || k_ffn_host[l] > D.F)
            return fail(SF_ERR_INVALID_ARG, "gate_scores_to_masks: keep count out of range at layer %d", l);
        kh.k[l] = k_head_host[l];
        kf.k[l] = k_ffn_host[l];
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int blocks = D.nl * D.P;
    const size_t lds = (size_t)(D.F > D.Hq ? D.F : D.Hq) * sizeof(uint32_t);
#define SF_MASK_ARGS dim3(2 * blocks), dim3(NT_), lds, st, g_head, g_ffn, D.Hq, D.Hk, D.F, D.P, blocks, kh, kf, head_mask, \
                     ffn_mask, head_idx, ffn_idx, group_idx, n_groups, head_group
    if (D.F >= 2048) {
        constexpr int NT_ = 1024;
        hipLaunchKernelGGL(keep_masks_kernel<NT_>, SF_MASK_ARGS);
    } else {
        constexpr int NT_ = MASK_NT;
        hipLaunchKernelGGL(keep_masks_kernel<NT_>, SF_MASK_ARGS);
    }
#undef SF_MASK_ARGS
    return check_launch("gate_scores_to_masks");
}
