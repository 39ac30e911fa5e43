// Internal interface of SentryAttend (sparse grouped-query attention,
// Sec. 4.4 of the paper, Eq. (6)).
#pragma once

#include "common.hpp"

namespace sf {

struct AttnArgs {
    int B, nH, nG, L, dh, U;                 // U active queries per head, 0..L
    const void *Q, *K, *V;
    sf_strides sq, sk, sv;
    int v_transposed;                        // V is [B,nG,dh,L] (sv.l = stride between dh rows)
    const int32_t *head_group; int hg_stride;   // head_group[pattern(b)*hg_stride + h]
    const int32_t *pattern_id;               // [B] or NULL
    const uint8_t *key_valid;                // [B,L] or NULL
    const int32_t *sample_idx; int n_sample; // [B,n_sample] key sample of the sparsity score, or NULL / 0
    const int32_t *u_active;                 // [B] or NULL: sample b selects min(u_active[b], U) queries (needs U < L)
    const int32_t *forced_sel;               // [B,selH,U] or NULL
    void *O; int64_t ldo;                    // [B,L,nH*dh]
    int32_t *sel_out;                        // [B,selH,U] or NULL
    float *score_out;                        // [B,selH,L] or NULL
    int selH;                                // heads per sample in forced_sel / sel_out / score_out (0 = nH)
    int skip_fill;                           // leave the lazy rows of O unwritten (the caller projects them itself)
    // Samples packed back to back in token-major Q, K, V and O (token compaction without padding): sample b starts
    // at row row0[b] (its batch strides are not used; V is token-major) and owns ext[b] >= its length rows of O,
    // the rows behind its tokens being padding that the fill gives the context vector (so that every row of O is
    // defined).  The per-sample arrays of the workspace, key_valid, sel and score keep their [B, ..., L] shape, L =
    // the longest sequence a sample may have; key_valid marks the sample's own rows.  NULL: samples b*L apart.
    const int32_t *row0, *ext;
    // [B, ceil(L/32)] or NULL: bit i of sample b is set when some head selected row i (cleared by the statistics
    // pass, set by the selection; what the active-row output projection starts from)
    uint32_t *act_bits;
    void *ws; size_t ws_bytes;
};

// Element offset of sample b in a token-major tensor with strides s, and its first row in O
__device__ __forceinline__ int64_t sample_offset(const int32_t *row0, int b, const sf_strides &s)
{
    return row0 ? (int64_t)row0[b] * s.l : (int64_t)b * s.b;
}
__device__ __forceinline__ int64_t sample_row(const int32_t *row0, int b, int L)
{
    return row0 ? (int64_t)row0[b] : (int64_t)b * L;
}

// Pieces of the workspace (all sizes derive from the same few integers, so the
// size query and the forward agree by construction).
struct AttnPlan {
    int splits;            // key splits of the active pass (1 = write O directly)
    int keys_per_split;    // multiple of 64
    int stat_chunks;       // partial-sum chunks of the K/V statistics
    int Upad;              // U rounded up to 32
    int Lp;                // L rounded up to 8 (row length of the transposed V copy)
    int Sp;                // key-sample size rounded up to 64 (0: no sample)
    size_t bytes;
    // carved pointers (NULL when planning only)
    void *vt; float *stat_part; float *stats; int32_t *n_valid; float *score;
    int32_t *sel; int32_t *slot; float *part_o; float *part_ml;
    void *ks; uint8_t *ks_valid; float *ks_stats; int32_t *n_keys;   // gathered key sample [B,nG,Sp,dh], its validity [B,Sp]
};
AttnPlan attn_plan(int dtype, const AttnArgs &a, void *ws);

int32_t attention_forward(int dtype, const AttnArgs &a, hipStream_t st);

// bf16 MFMA kernels (attention_bf16.hip)
// score [B,scoreH,L]; sel [B,selH,U].  The score is taken over the Lk keys `Kx` (strides skx) with
// validity key_mask [B,Lk] (NULL: all) and mean-key statistics `stats`; queries use a.key_valid.
int32_t score_bf16(const AttnArgs &a, const void *Kx, sf_strides skx, int Lk, const uint8_t *key_mask,
                   const float *stats, float *score, int scoreH, hipStream_t st);
int32_t attend_bf16(const AttnArgs &a, const AttnPlan &pl, const void *vt, sf_strides svt,
                    const int32_t *sel, int selH, hipStream_t st);

// Output projection when most rows are lazy (lazy_proj.hip).  lazy_cap: rows per sample of the compact buffers, 0
// when the shortcut does not apply.  slot [B,nH,L] and stats are the pieces of the attention plan.
int lazy_cap(int L, int nH, int U, int dh, int d);
void lazy_rows_active(const uint32_t *act_bits, const int32_t *pattern_id, int B, int L, int capA, int32_t *arow,
                      int32_t *pos_of, int32_t *n_act, int32_t *blk_pattern, hipStream_t st);
void lazy_att_compact(const void *att, int64_t ldo, const int32_t *slot, const float *stats, const int32_t *head_group,
                      int hg_stride, const int32_t *pattern_id, const int32_t *arow, const int32_t *n_act, int B, int nH,
                      int nG, int L, int dh, int capA, void *Ac, hipStream_t st);
// the compact rows and the projected context vectors c_b in one launch
void lazy_att_compact_ctx_proj(const void *att, int64_t ldo, const int32_t *slot, const float *stats,
                               const int32_t *head_group, int hg_stride, const int32_t *pattern_id, const int32_t *arow,
                               const int32_t *n_act, int B, int nH, int nG, int L, int dh, int capA, void *Ac,
                               const void *WoT, int64_t w_pstride, const void *bo, int d, float *cvec, hipStream_t st);
// FP8 arithmetic: the context vector quantised with 1/inv_sa, weights as E4M3 codes [P][d, ldw], ldw >= nH*dh
// (8-byte aligned rows)
void lazy_ctx_proj_q8(const float *stats, const int32_t *head_group, int hg_stride, const int32_t *pattern_id,
                      const void *WoT8, int64_t w_pstride, int ldw, const void *bo, int B, int nH, int nG, int dh, int d,
                      float inv_sa, float out_scale, float *cvec, hipStream_t st);
void lazy_combine_ln(const void *x, bool x_f32, const int32_t *pos_of, const float *Cc, const void *bo, const float *cvec,
                     int B, int L, int capA, const void *gamma, const void *beta, float eps, int d, float *x1, void *xn,
                     float q_inv, hipStream_t st);

constexpr int STAT_CHUNK = 128;     // keys per partial-sum block of the K/V statistics

}  // namespace sf
