/*
 * sentryfuse.h -- C ABI of the MI355X (gfx950) library for the pruned
 * multimodal encoder forward of SentryFuse: SentryGate keep-masks (Sec. 4.2,
 * Sec. 4.5 of the paper), their compaction into dense weight slices
 * (Sec. 4.5), SentryAttend sparse grouped-query attention (Sec. 4.4, Eq. (6)),
 * the pruned FFN (Sec. 4.5) and the pre-norm encoder stack around them.
 *
 * Conventions shared by every entry point
 *  - Every pointer is a DEVICE pointer unless its name ends in `_host`.
 *  - Every buffer is allocated and freed by the caller.  The library keeps no
 *    pointer after a call returns and allocates no device memory; scratch
 *    comes from the (workspace, workspace_bytes) pair, sized by the matching
 *    sf_*_workspace_bytes query.  Workspace must be 256-byte aligned.
 *  - `stream` is a hipStream_t.  Calls only enqueue work; outputs are valid
 *    once the caller has synchronised the stream.  Two calls that share a
 *    workspace must be ordered on one stream.
 *  - Return value: SF_OK or a negative sf_status.  On any error other than
 *    SF_ERR_HIP nothing has been enqueued and no output was touched.
 *    sf_last_error() returns a thread-local message for the last failure.
 *  - Results are deterministic: no floating-point atomics; the same inputs
 *    give the same bits.
 *  - dtype SF_F32: all floating tensors are fp32, fp32 arithmetic.
 *    dtype SF_BF16: all floating tensors (activations, weights, biases,
 *    LayerNorm parameters) are bf16; contractions run on bf16 MFMA with fp32
 *    accumulation; stored tensors are rounded to bf16 (nearest even) at: the
 *    LayerNorm output, Q, K, V, the attention output, the FFN hidden after
 *    the activation, and the output Y of each entry point.  Inside
 *    sf_encoder_forward the residual stream between layers is an fp32
 *    accumulation and is not rounded.
 *    dtype SF_F16: the FP16 variant of the model - the same, with IEEE
 *    binary16 in place of bf16 everywhere (fp16 MFMA, fp32 accumulation,
 *    round to nearest even at the same points; values beyond +-65504
 *    overflow to infinity, the caller's weights and activations must fit).
 *    It is served by a second build of these sources, libsentryfuse_f16.so
 *    (same entry points); libsentryfuse.so takes SF_F32 and SF_BF16 models,
 *    libsentryfuse_f16.so SF_F32 and SF_F16 models, the other 16-bit type
 *    returns SF_ERR_UNSUPPORTED.  Of the FP8 entry points the FP16 build runs
 *    the encoder ones (sf_compact_ffn_fp8, sf_compact_proj_fp8,
 *    sf_encoder_forward_fp8ffn, sf_encoder_forward_fp8); E4M3-stored weights
 *    (sf_compact_heads_channels_fp8), the stand-alone FFN block
 *    (sf_pruned_ffn_fp8_forward) and sf_quantize_fp8 on 16-bit input are built
 *    for bf16 models only.  Wherever a comment
 *    below says "bf16" for the model dtype, the FP16 build reads "binary16".
 *  - Gate scores, sparsity scores and all index tensors are fp32 / int32 /
 *    uint8 regardless of dtype.
 */
#ifndef SENTRYFUSE_H
#define SENTRYFUSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sf_status {
    SF_OK = 0,
    SF_ERR_INVALID_ARG = -1,   /* NULL where data is required, counts out of range */
    SF_ERR_SHAPE = -2,         /* sizes the kernels cannot take (see each call) */
    SF_ERR_UNSUPPORTED = -3,   /* dtype / flag combination not built */
    SF_ERR_WORKSPACE = -4,     /* workspace missing, misaligned or too small */
    SF_ERR_HIP = -5            /* a HIP launch failed; see sf_last_error() */
} sf_status;

enum { SF_F32 = 0, SF_BF16 = 1, SF_F16 = 2 };
enum { SF_RELU = 0, SF_GELU_ERF = 1 };
enum { SF_FLAG_FINAL_LN = 1u };

/* Problem descriptor (plain data).  Set struct_size = sizeof(sf_desc). */
typedef struct sf_desc {
    uint32_t struct_size;
    int32_t B;          /* samples */
    int32_t L;          /* tokens per sample (all modalities concatenated), the paper's T */
    int32_t d_model;    /* multiple of 8 (bf16) */
    int32_t Hq;         /* query heads of the dense model */
    int32_t Hk;         /* K/V groups of the dense model, Hq % Hk == 0 */
    int32_t dh;         /* head dim; bf16: 32, 64 or 128 */
    int32_t d_ff;       /* FFN hidden width of the dense model */
    int32_t n_layers;
    int32_t P;          /* number of modality-presence patterns in use */
    int32_t dtype;      /* SF_F32 | SF_BF16 (libsentryfuse.so) | SF_F16 (libsentryfuse_f16.so) */
    int32_t act;        /* SF_RELU | SF_GELU_ERF */
    int32_t c_factor;   /* c of U = c*ceil(ln L) (Sec. 4.4); 5 if <= 0 */
    int32_t U_override; /* < 0: use c_factor; >= 0: this many active queries (clipped to L) */
    uint32_t flags;     /* SF_FLAG_* */
    float ln_eps;       /* 1e-5 if <= 0 */
    int32_t ffn_pad;    /* kept FFN width is padded with zero channels to a multiple of
                           this; must be a multiple of 64; 64 if <= 0 */
    int32_t n_sample;   /* entries per sample of the key sample `sample_idx` of the sparsity
                           score (0 = the score uses every allowed key); at most 4096 */
} sf_desc;

const char *sf_last_error(void);

/* U = min(L, c*ceil(ln L)) of Sec. 4.4 (natural log: the worked example
 * T=128, c=5 gives 25), or the override.  Negative status on a bad desc. */
int32_t sf_num_active(const sf_desc *desc);

/* round_up(k_ffn, ffn_pad) */
int32_t sf_ffn_padded(const sf_desc *desc, int32_t k_ffn);

/* ------------------------------------------------------------------------
 * presence_to_key_valid -- Sec. 4.2 (the presence mask m in {0,1}^M of a
 * sample) and Sec. 4.4 (attention over the concatenated per-modality token
 * sequence): which positions sample b may use as attention keys,
 *   key_valid[b,j] = 1 if tok_modality[j] < 0 (a token of no modality, e.g. a
 *                      fusion token) or presence[b, tok_modality[j]] != 0,
 *                    0 otherwise.
 *   presence     [B,M] u8 device;  tok_modality [L] int32 device, values < M
 *                (an id >= M counts as absent);  key_valid [B,L] u8 device out.
 * The result is the key_valid argument of sf_sparse_gqa_forward and the
 * sf_encoder_forward family (a sample needs at least one allowed position;
 * the host cannot check device data).  0 <= M <= 64.  No workspace.
 */
int32_t sf_presence_to_key_valid(const uint8_t *presence, const int32_t *tok_modality, int32_t B,
                                 int32_t M, int32_t L, uint8_t *key_valid, void *stream);

/* ------------------------------------------------------------------------
 * gate_scores_to_masks -- Sec. 4.5, "Head pruning with GQA consistency" and
 * "FFN pruning".  For every (layer l, pattern p) the k_head_host[l] heads and
 * k_ffn_host[l] channels with the highest gate score g (Eq. (1)) are kept;
 * ties go to the lower index.  K/V groups kept = { floor(h/(Hq/Hk)) : h kept }.
 *
 *   g_head [n_layers,P,Hq] fp32, g_ffn [n_layers,P,d_ff] fp32 (no NaNs)
 *   k_head_host, k_ffn_host [n_layers] int32 HOST arrays, 1 <= k <= n
 * outputs (all required):
 *   head_mask [n_layers,P,Hq] u8, ffn_mask [n_layers,P,d_ff] u8   1 = kept
 *   head_idx  [n_layers,P,Hq]   kept heads ascending, then -1
 *   ffn_idx   [n_layers,P,d_ff] kept channels ascending, then -1
 *   group_idx [n_layers,P,Hk]   kept groups ascending, then -1
 *   n_groups  [n_layers,P]
 *   head_group[n_layers,P,Hq]   for the i-th kept head: rank of its group in
 *                               group_idx; then -1
 * Limits: Hq <= 64, d_ff <= 16384.  No workspace.
 * Keep counts, not a threshold, are the argument: one integer per layer makes
 * the compacted shapes the same for every presence pattern of a batch, which
 * the batched forward needs.  Sec. 4.5's global threshold for a pruning budget
 * is sf_budget_search below: it returns tau together with the per-layer counts
 * for which this call keeps exactly the units scoring >= tau.
 */
int32_t sf_gate_scores_to_masks(const sf_desc *desc, const float *g_head, const float *g_ffn,
                                const int32_t *k_head_host, const int32_t *k_ffn_host,
                                uint8_t *head_mask, uint8_t *ffn_mask, int32_t *head_idx,
                                int32_t *ffn_idx, int32_t *group_idx, int32_t *n_groups,
                                int32_t *head_group, void *stream);

/* Dense parameters of one encoder layer, unit-major: every head dimension and
 * every FFN channel is one contiguous row of d_model elements.
 *   Wq [Hq*dh, d]   column blocks of the paper's W_Q in R^{d x Hq*dh}
 *   Wk, Wv [Hk*dh, d]
 *   Wo [Hq*dh, d]   row blocks of the output projection
 *   W1 [d_ff, d]    columns of the paper's W_1 in R^{d x d_ff}
 *   W2 [d_ff, d]    rows of the paper's W_2 in R^{d_ff x d}
 *   bq [Hq*dh], bk, bv [Hk*dh], bo [d], b1 [d_ff], b2 [d]; any bias may be NULL
 *   ln1_g, ln1_b, ln2_g, ln2_b [d] (required by sf_encoder_forward) */
typedef struct sf_dense_layer {
    const void *Wq, *bq, *Wk, *bk, *Wv, *bv, *Wo, *bo;
    const void *W1, *b1, *W2, *b2;
    const void *ln1_g, *ln1_b, *ln2_g, *ln2_b;
} sf_dense_layer;

/* Compacted parameters of one layer for all P patterns (leading dimension P).
 * With Hq' = k_head, F' = k_ffn, Fp = sf_ffn_padded(F'), Nqkv = (Hq'+2*Hk)*dh:
 *   Wqkv [P, Nqkv, d]  rows: the Hq' kept query heads (ascending), then Hk
 *                      K-group slots, then Hk V-group slots; slot r holds kept
 *                      group r for r < n_groups and zeros otherwise
 *   bqkv [P, Nqkv]     (NULL iff bq, bk and bv are all NULL)
 *   WoT  [P, d, Hq'*dh] WoT[n, i*dh+e] = Wo[head_idx[i]*dh+e, n]
 *   W1   [P, Fp, d]    kept channels ascending, zero rows above F'
 *   b1   [P, Fp]       (NULL iff dense b1 is NULL)
 *   W2T  [P, d, Fp]    W2T[n, j] = W2[ffn_idx[j], n], zeros above F'
 * bo, b2 and the LayerNorm vectors are not pruned: they point at the dense
 * arrays.  head_group [P,Hq] and n_groups [P] are this layer's slices of the
 * sf_gate_scores_to_masks outputs. */
typedef struct sf_compact_layer {
    int32_t k_head;            /* Hq' */
    int32_t k_ffn;             /* F'  */
    void *Wqkv, *bqkv, *WoT, *W1, *b1, *W2T;
    const void *bo, *b2, *ln1_g, *ln1_b, *ln2_g, *ln2_b;
    const int32_t *head_group;
    const int32_t *n_groups;
} sf_compact_layer;

/* ------------------------------------------------------------------------
 * compact_heads_channels -- Sec. 4.5: keep the column blocks of W_Q for
 * H_keep, the blocks of W_K / W_V of the referenced groups, the matching row
 * blocks of the output projection, and W1' = W1[:, N_keep], W2' = W2[N_keep, :].
 * Pure data movement (bit-exact).  `layer` selects the slices of the index
 * tensors; dense_host / compact_host are HOST structs of DEVICE pointers.
 * compact_host->k_head / k_ffn must equal the counts used for the masks; the
 * caller has allocated Wqkv, bqkv, WoT, W1, b1, W2T at the sizes above and
 * copied bo, b2, ln*, head_group, n_groups pointers itself.  No workspace.
 */
int32_t sf_compact_heads_channels(const sf_desc *desc, int32_t layer,
                                  const sf_dense_layer *dense_host,
                                  const int32_t *head_idx, const int32_t *group_idx,
                                  const int32_t *n_groups, const int32_t *ffn_idx,
                                  const sf_compact_layer *compact_host, void *stream);

/* ------------------------------------------------------------------------
 * FP8 post-training quantisation of the weights (the paper's "compatibility
 * with quantization" experiment applies FP8 PTQ on top of the pruned model;
 * it names neither format nor scaling).  Here the six weight matrices of a
 * layer are stored as OCP E4M3 bytes (1-4-3, bias 7, finite only, 0x7F / 0xFF
 * = NaN, largest value 448) in the shapes of sf_dense_layer, with one fp32
 * scale per matrix; w = decode(byte) * scale.  Biases and LayerNorm vectors
 * stay in the model dtype.  sf_compact_heads_channels_fp8 is
 * sf_compact_heads_channels reading this storage: it gathers the kept blocks
 * and dequantises in the same pass (one rounding, from the exact product, to
 * the model dtype), so the forward path is unchanged and dense 16-bit weights
 * never exist.  d_model must be a multiple of 4, the matrices 4-byte aligned.
 */
typedef struct sf_dense_layer_fp8 {
    const void *Wq, *Wk, *Wv, *Wo, *W1, *W2;          /* uint8 E4M3 */
    float sq, sk, sv, so, s1, s2;                     /* per-matrix scales */
    const void *bq, *bk, *bv, *bo, *b1, *b2;          /* model dtype, any may be NULL */
    const void *ln1_g, *ln1_b, *ln2_g, *ln2_b;
} sf_dense_layer_fp8;
int32_t sf_compact_heads_channels_fp8(const sf_desc *desc, int32_t layer,
                                      const sf_dense_layer_fp8 *dense_host,
                                      const int32_t *head_idx, const int32_t *group_idx,
                                      const int32_t *n_groups, const int32_t *ffn_idx,
                                      const sf_compact_layer *compact_host, void *stream);

/* FP16 post-training quantisation of the weights (the FP16 points of the same
 * experiment): sf_compact_heads_channels reading the six weight matrices of
 * `dense_host` as IEEE binary16 (2 bytes per element, no scale; biases and
 * LayerNorm vectors in the model dtype).  The stored value is rounded once to
 * the model dtype in the gather: exact for an fp32 model (every binary16 value
 * is an fp32 value), one rounding to bf16 otherwise.  bf16 stays the 16-bit
 * compute type; there is no fp16 arithmetic.  d_model a multiple of 4, the
 * matrices 8-byte aligned. */
int32_t sf_compact_heads_channels_f16(const sf_desc *desc, int32_t layer,
                                      const sf_dense_layer *dense_host,
                                      const int32_t *head_idx, const int32_t *group_idx,
                                      const int32_t *n_groups, const int32_t *ffn_idx,
                                      const sf_compact_layer *compact_host, void *stream);

/* ------------------------------------------------------------------------
 * FP8 arithmetic for the pruned FFN (same experiment; the paper does not say
 * how its FP8 models compute).  Here both operands of the two FFN contractions
 * are E4M3 codes with one fp32 scale per tensor (W8A8, scales fixed offline),
 * products are exact, sums are fp32 on the matrix cores:
 *     xq = Q(LN2(x), sx)                  (LayerNorm in fp32, quantised from fp32)
 *     z  = (sum_k dec(xq) dec(W1q)) * (sx*s1) + b1        (fp32)
 *     hq = Q(act(z), sh)
 *     y  = (sum_f dec(hq) dec(W2q)) * (sh*s2) + b2 (+ x)  -> bf16
 * Q(t, s) = E4M3(t * (1/s)) with the reciprocal and the product in fp32, round
 * to nearest (ties to the even code), saturating at +-448.  NaN gives 0x7F in
 * sf_quantize_fp8 and after LayerNorm; the code of a NaN hidden value is
 * unspecified.
 *
 * sf_ffn_fp8: compact FFN weights of one layer for all P patterns.
 *   Fp8 = sf_ffn_fp8_padded(k_ffn): k_ffn rounded up to a multiple of 128
 *   W1q  [P, Fp8, d]  codes of the kept channels (ascending), zero above F'
 *   b1   [P, Fp8]     bf16, zeros above F' (NULL iff the dense b1 is NULL)
 *   W2Tq [P, d, Fp8]  W2Tq[n, j] = W2q[ffn_idx[j], n], zero above F'
 *   b2, ln2_g, ln2_b [d] bf16: the dense arrays;  s1, s2: the dense scales
 *   sx, sh: scales of the block's input (after LayerNorm when pre_ln) and of
 *           the hidden activations
 * sf_compact_ffn_fp8 fills W1q, b1, W2Tq from a dense FP8 layer (uses W1, W2,
 * b1 of `dense_host` and this layer's slice of ffn_idx; pure byte movement,
 * bit-exact); the caller sets k_ffn and the other fields.
 * sf_quantize_fp8: codes[i] = Q(x[i], scale), x of dtype SF_F32 or SF_BF16
 * (16-byte aligned), codes 8-byte aligned.
 * sf_pruned_ffn_fp8_forward: X, Y [B*L, d] bf16 (desc->dtype must be SF_BF16),
 * pattern_id as in sf_pruned_ffn_forward.  xq_out [B*L, d], hq_out [B*L, Fp8]
 * (16-byte aligned) receive the codes when not NULL.  Limits: d a multiple of
 * 128 (256 <= d, d <= 4096 with pre_ln), L >= 192, k_ffn > 128; anything else
 * returns SF_ERR_SHAPE / SF_ERR_UNSUPPORTED before a kernel is launched.
 */
typedef struct sf_ffn_fp8 {
    int32_t k_ffn;             /* F' */
    int32_t reserved;
    void *W1q, *b1, *W2Tq;
    const void *b2, *ln2_g, *ln2_b;
    float s1, s2, sx, sh;
} sf_ffn_fp8;
int32_t sf_ffn_fp8_padded(int32_t k_ffn);
int32_t sf_compact_ffn_fp8(const sf_desc *desc, int32_t layer, const sf_dense_layer_fp8 *dense_host,
                           const int32_t *ffn_idx, const sf_ffn_fp8 *ffn_host, void *stream);
int32_t sf_quantize_fp8(const void *x, int32_t dtype, int64_t n, float scale, uint8_t *codes,
                        void *stream);
size_t sf_pruned_ffn_fp8_workspace_bytes(const sf_desc *desc, int32_t k_ffn);
int32_t sf_pruned_ffn_fp8_forward(const sf_desc *desc, const sf_ffn_fp8 *ffn_host, const void *X,
                                  const int32_t *pattern_id, int32_t pre_ln, int32_t add_residual,
                                  void *Y, uint8_t *xq_out, uint8_t *hq_out, void *workspace,
                                  size_t workspace_bytes, void *stream);

/* sf_encoder_forward with the FFN of every layer in FP8 arithmetic (the
 * attention block is unchanged).  ffn_host [n_layers]: HOST array, entry l
 * built from layer l's FFN with k_ffn equal to layers_host[l].k_ffn; sx is the
 * scale of LN2 of the residual stream.  The limits of
 * sf_pruned_ffn_fp8_forward apply to every layer; the workspace is that of
 * sf_encoder_forward.  xq_out [n_layers, B*L, d] and hq_out (layer l's codes,
 * a [B*L, Fp8_l] array, at hq_out + l*B*L*max_l Fp8_l) receive the codes when
 * not NULL (16-byte aligned). */
int32_t sf_encoder_forward_fp8ffn(const sf_desc *desc, const sf_compact_layer *layers_host,
                                  const sf_ffn_fp8 *ffn_host, const void *X,
                                  const int32_t *pattern_id, const uint8_t *key_valid,
                                  const int32_t *sample_idx, const void *final_g,
                                  const void *final_b, const int32_t *forced_sel, void *Y,
                                  int32_t *sel_out, float *score_out, uint8_t *xq_out,
                                  uint8_t *hq_out, void *workspace, size_t workspace_bytes,
                                  void *stream);

/*
 * The attention projections in FP8 arithmetic (the other contractions of the
 * FP8 models of the quantisation experiment; this build's reading, the paper
 * does not say which contractions run in FP8).  Per layer:
 *     aq      = E4M3(LN1(x) / sx1)                        LN1 in fp32
 *     q, k, v = (aq . Wqkv8^T) * (sx1 * s_qkv) + bqkv     fp32 accumulation, stored as bf16
 *     oq      = E4M3(attention output / sa)
 *     x1      = x + (oq . WoT8^T) * (sa * so) + bo        fp32
 * SentryAttend runs unchanged on q, k, v.  Wq, Wk, Wv carry ONE scale (they are
 * one GEMM operand).  sf_compact_proj_fp8 gathers the kept rows of the dense
 * codes (sf_dense_layer_fp8 with sq == sk == sv) into
 *     Wqkv8 [P, (k_head + 2*Hk)*dh, d]      kept Q heads, K rows, V rows of the
 *                                           used groups (zero rows for unused slots)
 *     WoT8  [P, d, Kp]                      Kp = sf_proj_fp8_padded(k_head, dh) =
 *                                           k_head*dh rounded up to a multiple of 128
 *                                           (zero columns: the FP8 GEMM contracts over
 *                                           multiples of 128)
 * both DEVICE buffers of the caller, uint8, 16-byte aligned; biases bqkv, bo
 * and the LayerNorm vectors are those of the sf_compact_layer of the layer.
 * s_qkv, so must equal the dense scales; sx1, sa are chosen by the caller
 * (static activation scales).  Limits: bf16 model, d a multiple of 128 in
 * [256, 4096], (k_head + 2*Hk)*dh >= 192, L >= 192; anything else returns
 * SF_ERR_SHAPE / SF_ERR_UNSUPPORTED before a kernel is launched.
 */
typedef struct sf_proj_fp8 {
    int32_t k_head;            /* Hq' */
    int32_t reserved;
    void *Wqkv8, *WoT8;
    float s_qkv, so, sx1, sa;
} sf_proj_fp8;
int32_t sf_proj_fp8_padded(int32_t k_head, int32_t d_head);
int32_t sf_compact_proj_fp8(const sf_desc *desc, int32_t layer, const sf_dense_layer_fp8 *dense_host,
                            const int32_t *head_idx, const int32_t *group_idx,
                            const int32_t *n_groups, const sf_proj_fp8 *proj_host, void *stream);

/* sf_encoder_forward with the attention projections (proj_host != NULL) and /
 * or the FFNs (ffn_host != NULL) of every layer in FP8 arithmetic; at least one
 * of the two is given.  proj_host [n_layers]: HOST array, k_head equal to
 * layers_host[l].k_head.  The workspace is sf_encoder_fp8_workspace_bytes
 * (larger than sf_encoder_workspace_bytes: token-major V and the codes of the
 * attention output).  aq_out [n_layers, B*L, d] and oq_out (layer l's codes, a
 * [B*L, Kp_l] array over the KEPT heads in rank order followed by zero
 * padding, at oq_out + l*B*L*max_l Kp_l) receive the codes when not NULL (16-byte
 * aligned); xq_out, hq_out as in sf_encoder_forward_fp8ffn. */
size_t sf_encoder_fp8_workspace_bytes(const sf_desc *desc, const sf_compact_layer *layers_host);
int32_t sf_encoder_forward_fp8(const sf_desc *desc, const sf_compact_layer *layers_host,
                               const sf_ffn_fp8 *ffn_host, const sf_proj_fp8 *proj_host,
                               const void *X, const int32_t *pattern_id, const uint8_t *key_valid,
                               const int32_t *sample_idx, const void *final_g, const void *final_b,
                               const int32_t *forced_sel, void *Y, int32_t *sel_out,
                               float *score_out, uint8_t *xq_out, uint8_t *hq_out, uint8_t *aq_out,
                               uint8_t *oq_out, void *workspace, size_t workspace_bytes,
                               void *stream);

/* Element strides of a [B, heads, L, dh] tensor whose last dimension is
 * contiguous (for V with v_transposed: a [B, groups, dh, L] tensor whose L
 * dimension is contiguous and `l` is the stride between dh rows). */
typedef struct sf_strides { int64_t b, h, l; } sf_strides;

/* ------------------------------------------------------------------------
 * sparse_gqa_forward -- SentryAttend, Sec. 4.4.  For every sample b and head
 * h (using K/V group head_group[h]):
 *   1. sparsity score of query i over the allowed keys A_b:
 *        M_i = max_j s_ij - mean_j s_ij,  s_ij = q_i.k_j / sqrt(dh)
 *      (max-minus-mean is this library's reading of the measure the paper
 *      cites; disallowed queries score -inf);
 *   2. the U queries with the highest M_i are active (ties: lower index; at
 *      most |A_b| queries);
 *   3. active rows, Eq. (6): o_i = softmax_j(s_ij) V_g over A_b;
 *   4. every other row is the context vector mean_{j in A_b} v_j of its group.
 * uses desc->B, L, dh, dtype and the U of sf_num_active(desc).
 *   nH, nG        heads in Q, groups in K/V of THIS call (e.g. Hq', Hk)
 *   Q, K, V       strided tensors, see sf_strides; bf16: strides multiples of 8
 *   v_transposed  0: V is [B,nG,L,dh]; 1: V is [B,nG,dh,L]
 *   head_group    [n_maps, nH] int32, head -> group slot (0..nG-1)
 *   pattern_id    [B] int32 row of head_group used by sample b, or NULL (row 0)
 *   key_valid     [B,L] u8, 1 = key/query allowed, or NULL (all allowed);
 *                 a sample with no allowed key gives undefined rows for that
 *                 sample (callers validate presence on the host)
 *   sample_idx    [B,desc->n_sample] int32 or NULL: key sample of step 1 (the
 *                 sampled-key estimate of the measure, which is what makes the
 *                 score O(L log L) when n_sample ~ c*ceil(ln L)): max and mean
 *                 of step 1 run over the allowed keys listed here only.  A set:
 *                 duplicates and entries outside [0,L) are ignored; if no listed
 *                 key is allowed, every allowed query scores 0.  Steps 3 and 4
 *                 always use every allowed key.  Ignored when desc->n_sample = 0.
 *   forced_sel    [B,nH,U] int32 or NULL: active queries given by the caller
 *                 (ascending, distinct, -1 padded at the end); skips 1-2
 *   O             [B,L,nH*dh], row stride ldo elements
 *   sel_out       [B,nH,U] int32 or NULL: the active queries, ascending, -1 padded
 *   score_out     [B,nH,L] fp32 or NULL: M_i (not written when U >= L or forced_sel)
 */
size_t sf_sparse_gqa_workspace_bytes(const sf_desc *desc, int32_t nH, int32_t nG);
int32_t sf_sparse_gqa_forward(const sf_desc *desc, int32_t nH, int32_t nG,
                              const void *Q, sf_strides sq, const void *K, sf_strides sk,
                              const void *V, sf_strides sv, int32_t v_transposed,
                              const int32_t *head_group, const int32_t *pattern_id,
                              const uint8_t *key_valid, const int32_t *sample_idx,
                              const int32_t *forced_sel,
                              void *O, int64_t ldo, int32_t *sel_out, float *score_out,
                              void *workspace, size_t workspace_bytes, void *stream);

/* sf_sparse_gqa_forward for callers that cannot allocate or hold a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that
 * forbid device allocation.  Same arguments, same kernels and same results as
 * sf_sparse_gqa_forward, but the scratch memory (transposed V, statistics,
 * scores, active lists, key-split partials) is a buffer of
 * SF_STATIC_SCRATCH_BYTES built into the library's device image, one copy per
 * GPU, held until the process ends.  The call allocates and frees nothing.
 * A problem whose sf_sparse_gqa_workspace_bytes() exceeds the buffer is refused
 * with SF_ERR_WORKSPACE before anything is enqueued (the message names both
 * sizes).  All calls on one GPU share the buffer, so two calls that overlap in
 * time on one GPU (different streams or threads) race: serialise them, or use
 * sf_sparse_gqa_forward with a workspace per stream.  Nothing in the buffer
 * needs clearing between calls.  sf_sparse_gqa_static_capacity() returns
 * SF_STATIC_SCRATCH_BYTES. */
#define SF_STATIC_SCRATCH_BYTES (16u << 20)
size_t sf_sparse_gqa_static_capacity(void);
int32_t sf_sparse_gqa_forward_static(const sf_desc *desc, int32_t nH, int32_t nG,
                                     const void *Q, sf_strides sq, const void *K, sf_strides sk,
                                     const void *V, sf_strides sv, int32_t v_transposed,
                                     const int32_t *head_group, const int32_t *pattern_id,
                                     const uint8_t *key_valid, const int32_t *sample_idx,
                                     const int32_t *forced_sel,
                                     void *O, int64_t ldo, int32_t *sel_out, float *score_out,
                                     void *stream);

/* ------------------------------------------------------------------------
 * pruned_ffn_forward -- Sec. 4.5: Y = [X +] act(X' W1'^T + b1') W2' + b2 with
 * X' = LayerNorm(X) when pre_ln != 0, else X.  X, Y [B*L, d]; sample b uses
 * pattern pattern_id[b] (NULL: 0).  Uses k_ffn, W1, b1, W2T, b2, ln2_g, ln2_b
 * of `layer_host` (a HOST struct of device pointers).  Y may not alias X.
 */
size_t sf_pruned_ffn_workspace_bytes(const sf_desc *desc, int32_t k_ffn);
int32_t sf_pruned_ffn_forward(const sf_desc *desc, const sf_compact_layer *layer_host,
                              const void *X, const int32_t *pattern_id, int32_t pre_ln,
                              int32_t add_residual, void *Y, void *workspace,
                              size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * encoder_forward -- the pruned encoder: for l = 0..n_layers-1
 *     x <- x + OutProj( SentryAttend( QKV( LN1(x) ) ) )
 *     x <- x + FFN( LN2(x) )                       (pre-norm)
 * and a final LayerNorm when SF_FLAG_FINAL_LN is set.
 *   X [B,L,d] in, Y [B,L,d] out (Y may not alias X)
 *   layers_host [n_layers]  HOST array of sf_compact_layer
 *   pattern_id  [B] or NULL;  key_valid [B,L] or NULL
 *   sample_idx  [B,desc->n_sample] or NULL: key sample of the sparsity score, the
 *               same in every layer (see sf_sparse_gqa_forward)
 *   final_g, final_b [d]    (required with SF_FLAG_FINAL_LN)
 *   forced_sel  [n_layers,B,Hq'max,U] or NULL  (Hq'max = max k_head over layers)
 *   sel_out     [n_layers,B,Hq'max,U] or NULL  active queries per layer
 *   score_out   [n_layers,B,Hq'max,L] fp32 or NULL
 */
size_t sf_encoder_workspace_bytes(const sf_desc *desc, const sf_compact_layer *layers_host);
/* How sf_encoder_forward projects the attention output of a layer with k_head
 * kept heads (Sec. 4.4: the rows that are not selected all take their group's
 * context vector).  0: every row goes through the output projection.  n > 0:
 * at most a quarter of a sample's rows can be active in some head; only those (at
 * most n = k_head*U rounded up to 128 per sample) are projected, every other
 * row of a sample receives the projection of its context vectors, computed
 * once.  Same results up to the summation order of that one vector.  (A
 * reporting aid: the count of arithmetic actually done differs.) */
int32_t sf_active_projection_rows(const sf_desc *desc, int32_t k_head);
int32_t sf_encoder_forward(const sf_desc *desc, const sf_compact_layer *layers_host,
                           const void *X, const int32_t *pattern_id, const uint8_t *key_valid,
                           const int32_t *sample_idx, const void *final_g, const void *final_b,
                           const int32_t *forced_sel, void *Y, int32_t *sel_out,
                           float *score_out, void *workspace, size_t workspace_bytes,
                           void *stream);

/* ------------------------------------------------------------------------
 * Token compaction -- Sec. 4.2 / 4.4: the encoder runs over the concatenated
 * tokens of the modalities that are present.  sf_encoder_forward keeps the
 * tokens of absent modalities in place and masks them as keys (key_valid);
 * here they are dropped: every sample keeps its valid tokens, in order, at the
 * front of a shorter padded sequence of Lc positions, and its number of active
 * queries follows its own length T_b: u_active[b] = min(c*ceil(ln T_b), T_b)
 * (Sec. 4.4 with T = T_b; c = desc->c_factor).
 *
 * sf_token_compact (desc: B, L, d_model, dtype, c_factor of the full sequence):
 *   X           [B,L,d]  in;  token_valid [B,L] (non-zero = token exists)
 *   Lc          positions per compacted sample, 1 <= Lc <= L; the caller knows
 *               the presence patterns and passes at least the largest T_b
 *   Xc          [B,Lc,d]  valid tokens first, then zero rows
 *   valid_c     [B,Lc]    1 for positions < T_b
 *   row_index   [B,Lc]    token at each position, -1 behind T_b
 *   slot_of     [B,L]     position of each token, -1 for dropped tokens
 *   len         [B]       T_b (not clamped: a value above Lc says that tokens
 *                         were lost and the outputs must not be used)
 *   u_active    [B]
 * sf_encoder_forward_ragged is sf_encoder_forward on the compacted batch (a
 * descriptor with L = Lc whose U is at least the largest u_active[b], e.g.
 * U_override = c*ceil(ln Lc); U < Lc is required) with key_valid = valid_c and
 * u_active: sample b selects min(u_active[b], U) queries per head; sel_out rows
 * are padded with -1.  No forced selection.  The same workspace size applies.
 * sf_token_scatter writes Y[b,i,:] = Yc[b,slot_of[b,i],:] and zero rows for
 * dropped tokens (desc as for sf_token_compact).
 * All index outputs are bit-exact; no workspace.
 */
int32_t sf_token_compact(const sf_desc *desc, const void *X, const uint8_t *token_valid, int32_t Lc,
                         void *Xc, uint8_t *valid_c, int32_t *row_index, int32_t *slot_of,
                         int32_t *len, int32_t *u_active, void *stream);
int32_t sf_token_scatter(const sf_desc *desc, const void *Yc, const int32_t *slot_of, int32_t Lc,
                         void *Y, void *stream);
int32_t sf_encoder_forward_ragged(const sf_desc *desc, const sf_compact_layer *layers_host,
                                  const void *X, const int32_t *pattern_id,
                                  const uint8_t *key_valid, const int32_t *u_active,
                                  const int32_t *sample_idx, const void *final_g,
                                  const void *final_b, void *Y, int32_t *sel_out,
                                  float *score_out, void *workspace, size_t workspace_bytes,
                                  void *stream);

/*
 * Token compaction without padding (Sec. 4.2 / 4.4, as above; the layout is this
 * library's).  The valid tokens of all samples lie back to back in one
 * [Tc, d] buffer: samples ordered by presence pattern, then by sample number;
 * every pattern's run of rows starts on a multiple of 256, so a 256-row block
 * holds rows of one pattern (it may straddle samples).  LayerNorm and the four
 * GEMMs of a layer then run over the blocks in use only; the attention steps
 * see sample b as the rows row0[b] .. row0[b] + len[b] - 1 with at most L
 * positions, and its number of active queries is u_active[b] (formula above).
 * Behind the last run lie align(L, 256) rows of slack (zero input rows) that
 * the attention kernels may read but never use.
 *
 * sf_token_pack_plan is a host struct of device pointers, all written by
 * sf_token_pack (the caller allocates them and sets Tc):
 *   Tc           rows of the packed buffers, a positive multiple of 256;
 *                sf_token_pack_rows_max(desc) is enough for every input
 *                (desc->P = number of presence patterns); a caller that knows
 *                the presence counts can pass less
 *   len          [B]      T_b, the valid tokens of sample b
 *   u_active     [B]
 *   row0         [B]      first packed row of sample b
 *   ext          [B]      rows of the attention output that sample b answers
 *                         for: len[b], plus - for the last sample of a run -
 *                         the padding up to the next run (and the slack)
 *   valid_c      [B,L]    1 for positions < T_b
 *   blk_pattern  [Tc/256] presence pattern of each 256-row block, -1: unused
 *   src_row      [Tc]     source row b*L + i of each packed row, -1: padding
 *   dst_row      [B,L]    packed row of each token, -1 for dropped tokens
 *   n_rows       [2]      [0] rows in use (runs + slack), [1] rows needed.
 *                         n_rows[1] > Tc: the rows did not fit; the plan is
 *                         then the empty one (no sample has rows, Xp is zero,
 *                         the encoder does nothing) and the caller comes back
 *                         with Tc >= n_rows[1].  n_rows[1] = -1: a pattern
 *                         number outside [0, P); the empty plan as well.
 * sf_token_pack: X [B,L,d], token_valid [B,L], pattern_id [B] (NULL with P = 1)
 * in; the plan and Xp [Tc,d] (zero rows where src_row < 0) out.
 * sf_encoder_forward_packed is sf_encoder_forward over the packed rows (desc
 * as for the padded batch: B samples of at most L tokens, U >= every
 * u_active[b] and U < L); Xp, Yp [Tc,d]; sel_out [n_layers,B,kmax_head,U] holds
 * positions inside the sample, rows padded with -1; score_out
 * [n_layers,B,kmax_head,L].  Rows of Yp that are padding hold unspecified finite
 * or non-finite values and are never read by sf_token_unpack.  Projections and
 * FFN in FP8 arithmetic are not offered on packed rows.
 * sf_token_unpack writes Y[b,i,:] = Yp[dst_row[b,i],:], zero rows for dropped
 * tokens.  All index outputs are bit-exact.
 * Errors: SF_ERR_INVALID_ARG (NULL, Tc not a multiple of 256, aliasing),
 * SF_ERR_SHAPE (sf_token_pack: more than 4096 presence patterns), SF_ERR_WORKSPACE (sf_encoder_packed_workspace_bytes), as for
 * sf_encoder_forward.
 */
typedef struct sf_token_pack_plan {
    int32_t Tc;
    int32_t *len, *u_active, *row0, *ext;
    uint8_t *valid_c;
    int32_t *blk_pattern, *src_row, *dst_row, *n_rows;
} sf_token_pack_plan;
int32_t sf_token_pack_rows_max(const sf_desc *desc);
int32_t sf_token_pack(const sf_desc *desc, const void *X, const uint8_t *token_valid,
                      const int32_t *pattern_id, const sf_token_pack_plan *plan, void *Xp,
                      void *stream);
int32_t sf_token_unpack(const sf_desc *desc, const void *Yp, const sf_token_pack_plan *plan,
                        void *Y, void *stream);
size_t sf_encoder_packed_workspace_bytes(const sf_desc *desc, const sf_compact_layer *layers_host,
                                         int32_t Tc);
int32_t sf_encoder_forward_packed(const sf_desc *desc, const sf_compact_layer *layers_host,
                                  const void *Xp, const sf_token_pack_plan *plan,
                                  const int32_t *pattern_id, const int32_t *sample_idx,
                                  const void *final_g, const void *final_b, void *Yp,
                                  int32_t *sel_out, float *score_out, void *workspace,
                                  size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * Sparse-MoE FFN with pruned experts -- Sec. 4.5 "Sparse-MoE FFN pruning":
 * the number of experts E and the Top-k routing stay fixed; expert e keeps
 * its own channel set, W1_e' = W1_e[:, N_keep_e], W2_e' = W2_e[N_keep_e, :].
 * The paper fixes neither the router nor the combination; this library uses
 *   xn = LayerNorm(x) (pre_ln) or x;   logit_e = xn . Wr_e + br_e (fp32);
 *   the top_k experts with the highest logit (ties: lower index);
 *   p_e = softmax over the chosen logits;
 *   y = [x +] sum_{chosen e} p_e * ( act(xn W1_e'^T + b1_e') W2_e' + b2_e ).
 *
 * Dense expert parameters (device pointers in a HOST struct), unit-major:
 *   Wr [E,d], br [E] (NULL ok), W1 [E,F,d], b1 [E,F] (NULL ok),
 *   W2 [E,F,d], b2 [E,d] (NULL ok), ln_g, ln_b [d]      (F = desc->d_ff)
 * Compact form for all P patterns, Fp = sf_ffn_padded(k_ffn_max), k_ffn_max =
 * the largest per-expert keep count (narrower experts are zero padded):
 *   W1 [P,E,Fp,d], b1 [P,E,Fp], W2T [P,E,d,Fp], b2x [P,E,d] (b2 repeated per pattern)
 * sf_compact_moe_experts gathers them (bit-exact data movement):
 *   ffn_idx [E,P,F] kept channels of expert e for pattern p, ascending (e.g. the
 *   ffn_idx output of sf_gate_scores_to_masks run with n_layers = E on the
 *   expert-internal gate scores), k_ffn_host [E] HOST keep counts.
 * sf_moe_ffn_forward: X, Y [B*L, d] (Y may not alias X); sample b uses pattern
 *   pattern_id[b] (NULL: 0);
 *   forced_route [B*L, top_k] int32 or NULL: experts given by the caller
 *     (distinct, 0..E-1; values outside are clamped, an expert listed twice
 *     counts once, in its last slot, the other slot gets weight 0) instead of
 *     the Top-k choice; the weights are still the softmax of this call's
 *     logits of those experts;
 *   route_out [B*L, top_k] int32, weight_out [B*L, top_k] fp32,
 *   logit_out [B*L, E] fp32: any may be NULL.  route_out lists the chosen
 *   experts by descending logit.
 * bf16 rounding points: xn, each expert's hidden activations, Y.
 */
typedef struct sf_moe_dense {
    const void *Wr, *br, *W1, *b1, *W2, *b2, *ln_g, *ln_b;
} sf_moe_dense;
typedef struct sf_moe_compact {
    int32_t n_experts;         /* E <= 64 */
    int32_t top_k;             /* <= min(8, E) */
    int32_t k_ffn_max;         /* max over experts of the kept channel count */
    int32_t reserved;
    const void *Wr, *br;
    void *W1, *b1, *W2T, *b2x;
    const void *ln_g, *ln_b;
    int32_t *k_ffn;            /* device [E]: keep count of every expert, written by sf_compact_moe_experts */
} sf_moe_compact;
int32_t sf_compact_moe_experts(const sf_desc *desc, const sf_moe_dense *dense_host,
                               const int32_t *ffn_idx, const int32_t *k_ffn_host,
                               const sf_moe_compact *compact_host, void *stream);
size_t sf_moe_ffn_workspace_bytes(const sf_desc *desc, const sf_moe_compact *moe_host);
int32_t sf_moe_ffn_forward(const sf_desc *desc, const sf_moe_compact *moe_host, const void *X,
                           const int32_t *pattern_id, int32_t pre_ln, int32_t add_residual,
                           const int32_t *forced_route, void *Y, int32_t *route_out,
                           float *weight_out, float *logit_out, void *workspace,
                           size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * SentryGate on the device (plan construction; fp32 whatever the model dtype).
 *
 * sf_gate_eval - the importance scores of Eq. (1) for every layer and every
 * presence pattern in use:
 *   g_i(m) = sigmoid( zeta_i + gamma * f_i(m) ),  f = two-layer perceptron.
 * The paper gives neither the width nor the nonlinearity of f; here the first
 * layer is shared by the units of a layer, h = nonlin(Wa m + ba) with `hidden`
 * units (nonlin: ReLU or tanh), and unit i has its own output row,
 * f_i = Wb[i,:] . h + cb[i].  The units of a layer are its Hq heads followed
 * by its F channels (n_units = Hq + F).
 *   parameters (device pointers in a HOST struct, fp32):
 *     Wa [nl,hidden,M], ba [nl,hidden] (NULL ok), Wb [nl,n_units,hidden]
 *     (16-byte aligned), cb [nl,n_units] (NULL ok), zeta [nl,n_units], gamma [nl]
 *   pattern_bits [P] int32 device: bit j set = modality j present
 *   g_head [nl,P,Hq], g_ffn [nl,P,F] fp32 out: the layouts
 *   sf_gate_scores_to_masks takes.
 *
 * sf_budget_search - the global threshold of Sec. 4.5 for one platform
 * pattern and a cost budget (Sec. 4.2: FLOPs or energy).  Keep set of a
 * threshold v: every head and channel of every layer with score >= v; a layer
 * keeps at least its best head (with its K/V group) and its best channel.
 * Cost = c_fixed + sum_l (heads_l*c_head[l] + groups_l*c_group[l] +
 * channels_l*c_ffn[l]) in the caller's integer units (HOST arrays [nl], >= 0).
 * Finds the smallest score value whose keep set costs <= budget, i.e. the
 * largest network within the budget, by bisection over the ordered bit
 * patterns of the scores (exact, no sort).  Outputs (DEVICE memory):
 *   tau (that score; +inf when nothing fits), k_head [nl], k_ffn [nl] (sizes
 *   of the keep set: pass them to sf_gate_scores_to_masks, whose top-k with
 *   these counts selects exactly the units >= tau), cost, feasible (1 / 0;
 *   0: even the one-unit-per-layer network exceeds the budget; the outputs
 *   then describe that network).
 * Scores must not be NaN.  At most 64 layers and 64 K/V groups.
 */
enum { SF_GATE_RELU = 0, SF_GATE_TANH = 1 };
typedef struct sf_gate_params {
    int32_t n_modalities;      /* M <= 32 */
    int32_t hidden;            /* <= 1024 */
    int32_t nonlin;            /* SF_GATE_RELU | SF_GATE_TANH */
    int32_t reserved;
    const void *Wa, *ba, *Wb, *cb, *zeta, *gamma;
} sf_gate_params;
int32_t sf_gate_eval(const sf_desc *desc, const sf_gate_params *gate_host, const int32_t *pattern_bits,
                     float *g_head, float *g_ffn, void *stream);
int32_t sf_budget_search(const sf_desc *desc, const float *g_head, const float *g_ffn, int32_t pattern,
                         const int64_t *c_head_host, const int64_t *c_group_host,
                         const int64_t *c_ffn_host, int64_t c_fixed, int64_t budget, float *tau,
                         int32_t *k_head, int32_t *k_ffn, int64_t *cost, int32_t *feasible, void *stream);

/* ------------------------------------------------------------------------
 * Measurement aid (not part of the method): per-kernel HIP-event timing.
 * sf_profile_begin(kernel_class, max_launches) creates max_launches event
 * pairs; from then on every launch of that kernel class made by this library
 * (from any entry point, on any stream) is bracketed by one pair until
 * sf_profile_end, which synchronises the recorded events, returns the number
 * of launches seen, the sum of their durations in milliseconds and (when
 * each_ms_host is not NULL: a host array of max_launches floats) every
 * duration in launch order, and destroys the events.  Launches beyond max_launches are not timed.  Not
 * thread-safe; do not use under graph capture.
 */
enum { SF_KERNEL_GEMM = 0,      /* bf16 MFMA GEMM (all projections and both FFN GEMMs) */
       SF_KERNEL_SCORE = 1,     /* sparsity-score stream (QK^T with running max) */
       SF_KERNEL_ATTEND = 2 };  /* active-row attention (Eq. (6)) */
int32_t sf_profile_begin(int32_t kernel_class, int32_t max_launches);
int32_t sf_profile_end(int32_t *n_launches_host, float *total_ms_host, float *each_ms_host);

/* ------------------------------------------------------------------------
 * Measurement aids: what this GPU reaches on the two resources the kernels
 * are bound by, to be timed by the caller on the launch stream (the benchmark
 * reports both next to the published peaks).  No part of the method.
 *
 * sf_ceiling_mfma_launch: `workgroups` workgroups of 8 waves (two per SIMD)
 * each issue iters * 32 independent 32x32x16 bf16 (FP16 build: fp16) MFMAs
 * from operands held in registers - no memory traffic.  random_operands = 0:
 * one constant operand pattern; 1: rotating pseudo-random operands in [-1, 1)
 * (the data-dependent power draw of a real contraction, which lowers the
 * sustained clock).  sink [workgroups] fp32 device (never written in
 * practice).  Returns the flops of the launch, or a negative status.
 *
 * sf_ceiling_copy_launch: dst[0:bytes] = src[0:bytes] with 16 bytes per lane
 * (reads `bytes` and writes `bytes` of HBM); 16-byte aligned, bytes % 16 == 0.
 */
int64_t sf_ceiling_mfma_launch(int32_t workgroups, int32_t iters, int32_t random_operands,
                               float *sink, void *stream);
int32_t sf_ceiling_copy_launch(const void *src, void *dst, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SENTRYFUSE_H */
