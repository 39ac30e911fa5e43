/*
 * CPU oracle for the pruned multimodal encoder forward of SentryFuse
 * (SentryGate keep-masks + SentryAttend sparse grouped-query attention +
 * pruned FFN).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 implementation that
 * exists only so that tests, the smoke check and the benchmark's CPU-baseline
 * leg have something independent to compare the GPU library with.  It shares
 * no code, header, table or helper with the GPU library and must never be
 * called from the product path.
 *
 * Every function below takes HOST pointers.  All floating-point tensors are
 * double; "bf16 mode" (bf16 != 0) means: inputs already hold bf16-representable
 * values and every *stored* intermediate tensor is rounded to the nearest bf16
 * value (ties to even) at the points listed at orc_encoder_forward.
 *
 * Readings of the paper that the paper itself does not pin ("parity
 * unpinned"): the query sparsity score is max-minus-mean of the scaled dot
 * products (Sec. 4.4 only cites the measure), the lazy-row context vector is
 * the arithmetic mean of V_g (Sec. 4.4 says "aggregated"), the FFN activation
 * is ReLU or erf-GELU, and the layer is pre-norm.  The pins in tests/ only
 * check those readings for self-consistency; everything else is pinned.
 */
#ifndef SENTRY_ORACLE_H
#define SENTRY_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Number of active queries per head, Sec. 4.4: U = c * ceil(ln T), clipped to
 * T.  The worked example (n=8, T=128, c=5 -> U ~ 25) fixes the natural log. */
int32_t orc_num_active(int32_t T, int32_t c);

/* Round a double to the nearest bf16-representable value, ties to even. */
double orc_round_bf16(double x);
/* nearest IEEE binary16 value (ties to even, overflow to infinity, subnormals kept).  Wherever a function below takes
 * `bf16`, 0 = no storage rounding, 1 = bfloat16, 2 = binary16: the FP16 variant of the model has the same rounding points. */
double orc_round_f16(double x);

/*
 * Sec. 4.2 / Sec. 4.4: a sample's presence mask m in {0,1}^M decides which positions of the concatenated
 * per-modality token sequence may serve as attention keys (and as active queries):
 *   key_valid[b, j] = 1  if tok_modality[j] < 0           (a token of no modality, e.g. a fusion token: always there)
 *                        or presence[b, tok_modality[j]]   (token j belongs to a modality that sample b has)
 *                   = 0  otherwise.
 *   presence [B,M] (any non-zero byte = present), tok_modality [L] (values < M), key_valid [B,L] out.
 * returns 0; -1 on bad arguments (a modality id >= M); -2 when some sample has no allowed position at all.
 */
int32_t orc_key_valid(int32_t B, int32_t M, int32_t L, const uint8_t *presence, const int32_t *tok_modality,
                      uint8_t *key_valid);

/*
 * Sec. 4.5 "Head pruning with GQA consistency" / "FFN pruning", with integer
 * keep counts per layer: for each (layer l, presence pattern p) keep the
 * k_head[l] heads and k_ffn[l] channels with the highest gate score (ties: the
 * lower index wins).  K/V groups kept = { floor(h / (Hq/Hk)) : h kept }.
 *
 *   g_head [nl,P,Hq], g_ffn [nl,P,F]         gate scores
 *   head_mask [nl,P,Hq], ffn_mask [nl,P,F]   1 = kept
 *   head_idx [nl,P,Hq] (first k_head[l] valid, ascending, rest -1)
 *   ffn_idx  [nl,P,F]  (first k_ffn[l] valid, ascending, rest -1)
 *   group_idx [nl,P,Hk] kept groups ascending, rest -1;  n_groups [nl,P]
 *   head_group [nl,P,Hq]: for kept head i (i-th entry of head_idx) the rank of
 *                         its group inside group_idx; rest -1
 * returns 0, or -1 on bad arguments.
 */
int32_t orc_gate_scores_to_masks(int32_t nl, int32_t P, int32_t Hq, int32_t Hk, int32_t F,
                                 const float *g_head, const float *g_ffn,
                                 const int32_t *k_head, const int32_t *k_ffn,
                                 uint8_t *head_mask, uint8_t *ffn_mask,
                                 int32_t *head_idx, int32_t *ffn_idx,
                                 int32_t *group_idx, int32_t *n_groups, int32_t *head_group);

/* Row gather: dst[i, :] = src[idx[i], :] for i < n_keep (Sec. 4.5:
 * W1' = W1[:, N_keep], W2' = W2[N_keep, :], and the head blocks of W_Q).
 * rows are `row_len` doubles; `block` consecutive rows move per index. */
void orc_gather_rows(const double *src, const int32_t *idx, int32_t n_keep,
                     int32_t block, int64_t row_len, double *dst);

/* One encoder layer's parameters as the oracle sees them.  Unit-major: every
 * head dimension / FFN channel is one contiguous row of length d.
 *   Wq [nH*dh, d]  (column blocks of the paper's W_Q in R^{d x Hq*dh})
 *   Wk, Wv [nG*dh, d]
 *   Wo [nH*dh, d]  (row blocks of the output projection)
 *   W1 [F, d]      (columns of the paper's W_1 in R^{d x F})
 *   W2 [F, d]      (rows of the paper's W_2 in R^{F x d})
 * biases may be NULL.  head_group[h] = K/V group (0..nG-1) used by head h.
 * head_mask[h] / ffn_mask[f] = 0 removes the unit (NULL = keep all). */
typedef struct {
    int32_t nH, nG, dh, d, F;
    const double *Wq, *bq, *Wk, *bk, *Wv, *bv, *Wo, *bo;
    const double *W1, *b1, *W2, *b2;
    const double *ln1_g, *ln1_b, *ln2_g, *ln2_b;
    const int32_t *head_group;
    const uint8_t *head_mask;
    const uint8_t *ffn_mask;
} orc_layer;

/* LayerNorm over the last dimension (biased variance). y may alias x. */
void orc_layernorm(const double *x, int64_t rows, int32_t d, const double *gamma,
                   const double *beta, double eps, int32_t bf16, double *y);

/*
 * SentryAttend, Sec. 4.4 Eq. (6), for B samples.
 *   Q [B,nH,L,dh], K,V [B,nG,L,dh], head_group [nH] (shared by all samples)
 *   head_group_b: if not NULL, [B,nH] per-sample head->group map (overrides)
 *   key_valid [B,L] or NULL (all keys allowed)
 *   sample_idx [B,n_sample] or NULL: key sample of each sample for the
 *             sparsity score (the sampled-key estimate behind the O(T log T)
 *             claim of Sec. 4.4): the score's max and mean run over the allowed
 *             keys listed here only (a set: duplicates and entries outside
 *             [0,L) are ignored; an empty set scores every allowed query 0).
 *             Active-row attention and the context vector are unaffected.
 *   U         number of active queries per head (U >= L: every row active)
 *   forced_sel [B,nH,U] or NULL: use these query indices (entries < 0 skipped)
 *              instead of the oracle's own top-U choice
 * outputs (any may be NULL):
 *   O     [B,L,nH*dh]  heads concatenated in index order
 *   score [B,nH,L]     sparsity score M_i (-inf for disallowed queries)
 *   sel   [B,nH,U]     chosen queries ascending, padded with -1
 *   prob_check [2]     max |rowsum-1| over active rows, max prob on a
 *                      disallowed key (softmax invariants)
 * returns 0, or -1 on bad arguments (a sample with no allowed key).
 */
int32_t orc_sparse_gqa(int32_t B, int32_t nH, int32_t nG, int32_t L, int32_t dh,
                       const double *Q, const double *K, const double *V,
                       const int32_t *head_group, const int32_t *head_group_b,
                       const uint8_t *key_valid, const int32_t *sample_idx, int32_t n_sample,
                       int32_t U, const int32_t *forced_sel,
                       int32_t bf16, double *O, double *score, int32_t *sel,
                       double *prob_check);

/* Pruned FFN with residual, Sec. 4.5: y = x + act(LN2(x) W1'^T + b1') W2' + b2
 * for `rows` tokens of one pattern.  act: 0 ReLU, 1 erf-GELU.
 * add_residual = 0 drops the "x +".  pre_ln = 0 skips the LayerNorm. */
void orc_pruned_ffn(const orc_layer *w, const double *x, int64_t rows, int32_t act,
                    double eps, int32_t pre_ln, int32_t add_residual, int32_t bf16,
                    double *y);

/*
 * The whole pruned encoder forward: for l = 0..nl-1
 *     x <- x + Wo-proj( SentryAttend( QKV-proj( LN1(x) ) ) )
 *     x <- x + FFN( LN2(x) )
 * and an optional final LayerNorm.
 *   x [B,L,d] in, y [B,L,d] out
 *   layers [nl*P]      layer l of pattern p at layers[l*P + p]
 *   pattern_id [B]     (NULL = all 0)
 *   key_valid [B,L] or NULL
 *   sample_idx [B,n_sample] or NULL: key sample for the sparsity score, as in
 *              orc_sparse_gqa (the same sample in every layer)
 *   forced_sel [nl,B,nHmax,U] or NULL (nHmax = max nH over all layers)
 *   sel_out    [nl,B,nHmax,U] or NULL, score_out [nl,B,nHmax,L] or NULL
 *   final_g/final_b [d] or NULL (no final LN)
 * bf16 rounding points (bf16 != 0): LN outputs, Q, K, V, the attention output
 * O, the FFN hidden after the activation, and the final output y.  The
 * residual stream x itself is an accumulation and is NOT rounded between
 * layers ("bf16 inputs, fp32 accumulate"): with a bf16-stored stream two
 * equally valid implementations drift apart by several bf16 ulps over a few
 * layers, more than the 2e-2 parity bar.
 * returns 0 or -1.
 */
int32_t orc_encoder_forward(int32_t B, int32_t L, int32_t nl, int32_t P,
                            const orc_layer *layers, const int32_t *pattern_id,
                            const uint8_t *key_valid, const int32_t *sample_idx, int32_t n_sample,
                            int32_t U, int32_t act, double eps,
                            const int32_t *forced_sel, int32_t nHmax,
                            const double *final_g, const double *final_b, int32_t bf16,
                            const double *x, double *y, int32_t *sel_out, double *score_out);

/*
 * Sparse-MoE FFN with pruned experts, Sec. 4.5 "Sparse-MoE FFN pruning": the
 * number of experts E and the Top-k routing stay fixed; every expert e keeps
 * its own channel set (W1_e' = W1_e[:, N_keep_e], W2_e' = W2_e[N_keep_e, :]),
 * here given as a mask over its F channels.  One presence pattern per call.
 *   Wr [E,d], br [E] or NULL   router (not pruned)
 *   W1 [E,F,d], b1 [E,F] or NULL, W2 [E,F,d], b2 [E,d] or NULL (unit-major, as orc_layer)
 *   ffn_mask [E,F] or NULL     1 = channel kept
 *   ln_g, ln_b [d]             pre-norm LayerNorm of the block (used when pre_ln)
 * The paper fixes neither the router nor the combination; this library's
 * reading is the common one: with xn = LayerNorm(x) (or x),
 *   logit_e = xn . Wr_e + br_e;  the k experts with the highest logit are
 *   chosen (ties: lower expert index; the comparison is made on the logits
 *   rounded to fp32, the precision the GPU router compares in);
 *   p_e = softmax over the chosen logits;
 *   y = [x +] sum_{chosen e} p_e * ( act(xn W1_e'^T + b1_e') W2_e' + b2_e ).
 * bf16 rounding points: xn, each expert's hidden activations, and y.
 *   forced_route [rows,k] or NULL: use these experts (distinct, 0..E-1) instead
 *   route_out [rows,k] (chosen experts, descending logit), weight_out [rows,k],
 *   logit_out [rows,E]: any may be NULL
 * returns 0 or -1.
 */
typedef struct {
    int32_t d, F, E, k;
    const double *Wr, *br;
    const double *W1, *b1, *W2, *b2;
    const uint8_t *ffn_mask;
    const double *ln_g, *ln_b;
} orc_moe;
int32_t orc_moe_ffn(const orc_moe *m, const double *x, int64_t rows, int32_t act, double eps,
                    int32_t pre_ln, int32_t add_residual, int32_t bf16,
                    const int32_t *forced_route, double *y, int32_t *route_out,
                    double *weight_out, double *logit_out);

/* Threads the OpenMP runtime will use (for the benchmark's report). */
/*
 * SentryGate importance scores, Eq. (1):  g_i(m) = sigmoid( zeta_i + gamma * f_i(m) )  for the units i of one
 * layer (its heads and its FFN channels) and one modality-availability mask m in {0,1}^M.
 * f is a two-layer perceptron with a nonlinearity; the paper gives neither its width nor the nonlinearity.
 * Reading: the first layer is shared by the units of the layer, h = nonlin(Wa m + ba) with Hd hidden units,
 * and every unit has its own output row, f_i = Wb[i,:] . h + cb[i].  nonlin: 0 = ReLU, 1 = tanh.
 *   Wa [Hd,M], ba [Hd], Wb [n_units,Hd], cb [n_units], zeta [n_units]; bit j of pattern_bits = m_j
 *   g [n_units] (fp64)
 * returns 0, or -1 on bad arguments.
 */
int32_t orc_gate_eval(int32_t M, int32_t Hd, int32_t n_units, int32_t nonlin, const double *Wa,
                      const double *ba, const double *Wb, const double *cb, const double *zeta,
                      double gamma, uint32_t pattern_bits, double *g);

/*
 * Global threshold for a cost budget (Sec. 4.5, the paragraph before "Head pruning ...": the gate outputs of
 * all layers are evaluated for one platform mask and thresholded globally; Sec. 4.2: the threshold is chosen to
 * meet a FLOPs or energy budget).  Keep set of a threshold v: every head and channel with score >= v; a layer
 * whose heads (channels) all fall below v keeps its best head (channel), ties to the lower index, so that no
 * layer disappears (reading; the paper does not say).  K/V groups follow the kept heads as in
 * orc_gate_scores_to_masks.  Cost of a keep set, in integer units supplied by the caller:
 *   c_fixed + sum_l ( kept_heads_l * c_head[l] + kept_groups_l * c_group[l] + kept_channels_l * c_ffn[l] ).
 * Result: the smallest score value v among all units whose keep set costs <= budget (the largest network within
 * the budget); k_head[l], k_ffn[l] are the sizes of that keep set and *cost its cost.  Every candidate value is
 * tried (no search order is assumed).  Scores must not be NaN.
 *   g_head [nl,Hq], g_ffn [nl,F] (fp32, the scores of the platform's pattern)
 * returns 1 when such a value exists; 0 when even the one-unit-per-layer network exceeds the budget (then
 * *tau = +inf and the outputs describe that minimal network); -1 on bad arguments.
 */
int32_t orc_budget_search(int32_t nl, int32_t Hq, int32_t Hk, int32_t F, const float *g_head,
                          const float *g_ffn, const int64_t *c_head, const int64_t *c_group,
                          const int64_t *c_ffn, int64_t c_fixed, int64_t budget, float *tau,
                          int32_t *k_head, int32_t *k_ffn, int64_t *cost);

/*
 * FP8 post-training quantisation of the weights (Sec. 6, "Compatibility with quantization": FP8 PTQ on top of the
 * pruned model; the paper names neither the format nor the scaling: "parity unpinned" for that choice, the format's
 * decode and the rounding are pinned against a library implementation).  Reading: weights are stored as OCP E4M3
 * bytes (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities, S.1111.111 is NaN, largest finite
 * value 448, subnormals m * 2^-9) with one fp32 scale per weight matrix; the pruned forward runs on the
 * dequantised weight w = decode(byte) * scale, rounded to the model dtype (bf16, ties to even, when bf16 != 0;
 * fp32 otherwise).  The product of a 4-bit and a 24-bit significand is exact in double, so there is one rounding.
 *   orc_fp8_e4m3_decode: the value of one byte.
 *   orc_dequant_fp8: out[i] = round(decode(q[i]) * scale), n elements.
 */
double orc_fp8_e4m3_decode(uint8_t byte);
void orc_dequant_fp8(const uint8_t *q, int64_t n, float scale, int32_t bf16, double *out);

/*
 * FP16 post-training quantisation of the weights (same experiment, the FP16 points; the paper does not say what is
 * stored or how it is used: "parity unpinned" for that reading, the decode itself is pinned against a library
 * binary16).  Reading: weights are stored
 * as IEEE binary16 (1-5-10, subnormals, infinities, NaN), no scale; the forward runs on the stored value in the
 * model dtype: every binary16 value is an fp32 value, so an fp32 model computes on exactly the stored weights, and a
 * bf16 model on their one rounding to bf16 (ties to even).
 *   orc_f16_decode: the value of one bit pattern;  orc_dequant_f16: out[i] = round(decode(q[i])).
 */
double orc_f16_decode(uint16_t bits);
void orc_dequant_f16(const uint16_t *q, int64_t n, int32_t bf16, double *out);

/*
 * FP8 arithmetic for the pruned FFN (the second half of the same experiment: the paper reports FP8 models but
 * not how they compute; the scheme below is this build's reading, "parity unpinned" as far as the paper goes, pinned
 * against library casts, LayerNorm and matmul in the tests).  Reading: both operands of the two FFN contractions are E4M3 codes with one fp32
 * scale per tensor (W8A8, static scales chosen offline), products are exact and sums wide:
 *     xq  = Q(LN2(x), sx)                                    (LN2 in fp64, its result rounded to fp32)
 *     z   = (sum_k dec(xq_k) dec(W1q_fk)) * fl32(sx*s1) + b1_f      rounded to fp32
 *     hq  = Q(act(z), sh)
 *     y   = (sum_f dec(hq_f) dec(W2q_fn)) * fl32(sh*s2) + b2_n (+ x)   rounded to bf16 when bf16 != 0
 * with Q(t, s) = E4M3( fl32( t * fl32(1/s) ) ): one fp32 reciprocal, one fp32 product, then round to nearest,
 * ties to the even code, values beyond +-448 saturate to +-448, NaN gives 0x7F.  The code is decided from fp32
 * values because that is the precision the device path holds them in.  Removed channels (ffn_mask[f] = 0)
 * contribute nothing.  W1q, W2q [F,d] codes of the dense layout (one row per channel).
 *   orc_fp8_e4m3_encode: the code of one fp32 value.
 *   orc_quantize_fp8:    codes[i] = Q(x[i], scale).
 *   orc_pruned_ffn_fp8:  the block; xq_out [rows,d], hq_out [rows,F] (codes, 0 for removed channels) and z_out
 *                        [rows,F] (the fp32 value z, 0 for removed channels) may be NULL.  xq_forced / hq_forced
 *                        (NULL = none) replace the block's own codes of the input / of the hidden activations:
 *                        a code is a floating-point decision, and a test that has checked another
 *                        implementation's decisions compares the rest of the block on those.
 */
uint8_t orc_fp8_e4m3_encode(float t);
void orc_quantize_fp8(const float *x, int64_t n, float scale, uint8_t *codes);
void orc_pruned_ffn_fp8(int32_t d, int32_t F, const uint8_t *W1q, float s1, const double *b1,
                        const uint8_t *W2q, float s2, const double *b2, const double *ln_g,
                        const double *ln_b, const uint8_t *ffn_mask, float sx, float sh,
                        const double *x, int64_t rows, int32_t act, double eps, int32_t pre_ln,
                        int32_t add_residual, int32_t bf16, const uint8_t *xq_forced,
                        const uint8_t *hq_forced, double *y, uint8_t *xq_out, uint8_t *hq_out, double *z_out);

/* The encoder with the FFN of every layer in FP8 arithmetic (orc_pruned_ffn_fp8 on the unrounded residual stream,
 * LayerNorm vectors, biases and channel masks of `layers`); everything else as orc_encoder_forward, which is this
 * function with ffn8 = NULL.
 *   ffn8 [nl]          codes and scales of each layer's FFN in the layout of that layer's W1 / W2 (shared by all
 *                      patterns, so `layers` must hold the dense weights with their 0/1 channel masks)
 *   xq_forced [nl,B,L,d], hq_forced [nl,B,L,F] or NULL: codes to use instead of the oracle's own (see
 *              orc_pruned_ffn_fp8) in the layers l < n_forced_x / l < n_forced_h: a test walks the layers and takes
 *              the oracle's own decision of layer l on the other implementation's decisions of the layers before
 *   xq_out, hq_out: the codes used, same shapes, or NULL */
typedef struct {
    const uint8_t *W1q, *W2q;       /* [F,d] E4M3 codes */
    float s1, s2, sx, sh;
} orc_ffn8;
int32_t orc_encoder_forward_fp8ffn(int32_t B, int32_t L, int32_t nl, int32_t P,
                                   const orc_layer *layers, const orc_ffn8 *ffn8, const int32_t *pattern_id,
                                   const uint8_t *key_valid, const int32_t *sample_idx, int32_t n_sample,
                                   int32_t U, int32_t act, double eps,
                                   const int32_t *forced_sel, int32_t nHmax,
                                   const double *final_g, const double *final_b, int32_t bf16,
                                   const uint8_t *xq_forced, const uint8_t *hq_forced,
                                   int32_t n_forced_x, int32_t n_forced_h,
                                   const double *x, double *y, int32_t *sel_out, double *score_out,
                                   uint8_t *xq_out, uint8_t *hq_out);

/* FP8 arithmetic for the attention projections of one layer (used by every pattern).  The paper reports FP8 models
 * without saying which contractions run in FP8 or how: this reading is "parity unpinned" as far as the paper goes and
 * pinned in the tests against a numpy matrix form built on the library's float8 casts.  Reading, with Q(t, s) and
 * dec() as in the FFN block above:
 *     aq      = Q(LN1(x), sx1)                                     (LN1 in fp64, its result rounded to fp32)
 *     q, k, v = (sum_c dec(aq_c) dec(W8_uc)) * fl32(sx1*s_qkv) + b_u     stored as bf16 when bf16 != 0
 *     oq      = Q(attention output, sa)                            (0 for a removed head)
 *     x      <- x + (sum_c dec(oq_c) dec(Wo8_cn)) * fl32(sa*so) + bo_n
 * SentryAttend between the two runs on q, k, v as in the plain encoder.  E4M3 codes of the dense Wq [nH*dh, d],
 * Wk, Wv [nG*dh, d] carry ONE scale s_qkv (the three are one fused operand of one GEMM), those of Wo [nH*dh, d]
 * carry so. */
typedef struct {
    const uint8_t *Wq8, *Wk8, *Wv8, *Wo8;
    float s_qkv, so, sx1, sa;
} orc_proj8;
/* codes forced in / reported: xq = LN2 output [nl,B,L,d], hq = hidden [nl,B,L,F], aq = LN1 output [nl,B,L,d],
 * oq = attention output [nl,B,L,nH*dh]; forced in layers l < n_forced_* only */
typedef struct {
    const uint8_t *xq_forced, *hq_forced, *aq_forced, *oq_forced;
    int32_t n_forced_x, n_forced_h, n_forced_a, n_forced_o;
    uint8_t *xq_out, *hq_out, *aq_out, *oq_out;
} orc_fp8_io;
/* The encoder with the FFN (ffn8 != NULL) and / or the attention projections (proj8 != NULL) in FP8 arithmetic;
 * SentryAttend itself and the residual stream are unchanged.  io may be NULL. */
int32_t orc_encoder_forward_fp8(int32_t B, int32_t L, int32_t nl, int32_t P,
                                const orc_layer *layers, const orc_ffn8 *ffn8, const orc_proj8 *proj8,
                                const int32_t *pattern_id, const uint8_t *key_valid, const int32_t *sample_idx,
                                int32_t n_sample, int32_t U, int32_t act, double eps,
                                const int32_t *forced_sel, int32_t nHmax,
                                const double *final_g, const double *final_b, int32_t bf16,
                                const orc_fp8_io *io, const double *x, double *y, int32_t *sel_out, double *score_out);

int32_t orc_max_threads(void);

#ifdef __cplusplus
}
#endif
#endif
