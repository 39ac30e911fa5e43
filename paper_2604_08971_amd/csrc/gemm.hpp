// Interface of the GEMM used for every projection of the encoder layer:
//   C[b*L+i, n0+n] = act( sum_k A[b*L+i, k] * W[p(b)][n0+n, k] + bias[p(b)][n0+n] ) (+ R[b*L+i, n0+n])
// A is token-major, W is unit-major (one output feature per row), p(b) is the
// presence pattern of sample b, so tiles never straddle two samples.
#pragma once

#include "common.hpp"

namespace sf {

enum { EPI_ROWMAJOR = 0, EPI_VT = 1 };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2 };

struct GemmArgs {
    const void *A; int64_t lda;
    const void *W; int64_t ldw; int64_t w_pstride;       // elements between patterns
    const void *bias; int64_t bias_pstride;              // may be NULL; 0 stride = shared
    const int32_t *pattern_id;                           // [B] or NULL (pattern 0); a negative entry skips the sample
    const int32_t *n_lim, *k_lim;                        // per pattern, may be NULL: only the first n_lim[p] features
                                                         // are computed (the others are not written) and only the first
                                                         // k_lim[p] elements of K are summed (n_lim % 8 == 0,
                                                         // k_lim % 64 == 0, k_lim >= 64); device memory
    int B, L, N, K;                                      // N = number of output features of this launch
    int n0;                                              // first feature (row of W, entry of bias)
    int epi;                                             // EPI_ROWMAJOR: C[row, c0 + n], EPI_VT: C[b, n, i]
    int act;
    const void *R; int64_t ldr; int r0;                  // residual (NULL = none), first column r0
    void *C; int64_t ldc; int c0;                        // EPI_ROWMAJOR: row stride, first column
    const int32_t *row_map;                              // large bf16 row-major problems only (gemm_takes_row_map): row i
                                                         // of sample b reads A row row_map[b*L + i] (all of A within 4 GiB)
    int xcd_rows;                                        // hint: deal 256-row tiles to the 8 XCDs round-robin instead of in
                                                         // contiguous ranges (rows of unequal cost, e.g. n_lim / k_lim)
    int r_f32, c_f32;                                    // bf16 GEMM only: R / C hold fp32 (the residual stream)
    int64_t vt_b, vt_n;                                  // EPI_VT: strides of b and n (i contiguous)
    int f8;                                              // gemm_fp8() only: A and W hold E4M3 codes (lda, ldw, w_pstride in
                                                         // elements = bytes), K % 128 == 0
    float out_scale;                                     // f8: factor of the sum of code products (the two tensor scales)
    int c_f8; float c_scale;                             // f8: C receives E4M3 codes of act(value) * c_scale (ldc in bytes)
    void *VT; int vt_from;                               // large bf16 row-major problems only (gemm_takes_vt_split):
                                                         // features n >= vt_from go to VT[b, n - vt_from, i] (strides
                                                         // vt_b, vt_n, both % 8 == 0; vt_from % 8 == 0) instead of C
};

// dtype SF_BF16: bf16 MFMA, fp32 accumulate (K % 8 == 0, lda/ldw/ldr % 8 == 0,
// ldc % 4 == 0, 16-byte aligned bases).  dtype SF_F32: fp32 FMA.
int32_t gemm(int dtype, const GemmArgs &a, hipStream_t st);

// E4M3 x E4M3 -> fp32 accumulate (large row-major problems only, else SF_ERR_UNSUPPORTED / SF_ERR_SHAPE).
int32_t gemm_fp8(const GemmArgs &a, hipStream_t st);

// The pruned FFN in FP8 arithmetic (fp8_ffn.hip): checks, then LayerNorm + quantiser, up-projection writing codes,
// down-projection with the residual.  x_f32 / y_f32: X / Y hold fp32 (the encoder's residual stream).
// xq [B*L, d], hq [B*L, Fp8] receive the codes.
struct Dims;
int32_t ffn_fp8_check(const char *who, const Dims &D, const sf_ffn_fp8 *f, bool pre_ln);
int32_t ffn_fp8_forward(const Dims &D, const sf_ffn_fp8 &f, const void *X, bool x_f32, const int32_t *pattern_id,
                        bool pre_ln, bool add_residual, void *Y, bool y_f32, uint8_t *xq, uint8_t *hq, hipStream_t st,
                        bool xq_ready = false);      // xq_ready: xq already holds the codes of LN2(X)

// Quantisers of fp8_ffn.hip: y = E4M3(LayerNorm(x) * inv_scale) for rows of d elements (d % 8 == 0, d <= 4096, gamma /
// beta bf16, 16-byte aligned), and codes = E4M3(x * inv_scale) for n bf16 values (x 16-byte, codes 8-byte aligned).
void layernorm_q8(const void *X, bool x_f32, const void *gamma, const void *beta, float eps, int64_t rows, int d,
                  float inv_scale, uint8_t *y, hipStream_t st);
void quantize_fp8_bf16(const void *x, int64_t n, float inv_scale, uint8_t *codes, hipStream_t st);

// The attention projections in FP8 arithmetic (fp8_proj.hip).
int32_t proj_fp8_check(const char *who, const Dims &D, const sf_proj_fp8 *p, int k_head);
// vt[b, c, j] = src[b, j, col0 + c] for c < ncols, j < L (zeros for L <= j < Lp): the V columns of a token-major
// bf16 buffer into the key-contiguous layout the attention kernels read.
// codes[r, 0:K] = E4M3(x[r, 0:K] * inv_scale), codes[r, K:Kp] = 0 (x bf16 with row stride ld; K, Kp, ld % 8 == 0)
void quantize_rows_fp8(const void *x, int64_t ld, int64_t rows, int K, int Kp, float inv_scale, uint8_t *codes, hipStream_t st);
void transpose_v(const void *src, int64_t ld, int col0, int ncols, int B, int L, int Lp, void *vt, hipStream_t st,
                 const int32_t *row0 = nullptr);

// True when gemm() honours a.row_map for this problem (else it fails with SF_ERR_UNSUPPORTED).
bool gemm_takes_row_map(int dtype, const GemmArgs &a);

// True when gemm() honours a.VT / a.vt_from for this problem (else it fails with SF_ERR_UNSUPPORTED).
bool gemm_takes_vt_split(int dtype, const GemmArgs &a);

// LayerNorm over rows of d elements (biased variance).  gamma/beta are in the
// model dtype; x is fp32 when x_f32 (or dtype is SF_F32), y is in the model dtype.
void layernorm(int dtype, int x_f32, const void *x, const void *gamma, const void *beta, float eps,
               int64_t rows, int d, void *y, hipStream_t st);

}  // namespace sf
