/*
 * CPU oracle (TEST INFRASTRUCTURE ONLY) -- see sentry_oracle.h.
 *
 * Plain C, fp64 everywhere, single accumulator per output in index order,
 * no blocking and no fusion: each function is the definition written out.
 * OpenMP only splits independent output rows between threads.
 */
#include "sentry_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- SentryGate: Eq. (1) and the global threshold ------------------------ */
int32_t orc_gate_eval(int32_t M, int32_t Hd, int32_t n_units, int32_t nonlin, const double *Wa,
                      const double *ba, const double *Wb, const double *cb, const double *zeta,
                      double gamma, uint32_t pattern_bits, double *g)
{
    if (M < 1 || M > 32 || Hd < 1 || n_units < 1 || nonlin < 0 || nonlin > 1 || !Wa || !Wb || !zeta || !g)
        return -1;
    double *h = (double *)malloc(sizeof(double) * (size_t)Hd);
    if (!h) return -1;
    for (int32_t r = 0; r < Hd; ++r) {
        double a = ba ? ba[r] : 0.0;
        for (int32_t j = 0; j < M; ++j) {
            const double mj = (double)((pattern_bits >> j) & 1u);
            a += Wa[(int64_t)r * M + j] * mj;
        }
        h[r] = nonlin == 0 ? (a > 0.0 ? a : 0.0) : tanh(a);
    }
    for (int32_t i = 0; i < n_units; ++i) {
        double f = cb ? cb[i] : 0.0;
        for (int32_t r = 0; r < Hd; ++r) f += Wb[(int64_t)i * Hd + r] * h[r];
        const double z = zeta[i] + gamma * f;
        g[i] = 1.0 / (1.0 + exp(-z));
    }
    free(h);
    return 0;
}

/* cost and sizes of the keep set of threshold v (see the header) */
static int64_t keep_set_cost(int32_t nl, int32_t Hq, int32_t Hk, int32_t F, const float *g_head,
                             const float *g_ffn, const int64_t *c_head, const int64_t *c_group,
                             const int64_t *c_ffn, int64_t c_fixed, float v, int32_t *k_head,
                             int32_t *k_ffn)
{
    const int32_t per_group = Hq / Hk;
    int64_t cost = c_fixed;
    for (int32_t l = 0; l < nl; ++l) {
        const float *gh = g_head + (int64_t)l * Hq, *gf = g_ffn + (int64_t)l * F;
        int32_t kh = 0, kg = 0, kf = 0;
        for (int32_t grp = 0; grp < Hk; ++grp) {
            int any = 0;
            for (int32_t h = grp * per_group; h < (grp + 1) * per_group; ++h)
                if (gh[h] >= v) { ++kh; any = 1; }
            kg += any;
        }
        if (kh == 0) { kh = 1; kg = 1; }              /* the best head stays, with its group */
        for (int32_t c = 0; c < F; ++c)
            if (gf[c] >= v) ++kf;
        if (kf == 0) kf = 1;                          /* the best channel stays */
        cost += (int64_t)kh * c_head[l] + (int64_t)kg * c_group[l] + (int64_t)kf * c_ffn[l];
        if (k_head) k_head[l] = kh;
        if (k_ffn) k_ffn[l] = kf;
    }
    return cost;
}

int32_t orc_budget_search(int32_t nl, int32_t Hq, int32_t Hk, int32_t F, const float *g_head,
                          const float *g_ffn, const int64_t *c_head, const int64_t *c_group,
                          const int64_t *c_ffn, int64_t c_fixed, int64_t budget, float *tau,
                          int32_t *k_head, int32_t *k_ffn, int64_t *cost)
{
    if (nl < 1 || Hq < 1 || Hk < 1 || F < 1 || Hq % Hk != 0 || !g_head || !g_ffn || !c_head ||
        !c_group || !c_ffn || !tau || !k_head || !k_ffn || !cost)
        return -1;
    for (int32_t l = 0; l < nl; ++l)
        if (c_head[l] < 0 || c_group[l] < 0 || c_ffn[l] < 0) return -1;
    const int64_t n_head = (int64_t)nl * Hq, n_all = n_head + (int64_t)nl * F;
    int found = 0;
    float best = 0.f;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_all; ++i) {
        const float v = i < n_head ? g_head[i] : g_ffn[i - n_head];
        const int64_t c = keep_set_cost(nl, Hq, Hk, F, g_head, g_ffn, c_head, c_group, c_ffn, c_fixed, v,
                                        NULL, NULL);
        if (c <= budget) {
#pragma omp critical
            {
                if (!found || v < best) { best = v; found = 1; }
            }
        }
    }
    *tau = found ? best : INFINITY;
    *cost = keep_set_cost(nl, Hq, Hk, F, g_head, g_ffn, c_head, c_group, c_ffn, c_fixed, *tau, k_head, k_ffn);
    return found;
}

/* ---- FP8 (OCP E4M3) weights ---------------------------------------------- */
double orc_fp8_e4m3_decode(uint8_t byte)
{
    const int sign = byte >> 7, e = (byte >> 3) & 15, m = byte & 7;
    double v;
    if (e == 15 && m == 7) return NAN;                       /* the only non-finite code */
    if (e == 0) v = ldexp((double)m, -9);                    /* subnormal: (m/8) * 2^-6 */
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

void orc_dequant_fp8(const uint8_t *q, int64_t n, float scale, int32_t bf16, double *out)
{
    for (int64_t i = 0; i < n; ++i) {
        const double w = orc_fp8_e4m3_decode(q[i]) * (double)scale;      /* exact */
        out[i] = bf16 == 1 ? orc_round_bf16(w) : bf16 == 2 ? orc_round_f16(w) : (double)(float)w;
    }
}

int32_t orc_max_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- Sec. 4.4: U = c * ceil(ln T) -------------------------------------- */
int32_t orc_num_active(int32_t T, int32_t c)
{
    if (T <= 0 || c <= 0) return 0;
    double u = (double)c * ceil(log((double)T));
    if (u > (double)T) return T;
    return (int32_t)u;
}

/* ---- bf16: 8 significant bits, exponent range of binary32 -------------- */
double orc_round_bf16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);               /* |x| = m * 2^e, m in [0.5, 1) */
    int q = e - 8;                    /* spacing of bf16 values near x is 2^q */
    if (q < -133) q = -133;           /* subnormal range: fixed spacing 2^-133 */
    double r = ldexp(nearbyint(ldexp(x, -q)), q);   /* nearbyint: ties to even */
    if (fabs(r) >= ldexp(1.0, 128)) r = (x > 0) ? INFINITY : -INFINITY;
    return r;
}

/* ---- binary16: 11 significant bits, normal exponents -14..15 ------------ */
double orc_round_f16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);               /* |x| = m * 2^e, m in [0.5, 1) */
    int q = e - 11;                   /* spacing of binary16 values near x is 2^q */
    if (q < -24) q = -24;             /* subnormal range: fixed spacing 2^-24 */
    double r = ldexp(nearbyint(ldexp(x, -q)), q);   /* nearbyint: ties to even */
    if (fabs(r) > 65504.0) r = (x > 0) ? INFINITY : -INFINITY;
    return r;
}

/* The `bf16` argument of every function below is the model's storage type: 0 = none (fp64 throughout, or fp32 where
 * stated), 1 = bfloat16, 2 = IEEE binary16 (the FP16 variant of the model: the same rounding points) */
static inline double rnd(double x, int32_t bf16)
{
    return bf16 == 1 ? orc_round_bf16(x) : bf16 == 2 ? orc_round_f16(x) : x;
}

/* ---- Sec. 4.5: gate scores -> keep sets -------------------------------- */
typedef struct { float g; int32_t i; } scored;

static int by_score_desc_index_asc(const void *a, const void *b)
{
    const scored *x = (const scored *)a, *y = (const scored *)b;
    if (x->g > y->g) return -1;
    if (x->g < y->g) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

/* mark the k best of n scores; write mask[n] and ascending idx (padded -1) */
static void keep_top_k(const float *g, int32_t n, int32_t k, uint8_t *mask, int32_t *idx)
{
    scored *s = (scored *)malloc(sizeof(scored) * (size_t)n);
    for (int32_t i = 0; i < n; ++i) { s[i].g = g[i]; s[i].i = i; }
    qsort(s, (size_t)n, sizeof(scored), by_score_desc_index_asc);
    memset(mask, 0, (size_t)n);
    for (int32_t r = 0; r < k; ++r) mask[s[r].i] = 1;
    int32_t w = 0;
    for (int32_t i = 0; i < n; ++i) if (mask[i]) idx[w++] = i;
    for (; w < n; ++w) idx[w] = -1;
    free(s);
}

int32_t orc_key_valid(int32_t B, int32_t M, int32_t L, const uint8_t *presence, const int32_t *tok_modality,
                      uint8_t *key_valid)
{
    if (B < 1 || M < 0 || L < 1 || !tok_modality || !key_valid || (M > 0 && !presence)) return -1;
    for (int32_t j = 0; j < L; ++j)
        if (tok_modality[j] >= M) return -1;
    int32_t rc = 0;
    for (int32_t b = 0; b < B; ++b) {
        int32_t any = 0;
        for (int32_t j = 0; j < L; ++j) {
            const int32_t m = tok_modality[j];
            const uint8_t ok = (m < 0 || presence[(size_t)b * M + m] != 0) ? 1 : 0;
            key_valid[(size_t)b * L + j] = ok;
            any |= ok;
        }
        if (!any) rc = -2;
    }
    return rc;
}

int32_t orc_gate_scores_to_masks(int32_t nl, int32_t P, int32_t Hq, int32_t Hk, int32_t F,
                                 const float *g_head, const float *g_ffn,
                                 const int32_t *k_head, const int32_t *k_ffn,
                                 uint8_t *head_mask, uint8_t *ffn_mask,
                                 int32_t *head_idx, int32_t *ffn_idx,
                                 int32_t *group_idx, int32_t *n_groups, int32_t *head_group)
{
    if (nl < 1 || P < 1 || Hq < 1 || Hk < 1 || F < 1 || Hq % Hk != 0) return -1;
    const int32_t per_group = Hq / Hk;      /* heads sharing one K/V projection */
    for (int32_t l = 0; l < nl; ++l) {
        if (k_head[l] < 1 || k_head[l] > Hq || k_ffn[l] < 1 || k_ffn[l] > F) return -1;
        for (int32_t p = 0; p < P; ++p) {
            const int64_t lp = (int64_t)l * P + p;
            uint8_t *hm = head_mask + lp * Hq;
            int32_t *hi = head_idx + lp * Hq;
            keep_top_k(g_head + lp * Hq, Hq, k_head[l], hm, hi);
            keep_top_k(g_ffn + lp * F, F, k_ffn[l], ffn_mask + lp * F, ffn_idx + lp * F);

            /* K_keep = floor(H_keep / (Hq/Hk)); an unreferenced group is removed */
            int32_t *gi = group_idx + lp * Hk;
            int32_t ng = 0;
            for (int32_t g = 0; g < Hk; ++g) {
                int referenced = 0;
                for (int32_t h = 0; h < Hq; ++h)
                    if (hm[h] && h / per_group == g) referenced = 1;
                if (referenced) gi[ng++] = g;
            }
            n_groups[lp] = ng;
            for (int32_t g = ng; g < Hk; ++g) gi[g] = -1;

            int32_t *hg = head_group + lp * Hq;
            for (int32_t i = 0; i < Hq; ++i) {
                hg[i] = -1;
                if (hi[i] < 0) continue;
                for (int32_t r = 0; r < ng; ++r)
                    if (gi[r] == hi[i] / per_group) hg[i] = r;
            }
        }
    }
    return 0;
}

void orc_gather_rows(const double *src, const int32_t *idx, int32_t n_keep,
                     int32_t block, int64_t row_len, double *dst)
{
    for (int32_t i = 0; i < n_keep; ++i)
        for (int32_t r = 0; r < block; ++r)
            memcpy(dst + ((int64_t)i * block + r) * row_len,
                   src + ((int64_t)idx[i] * block + r) * row_len,
                   sizeof(double) * (size_t)row_len);
}

/* ---- LayerNorm ---------------------------------------------------------- */
void orc_layernorm(const double *x, int64_t rows, int32_t d, const double *gamma,
                   const double *beta, double eps, int32_t bf16, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * d;
        double *yr = y + r * d;
        double mean = 0.0;
        for (int32_t k = 0; k < d; ++k) mean += xr[k];
        mean /= d;
        double var = 0.0;
        for (int32_t k = 0; k < d; ++k) var += (xr[k] - mean) * (xr[k] - mean);
        var /= d;                                    /* biased variance */
        const double inv = 1.0 / sqrt(var + eps);
        for (int32_t k = 0; k < d; ++k) {
            double v = (xr[k] - mean) * inv;
            if (gamma) v *= gamma[k];
            if (beta) v += beta[k];
            yr[k] = rnd(v, bf16);
        }
    }
}

/* y[r, n] = sum_k x[r, k] * W[n, k] + b[n]  for the listed output units.
 * W is unit-major (one output unit per row).  out_stride = row length of y. */
static void project_units(const double *x, int64_t rows, int32_t d, const double *W,
                          const double *b, int32_t unit0, int32_t n_units, int32_t bf16,
                          double *y, int64_t out_stride, int32_t out0)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * d;
        for (int32_t n = 0; n < n_units; ++n) {
            const double *wn = W + (int64_t)(unit0 + n) * d;
            double acc = 0.0;
            for (int32_t k = 0; k < d; ++k) acc += xr[k] * wn[k];
            if (b) acc += b[unit0 + n];
            y[r * out_stride + out0 + n] = rnd(acc, bf16);
        }
    }
}

/* ---- SentryAttend for one (sample, head) -------------------------------- */
typedef struct { float m; int32_t i; } qscore;

static int by_m_desc_index_asc(const void *a, const void *b)
{
    const qscore *x = (const qscore *)a, *y = (const qscore *)b;
    if (x->m > y->m) return -1;
    if (x->m < y->m) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

static int int_asc(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * q [L,dh] one head's queries, k,v [L,dh] its group's keys/values,
 * valid [L] or NULL.  Writes o rows at o[i*o_stride + 0..dh).
 * score_out [L] or NULL, sel_out [U] or NULL, forced [U] or NULL.
 * score_keys [L] or NULL: when given, the sparsity score only looks at the
 * allowed keys j with score_keys[j] != 0 (the sampled-key estimate of the
 * measure); the attention of the active rows and the context vector always
 * use every allowed key.
 */
static void sgqa_one_head(int32_t L, int32_t dh, const double *q, const double *k,
                          const double *v, const uint8_t *valid, const uint8_t *score_keys,
                          int32_t U, const int32_t *forced, int32_t bf16, double *o,
                          int64_t o_stride, double *score_out, int32_t *sel_out,
                          double *prob_check)
{
    const double scale = 1.0 / sqrt((double)dh);
    int32_t n_allowed = 0, n_score = 0;
    for (int32_t j = 0; j < L; ++j) {
        if (valid && !valid[j]) continue;
        ++n_allowed;
        if (!score_keys || score_keys[j]) ++n_score;
    }

    /* sparsity score of every query: max_j s_ij - mean_j s_ij over the allowed
     * (and, if a sample is given, sampled) keys; 0 when that set is empty */
    double *M = (double *)malloc(sizeof(double) * (size_t)L);
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < L; ++i) {
        if (valid && !valid[i]) { M[i] = -INFINITY; continue; }
        if (n_score == 0) { M[i] = 0.0; continue; }
        double mx = -INFINITY, sum = 0.0;
        for (int32_t j = 0; j < L; ++j) {
            if (valid && !valid[j]) continue;
            if (score_keys && !score_keys[j]) continue;
            double s = 0.0;
            for (int32_t e = 0; e < dh; ++e) s += q[(int64_t)i * dh + e] * k[(int64_t)j * dh + e];
            s *= scale;
            if (s > mx) mx = s;
            sum += s;
        }
        M[i] = mx - sum / n_score;
    }
    if (score_out) memcpy(score_out, M, sizeof(double) * (size_t)L);

    /* active set: the U queries with the highest score (ties: lower index) */
    uint8_t *active = (uint8_t *)calloc((size_t)L, 1);
    int32_t *chosen = (int32_t *)malloc(sizeof(int32_t) * (size_t)(U > 0 ? U : 1));
    int32_t n_chosen = 0;
    if (forced) {
        for (int32_t r = 0; r < U; ++r)
            if (forced[r] >= 0 && forced[r] < L && !active[forced[r]]) {
                active[forced[r]] = 1;
                chosen[n_chosen++] = forced[r];
            }
    } else {
        qscore *qs = (qscore *)malloc(sizeof(qscore) * (size_t)L);
        int32_t nq = 0;
        for (int32_t i = 0; i < L; ++i)
            if (!valid || valid[i]) { qs[nq].m = (float)M[i]; qs[nq].i = i; ++nq; }
        qsort(qs, (size_t)nq, sizeof(qscore), by_m_desc_index_asc);
        for (int32_t r = 0; r < nq && r < U; ++r) {
            active[qs[r].i] = 1;
            chosen[n_chosen++] = qs[r].i;
        }
        free(qs);
    }
    qsort(chosen, (size_t)n_chosen, sizeof(int32_t), int_asc);
    if (sel_out) {
        for (int32_t r = 0; r < U; ++r) sel_out[r] = r < n_chosen ? chosen[r] : -1;
    }

    /* context vector: mean of V_g over allowed keys */
    double *ctx = (double *)calloc((size_t)dh, sizeof(double));
    for (int32_t j = 0; j < L; ++j) {
        if (valid && !valid[j]) continue;
        for (int32_t e = 0; e < dh; ++e) ctx[e] += v[(int64_t)j * dh + e];
    }
    for (int32_t e = 0; e < dh; ++e) ctx[e] /= n_allowed;

    double worst_sum = 0.0, worst_leak = 0.0;
#pragma omp parallel for schedule(static) reduction(max : worst_sum, worst_leak)
    for (int32_t i = 0; i < L; ++i) {
        double *oi = o + (int64_t)i * o_stride;
        if (!active[i]) {                       /* lazy row */
            for (int32_t e = 0; e < dh; ++e) oi[e] = rnd(ctx[e], bf16);
            continue;
        }
        /* active row, Eq. (6): softmax(q_i K_g^T / sqrt(d_k)) V_g */
        double *p = (double *)malloc(sizeof(double) * (size_t)L);
        double mx = -INFINITY;
        for (int32_t j = 0; j < L; ++j) {
            if (valid && !valid[j]) { p[j] = -INFINITY; continue; }
            double s = 0.0;
            for (int32_t e = 0; e < dh; ++e) s += q[(int64_t)i * dh + e] * k[(int64_t)j * dh + e];
            p[j] = s * scale;
            if (p[j] > mx) mx = p[j];
        }
        double den = 0.0;
        for (int32_t j = 0; j < L; ++j) {
            p[j] = (valid && !valid[j]) ? 0.0 : exp(p[j] - mx);
            den += p[j];
        }
        double rowsum = 0.0, leak = 0.0;
        for (int32_t j = 0; j < L; ++j) {
            p[j] /= den;
            rowsum += p[j];
            if (valid && !valid[j] && p[j] > leak) leak = p[j];
        }
        if (fabs(rowsum - 1.0) > worst_sum) worst_sum = fabs(rowsum - 1.0);
        if (leak > worst_leak) worst_leak = leak;
        for (int32_t e = 0; e < dh; ++e) {
            double acc = 0.0;
            for (int32_t j = 0; j < L; ++j) acc += p[j] * v[(int64_t)j * dh + e];
            oi[e] = rnd(acc, bf16);
        }
        free(p);
    }
    if (prob_check) {
        if (worst_sum > prob_check[0]) prob_check[0] = worst_sum;
        if (worst_leak > prob_check[1]) prob_check[1] = worst_leak;
    }
    free(ctx); free(chosen); free(active); free(M);
}

/* membership mask [L] of one sample's key sample (entries outside [0, L) are ignored) */
static uint8_t *sample_mask(const int32_t *sample_idx, int32_t n_sample, int32_t L)
{
    uint8_t *m = (uint8_t *)calloc((size_t)L, 1);
    for (int32_t r = 0; r < n_sample; ++r)
        if (sample_idx[r] >= 0 && sample_idx[r] < L) m[sample_idx[r]] = 1;
    return m;
}

int32_t orc_sparse_gqa(int32_t B, int32_t nH, int32_t nG, int32_t L, int32_t dh,
                       const double *Q, const double *K, const double *V,
                       const int32_t *head_group, const int32_t *head_group_b,
                       const uint8_t *key_valid, const int32_t *sample_idx, int32_t n_sample,
                       int32_t U, const int32_t *forced_sel,
                       int32_t bf16, double *O, double *score, int32_t *sel,
                       double *prob_check)
{
    if (B < 0 || nH < 1 || nG < 1 || L < 1 || dh < 1 || U < 0) return -1;
    if (prob_check) { prob_check[0] = 0.0; prob_check[1] = 0.0; }
    double *o_tmp = O ? NULL : (double *)malloc(sizeof(double) * (size_t)L * dh);
    for (int32_t b = 0; b < B; ++b) {
        const uint8_t *valid = key_valid ? key_valid + (int64_t)b * L : NULL;
        if (valid) {
            int32_t n = 0;
            for (int32_t j = 0; j < L; ++j) n += valid[j] != 0;
            if (n == 0) { free(o_tmp); return -1; }
        }
        uint8_t *skeys = sample_idx ? sample_mask(sample_idx + (int64_t)b * n_sample, n_sample, L) : NULL;
        for (int32_t h = 0; h < nH; ++h) {
            const int32_t g = head_group_b ? head_group_b[(int64_t)b * nH + h] : head_group[h];
            if (g < 0 || g >= nG) { free(o_tmp); free(skeys); return -1; }
            const int64_t bh = (int64_t)b * nH + h;
            sgqa_one_head(L, dh, Q + bh * L * dh, K + ((int64_t)b * nG + g) * L * dh,
                          V + ((int64_t)b * nG + g) * L * dh, valid, skeys, U,
                          forced_sel ? forced_sel + bh * U : NULL, bf16,
                          O ? O + (int64_t)b * L * nH * dh + (int64_t)h * dh : o_tmp,
                          O ? (int64_t)nH * dh : dh,
                          score ? score + bh * L : NULL, sel ? sel + bh * U : NULL,
                          prob_check);
        }
        free(skeys);
    }
    free(o_tmp);
    return 0;
}

/* ---- FFN ----------------------------------------------------------------- */
static double activation(double z, int32_t act)
{
    if (act == 1) return 0.5 * z * (1.0 + erf(z / sqrt(2.0)));   /* erf-GELU */
    return z > 0.0 ? z : 0.0;                                      /* ReLU */
}

/* bf16: rounding of the stored intermediates (LN output, hidden);
 * out_bf16: rounding of y itself */
static void ffn_core(const orc_layer *w, const double *x, int64_t rows, int32_t act,
                     double eps, int32_t pre_ln, int32_t add_residual, int32_t bf16,
                     int32_t out_bf16, double *y)
{
    const int32_t d = w->d, F = w->F;
    double *xn = (double *)malloc(sizeof(double) * (size_t)rows * d);
    double *hid = (double *)malloc(sizeof(double) * (size_t)rows * F);
    if (pre_ln) orc_layernorm(x, rows, d, w->ln2_g, w->ln2_b, eps, bf16, xn);
    else memcpy(xn, x, sizeof(double) * (size_t)rows * d);

    /* hidden = act(xn W1^T + b1), removed channels are exactly zero */
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int32_t f = 0; f < F; ++f) {
            if (w->ffn_mask && !w->ffn_mask[f]) { hid[r * F + f] = 0.0; continue; }
            double acc = 0.0;
            for (int32_t k = 0; k < d; ++k) acc += xn[r * d + k] * w->W1[(int64_t)f * d + k];
            if (w->b1) acc += w->b1[f];
            hid[r * F + f] = rnd(activation(acc, act), bf16);
        }
    }
    /* y = x + hidden W2 + b2 */
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int32_t n = 0; n < d; ++n) {
            double acc = 0.0;
            for (int32_t f = 0; f < F; ++f) {
                if (w->ffn_mask && !w->ffn_mask[f]) continue;
                acc += hid[r * F + f] * w->W2[(int64_t)f * d + n];
            }
            if (w->b2) acc += w->b2[n];
            if (add_residual) acc += x[r * d + n];
            y[r * d + n] = rnd(acc, out_bf16);
        }
    }
    free(hid); free(xn);
}

void orc_pruned_ffn(const orc_layer *w, const double *x, int64_t rows, int32_t act,
                    double eps, int32_t pre_ln, int32_t add_residual, int32_t bf16,
                    double *y)
{
    ffn_core(w, x, rows, act, eps, pre_ln, add_residual, bf16, bf16, y);
}

/* ---- FP16 (IEEE binary16) weight storage ---------------------------------- */
double orc_f16_decode(uint16_t bits)
{
    const int sign = bits >> 15, e = (bits >> 10) & 31, m = bits & 1023;
    double v;
    if (e == 31) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m, -24);               /* subnormal: m * 2^-10 * 2^-14 */
    else v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return sign ? -v : v;
}

void orc_dequant_f16(const uint16_t *q, int64_t n, int32_t bf16, double *out)
{
    for (int64_t i = 0; i < n; ++i) {
        const double w = orc_f16_decode(q[i]);                /* exact in fp32 as well */
        out[i] = rnd(w, bf16);
    }
}

/* ---- FP8 arithmetic (W8A8) for the pruned FFN ------------------------------ */
uint8_t orc_fp8_e4m3_encode(float t)
{
    if (isnan(t)) return 0x7F;
    const uint8_t sign = signbit(t) ? 0x80 : 0x00;
    const double a = fabs((double)t);
    if (a > 448.0) return sign | 0x7E;                        /* saturate (also infinities) */
    if (a < ldexp(1.0, -6)) {
        /* subnormal range, spacing 2^-9; 8 * 2^-9 is the smallest normal value, code 0x08 */
        return sign | (uint8_t)nearbyint(ldexp(a, 9));
    }
    int e;
    (void)frexp(a, &e);                                       /* a = 1.x * 2^(e-1) */
    int E = e - 1;
    int q = (int)nearbyint(ldexp(a, 3 - E));                  /* 8..16, ties to even */
    if (q == 16) { q = 8; ++E; }
    return sign | (uint8_t)(((E + 7) << 3) | (q - 8));
}

void orc_quantize_fp8(const float *x, int64_t n, float scale, uint8_t *codes)
{
    const volatile float r = 1.0f / scale;                    /* volatile: rounded to fp32 here */
    for (int64_t i = 0; i < n; ++i) {
        const volatile float t = x[i] * r;
        codes[i] = orc_fp8_e4m3_encode(t);
    }
}

void orc_pruned_ffn_fp8(int32_t d, int32_t F, const uint8_t *W1q, float s1, const double *b1,
                        const uint8_t *W2q, float s2, const double *b2, const double *ln_g,
                        const double *ln_b, const uint8_t *ffn_mask, float sx, float sh,
                        const double *x, int64_t rows, int32_t act, double eps, int32_t pre_ln,
                        int32_t add_residual, int32_t bf16, const uint8_t *xq_forced,
                        const uint8_t *hq_forced, double *y, uint8_t *xq_out, uint8_t *hq_out, double *z_out)
{
    double *xn = (double *)malloc(sizeof(double) * (size_t)rows * d);
    float *t32 = (float *)malloc(sizeof(float) * (size_t)rows * (d > F ? d : F));
    uint8_t *xq = (uint8_t *)malloc((size_t)rows * d);
    uint8_t *hq = (uint8_t *)malloc((size_t)rows * F);
    if (pre_ln) orc_layernorm(x, rows, d, ln_g, ln_b, eps, 0, xn);
    else memcpy(xn, x, sizeof(double) * (size_t)rows * d);
    for (int64_t i = 0; i < rows * d; ++i) t32[i] = (float)xn[i];
    orc_quantize_fp8(t32, rows * d, sx, xq);
    if (xq_forced) memcpy(xq, xq_forced, (size_t)rows * d);
    const volatile float os1 = sx * s1, os2 = sh * s2;        /* fp32 products */

#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int32_t f = 0; f < F; ++f) {
            if (ffn_mask && !ffn_mask[f]) { t32[r * F + f] = 0.f; if (z_out) z_out[r * F + f] = 0.0; continue; }
            double acc = 0.0;                                 /* products and sum exact in double */
            for (int32_t k = 0; k < d; ++k)
                acc += orc_fp8_e4m3_decode(xq[r * d + k]) * orc_fp8_e4m3_decode(W1q[(int64_t)f * d + k]);
            acc = acc * (double)os1 + (b1 ? b1[f] : 0.0);
            if (z_out) z_out[r * F + f] = (double)(float)acc;
            t32[r * F + f] = (float)activation((double)(float)acc, act);
        }
    orc_quantize_fp8(t32, rows * F, sh, hq);
    if (hq_forced) memcpy(hq, hq_forced, (size_t)rows * F);
    if (ffn_mask)
        for (int64_t r = 0; r < rows; ++r)
            for (int32_t f = 0; f < F; ++f)
                if (!ffn_mask[f]) hq[r * F + f] = 0;

#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int32_t n = 0; n < d; ++n) {
            double acc = 0.0;
            for (int32_t f = 0; f < F; ++f) {
                if (ffn_mask && !ffn_mask[f]) continue;
                acc += orc_fp8_e4m3_decode(hq[r * F + f]) * orc_fp8_e4m3_decode(W2q[(int64_t)f * d + n]);
            }
            acc = acc * (double)os2 + (b2 ? b2[n] : 0.0);
            if (add_residual) acc += x[r * d + n];
            y[r * d + n] = rnd(acc, bf16);
        }
    if (xq_out) memcpy(xq_out, xq, (size_t)rows * d);
    if (hq_out) memcpy(hq_out, hq, (size_t)rows * F);
    free(hq); free(xq); free(t32); free(xn);
}

/* ---- Sparse-MoE FFN ------------------------------------------------------- */
int32_t orc_moe_ffn(const orc_moe *m, const double *x, int64_t rows, int32_t act, double eps,
                    int32_t pre_ln, int32_t add_residual, int32_t bf16,
                    const int32_t *forced_route, double *y, int32_t *route_out,
                    double *weight_out, double *logit_out)
{
    const int32_t d = m->d, F = m->F, E = m->E, k = m->k;
    if (d < 1 || F < 1 || E < 1 || k < 1 || k > E || rows < 0) return -1;
    double *xn = (double *)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * d);
    if (pre_ln) orc_layernorm(x, rows, d, m->ln_g, m->ln_b, eps, bf16, xn);
    else memcpy(xn, x, sizeof(double) * (size_t)rows * d);
    int32_t rc = 0;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = xn + r * d;
        double *logit = (double *)malloc(sizeof(double) * (size_t)E);
        qscore *qs = (qscore *)malloc(sizeof(qscore) * (size_t)E);
        int32_t *pick = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
        double *hid = (double *)malloc(sizeof(double) * (size_t)F);
        for (int32_t e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int32_t c = 0; c < d; ++c) acc += xr[c] * m->Wr[(int64_t)e * d + c];
            if (m->br) acc += m->br[e];
            logit[e] = acc;
            if (logit_out) logit_out[r * E + e] = acc;
            qs[e].m = (float)acc;
            qs[e].i = e;
        }
        int bad = 0;
        if (forced_route) {
            for (int32_t s = 0; s < k; ++s) {
                pick[s] = forced_route[r * k + s];
                if (pick[s] < 0 || pick[s] >= E) bad = 1;
                for (int32_t t = 0; t < s; ++t) if (pick[t] == pick[s]) bad = 1;
            }
        } else {
            qsort(qs, (size_t)E, sizeof(qscore), by_m_desc_index_asc);
            for (int32_t s = 0; s < k; ++s) pick[s] = qs[s].i;
        }
        if (bad) {
#pragma omp atomic write
            rc = -1;
        } else {
            /* softmax over the chosen logits */
            double mx = -INFINITY, den = 0.0;
            for (int32_t s = 0; s < k; ++s) if (logit[pick[s]] > mx) mx = logit[pick[s]];
            for (int32_t s = 0; s < k; ++s) den += exp(logit[pick[s]] - mx);
            for (int32_t n = 0; n < d; ++n) y[r * d + n] = add_residual ? x[r * d + n] : 0.0;
            for (int32_t s = 0; s < k; ++s) {
                const int32_t e = pick[s];
                const double pe = exp(logit[e] - mx) / den;
                if (route_out) route_out[r * k + s] = e;
                if (weight_out) weight_out[r * k + s] = pe;
                const double *W1 = m->W1 + (int64_t)e * F * d, *W2 = m->W2 + (int64_t)e * F * d;
                for (int32_t f = 0; f < F; ++f) {
                    if (m->ffn_mask && !m->ffn_mask[(int64_t)e * F + f]) { hid[f] = 0.0; continue; }
                    double acc = 0.0;
                    for (int32_t c = 0; c < d; ++c) acc += xr[c] * W1[(int64_t)f * d + c];
                    if (m->b1) acc += m->b1[(int64_t)e * F + f];
                    hid[f] = rnd(activation(acc, act), bf16);
                }
                for (int32_t n = 0; n < d; ++n) {
                    double acc = 0.0;
                    for (int32_t f = 0; f < F; ++f) {
                        if (m->ffn_mask && !m->ffn_mask[(int64_t)e * F + f]) continue;
                        acc += hid[f] * W2[(int64_t)f * d + n];
                    }
                    if (m->b2) acc += m->b2[(int64_t)e * d + n];
                    y[r * d + n] += pe * acc;
                }
            }
            for (int32_t n = 0; n < d; ++n) y[r * d + n] = rnd(y[r * d + n], bf16);
        }
        free(hid); free(pick); free(qs); free(logit);
    }
    free(xn);
    return rc;
}

/* ---- encoder stack ------------------------------------------------------- */
int32_t orc_encoder_forward(int32_t B, int32_t L, int32_t nl, int32_t P,
                            const orc_layer *layers, const int32_t *pattern_id,
                            const uint8_t *key_valid, const int32_t *sample_idx, int32_t n_sample,
                            int32_t U, int32_t act, double eps,
                            const int32_t *forced_sel, int32_t nHmax,
                            const double *final_g, const double *final_b, int32_t bf16,
                            const double *x, double *y, int32_t *sel_out, double *score_out)
{
    return orc_encoder_forward_fp8ffn(B, L, nl, P, layers, NULL, pattern_id, key_valid, sample_idx, n_sample, U,
                                      act, eps, forced_sel, nHmax, final_g, final_b, bf16, NULL, NULL, 0, 0, x, y,
                                      sel_out, score_out, NULL, NULL);
}

int32_t orc_encoder_forward_fp8ffn(int32_t B, int32_t L, int32_t nl, int32_t P,
                                   const orc_layer *layers, const orc_ffn8 *ffn8, const int32_t *pattern_id,
                                   const uint8_t *key_valid, const int32_t *sample_idx, int32_t n_sample,
                                   int32_t U, int32_t act, double eps,
                                   const int32_t *forced_sel, int32_t nHmax,
                                   const double *final_g, const double *final_b, int32_t bf16,
                                   const uint8_t *xq_forced, const uint8_t *hq_forced,
                                   int32_t n_forced_x, int32_t n_forced_h,
                                   const double *x, double *y, int32_t *sel_out, double *score_out,
                                   uint8_t *xq_out, uint8_t *hq_out)
{
    orc_fp8_io io;
    memset(&io, 0, sizeof io);
    io.xq_forced = xq_forced; io.hq_forced = hq_forced; io.n_forced_x = n_forced_x; io.n_forced_h = n_forced_h;
    io.xq_out = xq_out; io.hq_out = hq_out;
    return orc_encoder_forward_fp8(B, L, nl, P, layers, ffn8, NULL, pattern_id, key_valid, sample_idx, n_sample, U,
                                   act, eps, forced_sel, nHmax, final_g, final_b, bf16, &io, x, y, sel_out, score_out);
}

/* acc[r, n] = (sum_k code(a[r,k]) * code(W[unit0+n, k])) * os + b[unit0+n]: the products of two E4M3 values and their
 * sum are exact in double */
static void project_units8(const uint8_t *aq, int64_t rows, int32_t d, const uint8_t *Wq8, double os,
                           const double *b, int32_t unit0, int32_t n_units, int32_t bf16, double *y,
                           int64_t out_stride, int32_t out0)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int32_t n = 0; n < n_units; ++n) {
            const uint8_t *wn = Wq8 + (int64_t)(unit0 + n) * d;
            double acc = 0.0;
            for (int32_t k = 0; k < d; ++k) acc += orc_fp8_e4m3_decode(aq[r * d + k]) * orc_fp8_e4m3_decode(wn[k]);
            acc = acc * os + (b ? b[unit0 + n] : 0.0);
            y[r * out_stride + out0 + n] = rnd(acc, bf16);
        }
}

int32_t orc_encoder_forward_fp8(int32_t B, int32_t L, int32_t nl, int32_t P,
                                const orc_layer *layers, const orc_ffn8 *ffn8, const orc_proj8 *proj8,
                                const int32_t *pattern_id, const uint8_t *key_valid, const int32_t *sample_idx,
                                int32_t n_sample, int32_t U, int32_t act, double eps,
                                const int32_t *forced_sel, int32_t nHmax,
                                const double *final_g, const double *final_b, int32_t bf16,
                                const orc_fp8_io *io, const double *x, double *y, int32_t *sel_out, double *score_out)
{
    orc_fp8_io none;
    memset(&none, 0, sizeof none);
    if (!io) io = &none;
    const uint8_t *xq_forced = io->xq_forced, *hq_forced = io->hq_forced;
    const int32_t n_forced_x = io->n_forced_x, n_forced_h = io->n_forced_h;
    uint8_t *xq_out = io->xq_out, *hq_out = io->hq_out;
    if (B < 0 || L < 1 || nl < 1 || P < 1 || U < 0) return -1;
    const int32_t d = layers[0].d;
    const int64_t Ld = (int64_t)L * d;
    double *cur = (double *)malloc(sizeof(double) * (size_t)Ld);
    double *xn = (double *)malloc(sizeof(double) * (size_t)Ld);
    int32_t rc = 0;

    for (int32_t b = 0; b < B && rc == 0; ++b) {
        const uint8_t *valid = key_valid ? key_valid + (int64_t)b * L : NULL;
        if (valid) {
            int32_t n = 0;
            for (int32_t j = 0; j < L; ++j) n += valid[j] != 0;
            if (n == 0) { rc = -1; break; }
        }
        const int32_t p = pattern_id ? pattern_id[b] : 0;
        if (p < 0 || p >= P) { rc = -1; break; }
        memcpy(cur, x + b * Ld, sizeof(double) * (size_t)Ld);
        uint8_t *skeys = sample_idx ? sample_mask(sample_idx + (int64_t)b * n_sample, n_sample, L) : NULL;

        for (int32_t l = 0; l < nl; ++l) {
            const orc_layer *w = &layers[(int64_t)l * P + p];
            const int32_t nH = w->nH, nG = w->nG, dh = w->dh;
            if (w->d != d || nH > nHmax) { rc = -1; break; }
            double *Q = (double *)calloc((size_t)nH * L * dh, sizeof(double));
            double *Kg = (double *)calloc((size_t)nG * L * dh, sizeof(double));
            double *Vg = (double *)calloc((size_t)nG * L * dh, sizeof(double));
            double *O = (double *)calloc((size_t)L * nH * dh, sizeof(double));

            const orc_proj8 *pj = proj8 ? &proj8[l] : NULL;
            const int64_t blk = (int64_t)l * B + b;
            uint8_t *aq = NULL;
            if (pj) {
                /* FP8 arithmetic for the projections: LN1(x) in fp32 -> E4M3 codes with the layer's scale */
                orc_layernorm(cur, L, d, w->ln1_g, w->ln1_b, eps, 0, xn);
                float *t32 = (float *)malloc(sizeof(float) * (size_t)Ld);
                aq = (uint8_t *)malloc((size_t)Ld);
                for (int64_t t = 0; t < Ld; ++t) t32[t] = (float)xn[t];
                orc_quantize_fp8(t32, Ld, pj->sx1, aq);
                if (io->aq_forced && l < io->n_forced_a) memcpy(aq, io->aq_forced + blk * Ld, (size_t)Ld);
                if (io->aq_out) memcpy(io->aq_out + blk * Ld, aq, (size_t)Ld);
                free(t32);
            } else
            orc_layernorm(cur, L, d, w->ln1_g, w->ln1_b, eps, bf16, xn);
            const volatile float os_qkv = pj ? pj->sx1 * pj->s_qkv : 0.f;      /* fp32 product */

            /* per-head Q, per-group K/V (only for units that survive) */
            for (int32_t h = 0; h < nH; ++h) {
                if (w->head_mask && !w->head_mask[h]) continue;
                if (pj) project_units8(aq, L, d, pj->Wq8, (double)os_qkv, w->bq, h * dh, dh, bf16, Q + (int64_t)h * L * dh, dh, 0);
                else
                project_units(xn, L, d, w->Wq, w->bq, h * dh, dh, bf16, Q + (int64_t)h * L * dh, dh, 0);
            }
            for (int32_t g = 0; g < nG; ++g) {
                int used = 0;
                for (int32_t h = 0; h < nH; ++h)
                    if ((!w->head_mask || w->head_mask[h]) && w->head_group[h] == g) used = 1;
                if (!used) continue;
                if (pj) {
                    project_units8(aq, L, d, pj->Wk8, (double)os_qkv, w->bk, g * dh, dh, bf16, Kg + (int64_t)g * L * dh, dh, 0);
                    project_units8(aq, L, d, pj->Wv8, (double)os_qkv, w->bv, g * dh, dh, bf16, Vg + (int64_t)g * L * dh, dh, 0);
                    continue;
                }
                project_units(xn, L, d, w->Wk, w->bk, g * dh, dh, bf16, Kg + (int64_t)g * L * dh, dh, 0);
                project_units(xn, L, d, w->Wv, w->bv, g * dh, dh, bf16, Vg + (int64_t)g * L * dh, dh, 0);
            }
            free(aq);

            /* SentryAttend per surviving head; a removed head's output is 0 */
            for (int32_t h = 0; h < nH; ++h) {
                if (w->head_mask && !w->head_mask[h]) continue;
                const int32_t g = w->head_group[h];
                const int64_t slot = (((int64_t)l * B + b) * nHmax + h);
                sgqa_one_head(L, dh, Q + (int64_t)h * L * dh, Kg + (int64_t)g * L * dh,
                              Vg + (int64_t)g * L * dh, valid, skeys, U,
                              forced_sel ? forced_sel + slot * U : NULL, bf16,
                              O + (int64_t)h * dh, (int64_t)nH * dh,
                              score_out ? score_out + slot * L : NULL,
                              sel_out ? sel_out + slot * U : NULL, NULL);
            }

            if (pj) {
                /* x <- x + (codes(O) . codes(Wo)) * (sa * so) + bo: the attention output is quantised with the
                 * layer's scale; a removed head's output is 0, code 0 */
                const int64_t no = (int64_t)L * nH * dh;
                float *t32 = (float *)malloc(sizeof(float) * (size_t)no);
                uint8_t *oq = (uint8_t *)malloc((size_t)no);
                for (int64_t t = 0; t < no; ++t) t32[t] = (float)O[t];
                orc_quantize_fp8(t32, no, pj->sa, oq);
                if (io->oq_forced && l < io->n_forced_o) memcpy(oq, io->oq_forced + blk * no, (size_t)no);
                for (int32_t i = 0; i < L; ++i)
                    for (int32_t h = 0; h < nH; ++h)
                        if (w->head_mask && !w->head_mask[h]) memset(oq + ((int64_t)i * nH + h) * dh, 0, (size_t)dh);
                if (io->oq_out) memcpy(io->oq_out + blk * no, oq, (size_t)no);
                const volatile float os_o = pj->sa * pj->so;
#pragma omp parallel for schedule(static)
                for (int32_t i = 0; i < L; ++i)
                    for (int32_t n = 0; n < d; ++n) {
                        double acc = 0.0;
                        for (int32_t c = 0; c < nH * dh; ++c)
                            acc += orc_fp8_e4m3_decode(oq[(int64_t)i * nH * dh + c]) *
                                   orc_fp8_e4m3_decode(pj->Wo8[(int64_t)c * d + n]);
                        acc = acc * (double)os_o + (w->bo ? w->bo[n] : 0.0);
                        xn[(int64_t)i * d + n] = cur[(int64_t)i * d + n] + acc;
                    }
                free(oq); free(t32);
            } else {
                /* x <- x + O Wo + bo  (rows of Wo belonging to removed heads never enter) */
#pragma omp parallel for schedule(static)
                for (int32_t i = 0; i < L; ++i) {
                    for (int32_t n = 0; n < d; ++n) {
                        double acc = 0.0;
                        for (int32_t h = 0; h < nH; ++h) {
                            if (w->head_mask && !w->head_mask[h]) continue;
                            for (int32_t e = 0; e < dh; ++e)
                                acc += O[(int64_t)i * nH * dh + h * dh + e] *
                                       w->Wo[((int64_t)h * dh + e) * d + n];
                        }
                        if (w->bo) acc += w->bo[n];
                        xn[(int64_t)i * d + n] = cur[(int64_t)i * d + n] + acc;   /* stream stays unrounded */
                    }
                }
            }
            memcpy(cur, xn, sizeof(double) * (size_t)Ld);

            /* x <- x + FFN(LN2(x)) */
            if (ffn8) {
                /* the FFN of this layer in FP8 arithmetic; the stream stays unrounded */
                const orc_ffn8 *f = &ffn8[l];
                orc_pruned_ffn_fp8(d, w->F, f->W1q, f->s1, w->b1, f->W2q, f->s2, w->b2, w->ln2_g, w->ln2_b,
                                   w->ffn_mask, f->sx, f->sh, cur, L, act, eps, 1, 1, 0,
                                   xq_forced && l < n_forced_x ? xq_forced + blk * L * d : NULL,
                                   hq_forced && l < n_forced_h ? hq_forced + blk * L * w->F : NULL, xn,
                                   xq_out ? xq_out + blk * L * d : NULL, hq_out ? hq_out + blk * L * w->F : NULL,
                                   NULL);
            } else
            ffn_core(w, cur, L, act, eps, 1, 1, bf16, 0, xn);
            memcpy(cur, xn, sizeof(double) * (size_t)Ld);

            free(O); free(Vg); free(Kg); free(Q);
        }
        free(skeys);
        if (rc) break;
        if (final_g || final_b) {
            orc_layernorm(cur, L, d, final_g, final_b, eps, bf16, y + b * Ld);
        } else {
            for (int64_t t = 0; t < Ld; ++t) y[b * Ld + t] = rnd(cur[t], bf16);   /* the output is a stored tensor */
        }
    }
    free(xn); free(cur);
    return rc;
}
