// Descriptor handling, error reporting, pruned_ffn_forward and encoder_forward
// (the pre-norm layer stack around SentryAttend and the pruned FFN; Sec. 4.4
// and Sec. 4.5 of the paper).
#include <algorithm>
#include <math.h>
#include <string.h>

#include "attention.hpp"
#include "gemm.hpp"

namespace sf {

char *err_buf()
{
    static thread_local char buf[512] = "";
    return buf;
}

int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(err_buf(), 512, fmt, ap);
    va_end(ap);
    return code;
}

int32_t check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SF_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return SF_OK;
}

// ---- per-kernel event timing ----------------------------------------------------
static struct {
    int kernel_class = -1;
    int cap = 0, n = 0;
    hipEvent_t *start = nullptr, *stop = nullptr;
} g_prof;

ProfScope::ProfScope(int kernel_class, hipStream_t s) : slot(-1), st(s)
{
    if (g_prof.kernel_class == kernel_class && g_prof.n < g_prof.cap) {
        slot = g_prof.n++;
        (void)hipEventRecord(g_prof.start[slot], st);
    }
}

ProfScope::~ProfScope()
{
    if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], st);
}

int32_t read_desc(const sf_desc *desc, Dims &D)
{
    if (!desc) return fail(SF_ERR_INVALID_ARG, "descriptor is NULL");
    if (desc->struct_size != sizeof(sf_desc))
        return fail(SF_ERR_INVALID_ARG, "descriptor struct_size %u, expected %zu", desc->struct_size, sizeof(sf_desc));
    D.B = desc->B; D.L = desc->L; D.d = desc->d_model; D.Hq = desc->Hq; D.Hk = desc->Hk; D.dh = desc->dh;
    D.F = desc->d_ff; D.nl = desc->n_layers; D.P = desc->P; D.dtype = desc->dtype; D.act = desc->act;
    D.flags = desc->flags;
    D.eps = desc->ln_eps > 0.f ? desc->ln_eps : 1e-5f;
    D.ffn_pad = desc->ffn_pad > 0 ? desc->ffn_pad : 64;
    D.n_sample = desc->n_sample;
    if (D.n_sample < 0 || D.n_sample > 4096) return fail(SF_ERR_INVALID_ARG, "descriptor: n_sample must be in [0, 4096]");
    if (D.B < 1 || D.L < 1 || D.d < 1 || D.Hq < 1 || D.Hk < 1 || D.dh < 1 || D.F < 1 || D.nl < 1 || D.P < 1)
        return fail(SF_ERR_INVALID_ARG, "descriptor: sizes must be positive");
    if (D.Hq % D.Hk) return fail(SF_ERR_INVALID_ARG, "descriptor: Hq %% Hk != 0");
    if (D.dtype == SF_DTYPE_16_OTHER)
        return fail(SF_ERR_UNSUPPORTED, "descriptor: this build of the library computes 16-bit models in %s; %s",
                    SF_DTYPE_16 == SF_F16 ? "IEEE binary16 (SF_F16)" : "bfloat16 (SF_BF16)",
                    SF_DTYPE_16 == SF_F16 ? "SF_BF16 models take libsentryfuse.so" : "SF_F16 models take libsentryfuse_f16.so");
    if (D.dtype != SF_F32 && D.dtype != SF_DTYPE_16) return fail(SF_ERR_UNSUPPORTED, "descriptor: unknown dtype");
    if (D.dtype == SF_DTYPE_16) D.dtype = SF_BF16;      // from here on SF_BF16 stands for "the 16-bit type of this build"
    if (D.act != SF_RELU && D.act != SF_GELU_ERF) return fail(SF_ERR_UNSUPPORTED, "descriptor: unknown activation");
    if (D.ffn_pad % 64) return fail(SF_ERR_SHAPE, "descriptor: ffn_pad must be a multiple of 64");
    if (D.dtype == SF_BF16 && (D.d % 8 || D.dh % 8))
        return fail(SF_ERR_SHAPE, "descriptor: bf16 needs d_model and dh to be multiples of 8");
    if ((int64_t)D.B * D.L > (int64_t)1 << 30) return fail(SF_ERR_SHAPE, "descriptor: B*L too large");
    const int c = desc->c_factor > 0 ? desc->c_factor : 5;
    if (desc->U_override >= 0) {
        D.U = desc->U_override < D.L ? desc->U_override : D.L;
    } else {
        const double u = (double)c * ceil(log((double)D.L));      // natural log, Sec. 4.4 worked example
        D.U = u < (double)D.L ? (int)u : D.L;
    }
    return SF_OK;
}

static int gemm_act(int act) { return act == SF_GELU_ERF ? ACT_GELU : ACT_RELU; }

// ---- FFN ------------------------------------------------------------------------
struct FfnWs { void *xn, *hid; size_t bytes; };
static FfnWs ffn_ws(const Dims &D, int Fp, bool pre_ln, void *ws)
{
    Carver c(ws);
    FfnWs w{};
    const size_t es = elem_size(D.dtype), rows = (size_t)D.B * D.L;
    w.xn = pre_ln ? c.take<char>(rows * D.d * es) : nullptr;
    w.hid = c.take<char>(rows * Fp * es);
    w.bytes = c.off;
    return w;
}

// x_f32 / y_f32: X / Y hold fp32 although the model dtype is bf16 (the
// encoder's residual stream).  With x_f32, pre_ln is required (the GEMM reads bf16).
static int32_t ffn_forward(const Dims &D, const sf_compact_layer &ly, const void *X, bool x_f32,
                           const int32_t *pattern_id, bool pre_ln, bool add_residual, void *Y, bool y_f32,
                           void *xn, void *hid, hipStream_t st, bool xn_ready = false)
{
    const int Fp = (int)align_up(ly.k_ffn, D.ffn_pad);
    const void *in = X;
    if (xn_ready) {
        in = xn;                              // LN2(X) is already there (written together with X)
    } else if (pre_ln) {
        layernorm(D.dtype, x_f32, X, ly.ln2_g, ly.ln2_b, D.eps, (int64_t)D.B * D.L, D.d, xn, st);
        in = xn;
    }
    GemmArgs g{};
    g.A = in; g.lda = D.d; g.W = ly.W1; g.ldw = D.d; g.w_pstride = (int64_t)Fp * D.d;
    g.bias = ly.b1; g.bias_pstride = Fp; g.pattern_id = pattern_id;
    g.B = D.B; g.L = D.L; g.N = Fp; g.K = D.d; g.epi = EPI_ROWMAJOR; g.act = gemm_act(D.act);
    g.C = hid; g.ldc = Fp;
    if (int32_t rc = gemm(D.dtype, g, st)) return rc;

    GemmArgs h{};
    h.A = hid; h.lda = Fp; h.W = ly.W2T; h.ldw = Fp; h.w_pstride = (int64_t)D.d * Fp;
    h.bias = ly.b2; h.bias_pstride = 0; h.pattern_id = pattern_id;
    h.B = D.B; h.L = D.L; h.N = D.d; h.K = Fp; h.epi = EPI_ROWMAJOR; h.act = ACT_NONE;
    h.R = add_residual ? X : nullptr; h.ldr = D.d; h.r_f32 = x_f32;
    h.C = Y; h.ldc = D.d; h.c_f32 = y_f32;
    return gemm(D.dtype, h, st);
}

// ---- encoder ----------------------------------------------------------------------
struct EncWs {
    void *xn, *qkv, *vt, *att, *x1, *x2, *hid, *attn_ws;     // x1, x2: the fp32 residual stream
    // output projection of the active rows only (lazy_proj.hip): compact rows, their projection, row maps, c_b
    void *lz_A; float *lz_C, *lz_c; int32_t *lz_arow, *lz_pos, *lz_n, *lz_cnt, *lz_blk; int lz_cap;
    uint8_t *lz_A8;                                          // ... and of the compact rows
    uint8_t *oq;                                             // projections in FP8 arithmetic: codes of the attention output
    size_t attn_ws_bytes, bytes;
    int kh_max, Fp_max, Lp;
};

static AttnArgs enc_attn_args(const Dims &D, int kh)
{
    AttnArgs a{};
    a.B = D.B; a.nH = kh; a.nG = D.Hk; a.L = D.L; a.dh = D.dh; a.U = D.U; a.n_sample = D.n_sample;
    a.v_transposed = D.dtype == SF_BF16;
    return a;
}

// rows_tok > 0: the token-major buffers hold that many rows (samples packed back to back) instead of B*L, and Q, K
// and V are all token-major (V is transposed by a pass of its own)
static int32_t enc_ws(const Dims &D, const sf_compact_layer *layers, void *ws, EncWs &w, bool proj8 = false,
                      size_t rows_tok = 0)
{
    w = EncWs{};
    int kh_max = 0, kf_max = 0;
    for (int l = 0; l < D.nl; ++l) {
        if (layers[l].k_head < 1 || layers[l].k_head > D.Hq || layers[l].k_ffn < 1 || layers[l].k_ffn > D.F)
            return fail(SF_ERR_INVALID_ARG, "encoder: keep counts of layer %d out of range", l);
        if (layers[l].k_head > kh_max) kh_max = layers[l].k_head;
        if (layers[l].k_ffn > kf_max) kf_max = layers[l].k_ffn;
    }
    w.kh_max = kh_max;
    w.Fp_max = (int)align_up(kf_max, D.ffn_pad);
    w.Lp = (int)align_up(D.L, 8);
    const size_t es = elem_size(D.dtype), rows = rows_tok ? rows_tok : (size_t)D.B * D.L;
    const bool bf = D.dtype == SF_BF16;
    if (rows_tok) proj8 = true;              // same buffer shapes: Q, K, V token-major and a transposed copy of V
    Carver c(ws);
    w.xn = c.take<char>(rows * D.d * es);
    // bf16: Q and K token-major, V transposed [B,Hk,dh,Lp]; fp32: Q, K, V token-major
    // (projections in FP8 arithmetic: the GEMM writes V token-major too, a second pass transposes it)
    w.qkv = c.take<char>(rows * (size_t)(kh_max + (bf && !proj8 ? 1 : 2) * D.Hk) * D.dh * es);
    w.vt = bf ? c.take<char>((size_t)D.B * D.Hk * D.dh * w.Lp * es) : nullptr;
    w.att = c.take<char>(rows * (size_t)kh_max * D.dh * es);
    w.x1 = c.take<float>(rows * D.d);
    w.x2 = D.nl > 1 || (D.flags & SF_FLAG_FINAL_LN) ? c.take<float>(rows * D.d) : nullptr;
    w.hid = c.take<char>(rows * (size_t)w.Fp_max * es);
    size_t amax = 0;
    for (int l = 0; l < D.nl; ++l) {
        const size_t b = attn_plan(D.dtype, enc_attn_args(D, layers[l].k_head), nullptr).bytes;
        if (b > amax) amax = b;
    }
    w.attn_ws_bytes = amax;
    w.attn_ws = c.take<char>(amax);
    const size_t Kp_max = align_up((size_t)kh_max * D.dh, 128);      // code rows are padded to the FP8 GEMM's K step
    w.oq = proj8 && !rows_tok ? c.take<uint8_t>(rows * Kp_max) : nullptr;
    w.lz_cap = bf && !rows_tok ? lazy_cap(D.L, kh_max, D.U, D.dh, D.d) : 0;
    if (w.lz_cap) {
        const size_t crow = (size_t)D.B * w.lz_cap;
        w.lz_A = c.take<char>(crow * kh_max * D.dh * es);
        w.lz_A8 = proj8 ? c.take<uint8_t>(crow * Kp_max) : nullptr;
        w.lz_C = c.take<float>(crow * D.d);
        w.lz_c = c.take<float>((size_t)D.B * D.d);
        w.lz_arow = c.take<int32_t>(crow);
        w.lz_pos = c.take<int32_t>(rows);
        w.lz_n = c.take<int32_t>(D.B);
        w.lz_cnt = c.take<int32_t>((size_t)D.B * ceil_div(D.L, 32));      // one bit per row: selected by some head
        w.lz_blk = c.take<int32_t>((size_t)D.B * (w.lz_cap / 128));
    }
    w.bytes = c.off;
    return SF_OK;
}

}  // namespace sf

using namespace sf;

extern "C" const char *sf_last_error(void) { return err_buf(); }

extern "C" int32_t sf_profile_begin(int32_t kernel_class, int32_t max_launches)
{
    if (g_prof.kernel_class >= 0) return fail(SF_ERR_INVALID_ARG, "profile: already profiling");
    if (kernel_class < 0 || kernel_class > SF_KERNEL_ATTEND || max_launches < 1 || max_launches > (1 << 20))
        return fail(SF_ERR_INVALID_ARG, "profile: bad kernel class or launch count");
    g_prof.start = new hipEvent_t[max_launches];
    g_prof.stop = new hipEvent_t[max_launches];
    for (int i = 0; i < max_launches; ++i) {
        if (hipEventCreate(&g_prof.start[i]) != hipSuccess || hipEventCreate(&g_prof.stop[i]) != hipSuccess)
            return fail(SF_ERR_HIP, "profile: hipEventCreate failed");
    }
    g_prof.cap = max_launches;
    g_prof.n = 0;
    g_prof.kernel_class = kernel_class;
    return SF_OK;
}

extern "C" int32_t sf_profile_end(int32_t *n_launches, float *total_ms, float *each_ms)
{
    if (g_prof.kernel_class < 0) return fail(SF_ERR_INVALID_ARG, "profile: not profiling");
    g_prof.kernel_class = -1;
    float sum = 0.f;
    int32_t rc = SF_OK;
    for (int i = 0; i < g_prof.n; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) != hipSuccess)
            rc = fail(SF_ERR_HIP, "profile: reading event %d failed", i);
        sum += ms;
        if (each_ms) each_ms[i] = ms;
    }
    for (int i = 0; i < g_prof.cap; ++i) { (void)hipEventDestroy(g_prof.start[i]); (void)hipEventDestroy(g_prof.stop[i]); }
    delete[] g_prof.start;
    delete[] g_prof.stop;
    if (n_launches) *n_launches = g_prof.n;
    if (total_ms) *total_ms = sum;
    g_prof.start = g_prof.stop = nullptr;
    g_prof.cap = g_prof.n = 0;
    return rc;
}

extern "C" int32_t sf_num_active(const sf_desc *desc)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    return D.U;
}

extern "C" int32_t sf_ffn_padded(const sf_desc *desc, int32_t k_ffn)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (k_ffn < 1 || k_ffn > D.F) return fail(SF_ERR_INVALID_ARG, "ffn_padded: k_ffn out of range");
    return (int32_t)align_up(k_ffn, D.ffn_pad);
}

extern "C" size_t sf_pruned_ffn_workspace_bytes(const sf_desc *desc, int32_t k_ffn)
{
    Dims D;
    if (read_desc(desc, D) || k_ffn < 1 || k_ffn > D.F) return 0;
    return ffn_ws(D, (int)align_up(k_ffn, D.ffn_pad), true, nullptr).bytes;
}

extern "C" int32_t sf_pruned_ffn_forward(const sf_desc *desc, const sf_compact_layer *ly, const void *X,
                                         const int32_t *pattern_id, int32_t pre_ln, int32_t add_residual,
                                         void *Y, void *workspace, size_t workspace_bytes, void *stream)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (!ly || !X || !Y) return fail(SF_ERR_INVALID_ARG, "pruned_ffn: NULL argument");
    if (X == Y) return fail(SF_ERR_INVALID_ARG, "pruned_ffn: Y may not alias X");
    if (ly->k_ffn < 1 || ly->k_ffn > D.F) return fail(SF_ERR_INVALID_ARG, "pruned_ffn: k_ffn out of range");
    if (!ly->W1 || !ly->W2T) return fail(SF_ERR_INVALID_ARG, "pruned_ffn: NULL weight pointer");
    if (D.P > 1 && !pattern_id) return fail(SF_ERR_INVALID_ARG, "pruned_ffn: pattern_id required when P > 1");
    const int Fp = (int)align_up(ly->k_ffn, D.ffn_pad);
    FfnWs w = ffn_ws(D, Fp, pre_ln != 0, workspace);
    if (!workspace || workspace_bytes < w.bytes || ((uintptr_t)workspace & 255))
        return fail(SF_ERR_WORKSPACE, "pruned_ffn: workspace of %zu bytes (256-byte aligned) required, got %zu",
                    w.bytes, workspace_bytes);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (int32_t rc = ffn_forward(D, *ly, X, false, pattern_id, pre_ln != 0, add_residual != 0, Y, false, w.xn,
                                 w.hid, st))
        return rc;
    return check_launch("pruned_ffn_forward");
}

extern "C" int32_t sf_active_projection_rows(const sf_desc *desc, int32_t k_head)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (k_head < 1 || k_head > D.Hq) return fail(SF_ERR_INVALID_ARG, "active_projection_rows: k_head out of range");
    return D.dtype == SF_BF16 ? lazy_cap(D.L, k_head, D.U, D.dh, D.d) : 0;
}

extern "C" size_t sf_encoder_workspace_bytes(const sf_desc *desc, const sf_compact_layer *layers)
{
    Dims D;
    EncWs w;
    if (read_desc(desc, D) || !layers || enc_ws(D, layers, nullptr, w)) return 0;
    return w.bytes;
}

static int32_t encoder_forward_impl(const sf_desc *desc, const sf_compact_layer *layers, const void *X,
                                    const int32_t *pattern_id, const uint8_t *key_valid,
                                    const int32_t *sample_idx, const int32_t *u_active, const void *final_g,
                                    const void *final_b, const int32_t *forced_sel,
                                    void *Y, int32_t *sel_out, float *score_out, void *workspace,
                                    size_t workspace_bytes, void *stream, const sf_ffn_fp8 *ffn8 = nullptr,
                                    uint8_t *xq_out = nullptr, uint8_t *hq_out = nullptr,
                                    const sf_proj_fp8 *proj8 = nullptr, uint8_t *aq_out = nullptr,
                                    uint8_t *oq_out = nullptr, const sf_token_pack_plan *pk = nullptr)
{
    Dims D;
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (pk && (ffn8 || proj8)) return fail(SF_ERR_UNSUPPORTED, "encoder(packed): no FP8 arithmetic on packed rows");
    int Fp8_max = 0;
    if (ffn8) {
        if (!layers) return fail(SF_ERR_INVALID_ARG, "encoder: NULL argument");
        for (int l = 0; l < D.nl; ++l) {
            if (int32_t rc = ffn_fp8_check("encoder(fp8 ffn)", D, &ffn8[l], true)) return rc;
            if (ffn8[l].k_ffn != layers[l].k_ffn)
                return fail(SF_ERR_INVALID_ARG, "encoder(fp8 ffn): k_ffn of layer %d differs from the compact layer's", l);
            Fp8_max = std::max(Fp8_max, (int)sf_ffn_fp8_padded(ffn8[l].k_ffn));
        }
        if (((uintptr_t)xq_out | (uintptr_t)hq_out) & 15)
            return fail(SF_ERR_INVALID_ARG, "encoder(fp8 ffn): 16-byte aligned code buffers required");
    }
    if (proj8) {
        if (!layers) return fail(SF_ERR_INVALID_ARG, "encoder: NULL argument");
        for (int l = 0; l < D.nl; ++l)
            if (int32_t rc = proj_fp8_check("encoder(fp8 projections)", D, &proj8[l], layers[l].k_head)) return rc;
        if (((uintptr_t)aq_out | (uintptr_t)oq_out) & 15)
            return fail(SF_ERR_INVALID_ARG, "encoder(fp8 projections): 16-byte aligned code buffers required");
        // the fused LayerNorm + quantiser reads 16 bytes per lane (layers after the first read the workspace)
        uintptr_t al = (uintptr_t)X;
        for (int l = 0; l < D.nl; ++l) al |= (uintptr_t)layers[l].ln1_g | (uintptr_t)layers[l].ln1_b;
        if (al & 15)
            return fail(SF_ERR_INVALID_ARG,
                        "encoder(fp8 projections): 16-byte aligned input and LayerNorm vectors required");
    }
    if (u_active && D.U >= D.L)
        return fail(SF_ERR_UNSUPPORTED, "encoder: per-sample active counts need U < L (U = %d, L = %d)", D.U, D.L);
    if (!layers || !X || !Y) return fail(SF_ERR_INVALID_ARG, "encoder: NULL argument");
    if (X == Y) return fail(SF_ERR_INVALID_ARG, "encoder: Y may not alias X");
    if (D.P > 1 && !pattern_id) return fail(SF_ERR_INVALID_ARG, "encoder: pattern_id required when P > 1");
    if ((D.flags & SF_FLAG_FINAL_LN) && (!final_g || !final_b))
        return fail(SF_ERR_INVALID_ARG, "encoder: final LayerNorm parameters missing");
    for (int l = 0; l < D.nl; ++l) {
        const sf_compact_layer &ly = layers[l];
        if (!ly.Wqkv || !ly.WoT || !ly.W1 || !ly.W2T || !ly.ln1_g || !ly.ln1_b || !ly.ln2_g || !ly.ln2_b ||
            !ly.head_group)
            return fail(SF_ERR_INVALID_ARG, "encoder: NULL pointer in layer %d", l);
    }
    // shape limits of the attention kernels, checked before anything is enqueued
    if (D.L > 16384) return fail(SF_ERR_SHAPE, "encoder: L <= 16384 required");
    if (D.dtype == SF_BF16 && D.dh != 32 && D.dh != 64 && D.dh != 128)
        return fail(SF_ERR_SHAPE, "encoder(bf16): dh must be 32, 64 or 128");
    if (D.dtype == SF_F32 && (D.dh % 4 || D.dh > 256))
        return fail(SF_ERR_SHAPE, "encoder(f32): dh must be a multiple of 4, at most 256");
    if (D.Hq > 64) return fail(SF_ERR_SHAPE, "encoder: Hq <= 64 required");
    EncWs w;
    if (int32_t rc = enc_ws(D, layers, workspace, w, proj8 != nullptr, pk ? (size_t)pk->Tc : 0)) return rc;
    if (!workspace || workspace_bytes < w.bytes || ((uintptr_t)workspace & 255))
        return fail(SF_ERR_WORKSPACE, "encoder: workspace of %zu bytes (256-byte aligned) required, got %zu",
                    w.bytes, workspace_bytes);

    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = D.dtype == SF_BF16;
    const size_t es = elem_size(D.dtype);
    // Packed rows: the row-wise steps (LayerNorm, GEMMs) see Tc/256 "samples" of 256 rows, each with the pattern of
    // its block (negative: unused, skipped); only the attention steps see the real samples.
    Dims Dg = D;
    const int32_t *gpat = pattern_id;
    if (pk) { Dg.B = pk->Tc / 256; Dg.L = 256; gpat = pk->blk_pattern; }
    const int64_t rows = (int64_t)Dg.B * Dg.L;
    // The residual stream is kept in fp32 between layers (x1 after the attention
    // block, x2 after the FFN); only the tensors feeding a contraction and the
    // final output are stored in the model dtype.
    const void *in = X;
    bool in_f32 = !bf;
    const bool final_ln = (D.flags & SF_FLAG_FINAL_LN) != 0;
    for (int l = 0; l < D.nl; ++l) {
        const sf_compact_layer &ly = layers[l];
        const int kh = ly.k_head, dh = D.dh, Hk = D.Hk;
        const int Nqk = (kh + Hk) * dh, Nqkv = (kh + 2 * Hk) * dh;
        const int ldq = bf && !proj8 && !pk ? Nqk : Nqkv;   // row length of the token-major buffer

        // x' = LN1(x);  Q, K (token-major) and V (bf16: transposed) = x' Wqkv'^T + b
        if (proj8) {
            // the same in FP8 arithmetic: codes of LN1(x), one GEMM for Q, K, V (token-major), V transposed after it
            const sf_proj_fp8 &pj = proj8[l];
            uint8_t *aq = aq_out ? aq_out + (size_t)l * rows * D.d : static_cast<uint8_t *>(w.xn);
            layernorm_q8(in, in_f32, ly.ln1_g, ly.ln1_b, D.eps, rows, D.d, 1.0f / pj.sx1, aq, st);
            GemmArgs q8{};
            q8.f8 = 1; q8.A = aq; q8.lda = D.d; q8.W = pj.Wqkv8; q8.ldw = D.d; q8.w_pstride = (int64_t)Nqkv * D.d;
            q8.bias = ly.bqkv; q8.bias_pstride = Nqkv; q8.pattern_id = pattern_id;
            q8.B = D.B; q8.L = D.L; q8.N = Nqkv; q8.K = D.d; q8.epi = EPI_ROWMAJOR; q8.act = ACT_NONE;
            q8.out_scale = pj.sx1 * pj.s_qkv; q8.C = w.qkv; q8.ldc = Nqkv;
            if (int32_t rc = gemm_fp8(q8, st)) return rc;
            transpose_v(w.qkv, Nqkv, Nqk, Hk * dh, D.B, D.L, w.Lp, w.vt, st);
        } else {
            layernorm(D.dtype, in_f32, in, ly.ln1_g, ly.ln1_b, D.eps, rows, D.d, w.xn, st);
            GemmArgs g{};
            g.A = w.xn; g.lda = D.d; g.W = ly.Wqkv; g.ldw = D.d; g.w_pstride = (int64_t)Nqkv * D.d;
            g.bias = ly.bqkv; g.bias_pstride = Nqkv; g.pattern_id = gpat;
            g.B = Dg.B; g.L = Dg.L; g.K = D.d; g.act = ACT_NONE; g.epi = EPI_ROWMAJOR;
            g.C = w.qkv; g.ldc = ldq; g.n0 = 0; g.N = bf && !pk ? Nqk : Nqkv;
            if (bf && pk) {
                // Q, K, V token-major in one launch; V^T per sample (what the attention kernels read) by a pass of
                // its own, since a 256-row block of packed rows may straddle samples
                if (int32_t rc = gemm(D.dtype, g, st)) return rc;
                transpose_v(w.qkv, Nqkv, Nqk, Hk * dh, D.B, D.L, w.Lp, w.vt, st, pk->row0);
            } else if (bf) {
                // one launch for Q, K and V when the large-tile kernel takes it (V is the transposed column range:
                // the normalised input is read once); otherwise Q/K and V separately
                GemmArgs q3 = g;
                q3.N = Nqkv; q3.VT = w.vt; q3.vt_from = Nqk; q3.vt_b = (int64_t)Hk * dh * w.Lp; q3.vt_n = w.Lp;
                if (gemm_takes_vt_split(D.dtype, q3)) {
                    if (int32_t rc = gemm(D.dtype, q3, st)) return rc;
                } else {
                    if (int32_t rc = gemm(D.dtype, g, st)) return rc;
                    g.n0 = Nqk; g.N = Hk * dh; g.epi = EPI_VT; g.C = w.vt;
                    g.vt_b = q3.vt_b; g.vt_n = q3.vt_n;
                    if (int32_t rc = gemm(D.dtype, g, st)) return rc;
                }
            } else {
                if (int32_t rc = gemm(D.dtype, g, st)) return rc;
            }
        }

        // SentryAttend over the kept heads
        AttnArgs a = enc_attn_args(D, kh);
        a.Q = w.qkv; a.sq = sf_strides{(int64_t)D.L * ldq, dh, ldq};
        a.K = (const char *)w.qkv + (size_t)kh * dh * es; a.sk = a.sq;
        if (bf) {
            a.V = w.vt; a.sv = sf_strides{(int64_t)Hk * dh * w.Lp, (int64_t)dh * w.Lp, w.Lp};
        } else {
            a.V = (const char *)w.qkv + (size_t)(kh + Hk) * dh * es; a.sv = a.sq;
        }
        a.head_group = ly.head_group; a.hg_stride = D.Hq; a.pattern_id = pattern_id; a.key_valid = key_valid;
        if (pk) { a.row0 = pk->row0; a.ext = pk->ext; }
        a.sample_idx = D.n_sample > 0 ? sample_idx : nullptr;
        a.u_active = u_active;
        a.selH = w.kh_max;
        const size_t sel_layer = (size_t)D.B * w.kh_max * D.U, score_layer = (size_t)D.B * w.kh_max * D.L;
        a.forced_sel = forced_sel ? forced_sel + l * sel_layer : nullptr;
        a.sel_out = sel_out ? sel_out + l * sel_layer : nullptr;
        a.score_out = score_out ? score_out + l * score_layer : nullptr;
        a.O = w.att; a.ldo = (int64_t)kh * dh;
        a.ws = w.attn_ws; a.ws_bytes = w.attn_ws_bytes;
        // Most rows lazy in every head: project only the active rows, the rest of a sample shares one vector
        // (in FP8 arithmetic the compact rows go through the FP8 GEMM, which wants at least 192 rows per sample)
        const int capA = w.lz_cap ? lazy_cap(D.L, kh, D.U, dh, D.d) : 0;
        const bool lazy = !pk && capA > 0 && capA <= w.lz_cap && (!proj8 || capA >= 256) &&
                          !(((uintptr_t)ly.bo | (uintptr_t)ly.ln2_g | (uintptr_t)ly.ln2_b | (uintptr_t)in) & 15);
        a.skip_fill = lazy && !(proj8 && oq_out);        // a caller who wants the codes of every row gets the rows filled
        a.act_bits = lazy ? reinterpret_cast<uint32_t *>(w.lz_cnt) : nullptr;
        if (int32_t rc = attention_forward(D.dtype, a, st)) return rc;
        if (lazy) {
            const AttnPlan pl = attn_plan(D.dtype, a, a.ws);
            lazy_rows_active(a.act_bits, pattern_id, D.B, D.L, capA, w.lz_arow, w.lz_pos, w.lz_n, w.lz_blk, st);
            if (proj8) {
                lazy_att_compact(w.att, a.ldo, pl.slot, pl.stats, ly.head_group, D.Hq, pattern_id, w.lz_arow, w.lz_n, D.B,
                                 kh, Hk, D.L, dh, capA, w.lz_A, st);
                // the same rows in FP8 arithmetic: codes of the compact rows, FP8 GEMM per sample, and the shared
                // vector from the codes of the context vector
                const sf_proj_fp8 &pj = proj8[l];
                const int Kh = kh * dh;
                const int64_t Ko = (int64_t)align_up((size_t)Kh, 128);
                quantize_rows_fp8(w.lz_A, Kh, (int64_t)D.B * capA, Kh, (int)Ko, 1.0f / pj.sa, w.lz_A8, st);
                if (oq_out)
                    quantize_rows_fp8(w.att, Kh, rows, Kh, (int)Ko, 1.0f / pj.sa,
                                      oq_out + (size_t)l * rows * align_up((size_t)w.kh_max * dh, 128), st);
                GemmArgs o8{};
                o8.f8 = 1; o8.A = w.lz_A8; o8.lda = Ko; o8.W = pj.WoT8; o8.ldw = Ko; o8.w_pstride = (int64_t)D.d * Ko;
                o8.pattern_id = pattern_id;
                o8.B = D.B; o8.L = capA; o8.N = D.d; o8.K = (int)Ko; o8.epi = EPI_ROWMAJOR; o8.act = ACT_NONE;
                o8.out_scale = pj.sa * pj.so; o8.C = w.lz_C; o8.ldc = D.d; o8.c_f32 = 1;
                if (int32_t rc = gemm_fp8(o8, st)) return rc;
                lazy_ctx_proj_q8(pl.stats, ly.head_group, D.Hq, pattern_id, pj.WoT8, (int64_t)D.d * Ko, (int)Ko, ly.bo,
                                 D.B, kh, Hk, dh, D.d, 1.0f / pj.sa, pj.sa * pj.so, w.lz_c, st);
            } else {
                lazy_att_compact_ctx_proj(w.att, a.ldo, pl.slot, pl.stats, ly.head_group, D.Hq, pattern_id, w.lz_arow,
                                          w.lz_n, D.B, kh, Hk, D.L, dh, capA, w.lz_A, ly.WoT, (int64_t)D.d * kh * dh, ly.bo,
                                          D.d, w.lz_c, st);
                GemmArgs o{};
                o.A = w.lz_A; o.lda = (int64_t)kh * dh; o.W = ly.WoT; o.ldw = (int64_t)kh * dh;
                // 128-row blocks of the compact buffer, each with its sample's pattern (-1: no rows, skipped)
                o.w_pstride = (int64_t)D.d * kh * dh; o.pattern_id = w.lz_blk;
                o.B = D.B * (capA / 128); o.L = 128; o.N = D.d; o.K = kh * dh; o.epi = EPI_ROWMAJOR; o.act = ACT_NONE;
                o.C = w.lz_C; o.ldc = D.d; o.c_f32 = 1;
                if (int32_t rc = gemm(D.dtype, o, st)) return rc;
            }
            // x1 = x + projection, and xn = LN2(x1) (bf16, or E4M3 codes for an FFN in FP8 arithmetic), in one pass
            const bool to_y = l == D.nl - 1 && !final_ln;
            if (ffn8) {
                uint8_t *xq = xq_out ? xq_out + (size_t)l * rows * D.d : static_cast<uint8_t *>(w.xn);
                uint8_t *hq = hq_out ? hq_out + (size_t)l * rows * Fp8_max : static_cast<uint8_t *>(w.hid);
                lazy_combine_ln(in, in_f32, w.lz_pos, w.lz_C, ly.bo, w.lz_c, D.B, D.L, capA, ly.ln2_g, ly.ln2_b, D.eps,
                                D.d, static_cast<float *>(w.x1), xq, 1.0f / ffn8[l].sx, st);
                if (int32_t rc = ffn_fp8_forward(D, ffn8[l], w.x1, true, pattern_id, true, true, to_y ? Y : w.x2, !to_y,
                                                 xq, hq, st, true))
                    return rc;
            } else {
                lazy_combine_ln(in, in_f32, w.lz_pos, w.lz_C, ly.bo, w.lz_c, D.B, D.L, capA, ly.ln2_g, ly.ln2_b, D.eps,
                                D.d, static_cast<float *>(w.x1), w.xn, 0.f, st);
                if (int32_t rc = ffn_forward(D, ly, w.x1, true, pattern_id, true, true, to_y ? Y : w.x2, !to_y, w.xn,
                                             w.hid, st, true))
                    return rc;
            }
            in = w.x2;
            in_f32 = true;
            continue;
        }

        // x1 = x + att Wo' + bo   (only the kept heads' rows of Wo exist)
        if (proj8) {
            const sf_proj_fp8 &pj = proj8[l];
            const int Kh = kh * dh;
            const int64_t Ko = (int64_t)align_up((size_t)Kh, 128);
            uint8_t *oq = oq_out ? oq_out + (size_t)l * rows * align_up((size_t)w.kh_max * dh, 128) : w.oq;
            quantize_rows_fp8(w.att, Kh, rows, Kh, (int)Ko, 1.0f / pj.sa, oq, st);
            GemmArgs o8{};
            o8.f8 = 1; o8.A = oq; o8.lda = Ko; o8.W = pj.WoT8; o8.ldw = Ko; o8.w_pstride = (int64_t)D.d * Ko;
            o8.bias = ly.bo; o8.bias_pstride = 0; o8.pattern_id = pattern_id;
            o8.B = D.B; o8.L = D.L; o8.N = D.d; o8.K = (int)Ko; o8.epi = EPI_ROWMAJOR; o8.act = ACT_NONE;
            o8.out_scale = pj.sa * pj.so;
            o8.R = in; o8.ldr = D.d; o8.r_f32 = in_f32; o8.C = w.x1; o8.ldc = D.d; o8.c_f32 = 1;
            if (int32_t rc = gemm_fp8(o8, st)) return rc;
        } else {
            GemmArgs o{};
            o.A = w.att; o.lda = (int64_t)kh * dh; o.W = ly.WoT; o.ldw = (int64_t)kh * dh;
            o.w_pstride = (int64_t)D.d * kh * dh; o.bias = ly.bo; o.bias_pstride = 0; o.pattern_id = gpat;
            o.B = Dg.B; o.L = Dg.L; o.N = D.d; o.K = kh * dh; o.epi = EPI_ROWMAJOR; o.act = ACT_NONE;
            o.R = in; o.ldr = D.d; o.r_f32 = in_f32; o.C = w.x1; o.ldc = D.d; o.c_f32 = 1;
            if (int32_t rc = gemm(D.dtype, o, st)) return rc;
        }

        // x2 = x1 + FFN(LN2(x1)); the last layer without a final LN writes Y directly
        const bool to_y = l == D.nl - 1 && !final_ln;
        if (ffn8) {
            // the codes of LN2(x1) take the place of the normalised input, those of the hidden activations the
            // place of the 16-bit hidden buffer (both are smaller)
            uint8_t *xq = xq_out ? xq_out + (size_t)l * rows * D.d : static_cast<uint8_t *>(w.xn);
            uint8_t *hq = hq_out ? hq_out + (size_t)l * rows * Fp8_max : static_cast<uint8_t *>(w.hid);
            if (int32_t rc = ffn_fp8_forward(D, ffn8[l], w.x1, true, pattern_id, true, true, to_y ? Y : w.x2, !to_y,
                                             xq, hq, st))
                return rc;
        } else if (int32_t rc = ffn_forward(Dg, ly, w.x1, true, gpat, true, true, to_y ? Y : w.x2, !to_y, w.xn,
                                            w.hid, st))
            return rc;
        in = w.x2;
        in_f32 = true;
    }
    if (final_ln) layernorm(D.dtype, 1, w.x2, final_g, final_b, D.eps, rows, D.d, Y, st);
    return check_launch("encoder_forward");
}

extern "C" int32_t sf_encoder_forward(const sf_desc *desc, const sf_compact_layer *layers, const void *X,
                                      const int32_t *pattern_id, const uint8_t *key_valid,
                                      const int32_t *sample_idx, const void *final_g, const void *final_b,
                                      const int32_t *forced_sel,
                                      void *Y, int32_t *sel_out, float *score_out, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    return encoder_forward_impl(desc, layers, X, pattern_id, key_valid, sample_idx, nullptr, final_g, final_b,
                                forced_sel, Y, sel_out, score_out, workspace, workspace_bytes, stream);
}

extern "C" int32_t sf_encoder_forward_fp8ffn(const sf_desc *desc, const sf_compact_layer *layers,
                                             const sf_ffn_fp8 *ffn8, const void *X, const int32_t *pattern_id,
                                             const uint8_t *key_valid, const int32_t *sample_idx,
                                             const void *final_g, const void *final_b, const int32_t *forced_sel,
                                             void *Y, int32_t *sel_out, float *score_out, uint8_t *xq_out,
                                             uint8_t *hq_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!ffn8) return fail(SF_ERR_INVALID_ARG, "encoder(fp8 ffn): ffn8 is NULL");
    return encoder_forward_impl(desc, layers, X, pattern_id, key_valid, sample_idx, nullptr, final_g, final_b,
                                forced_sel, Y, sel_out, score_out, workspace, workspace_bytes, stream, ffn8, xq_out,
                                hq_out);
}

extern "C" int32_t sf_encoder_forward_ragged(const sf_desc *desc, const sf_compact_layer *layers, const void *X,
                                             const int32_t *pattern_id, const uint8_t *key_valid,
                                             const int32_t *u_active, const int32_t *sample_idx,
                                             const void *final_g, const void *final_b, void *Y,
                                             int32_t *sel_out, float *score_out, void *workspace,
                                             size_t workspace_bytes, void *stream)
{
    if (!u_active) return fail(SF_ERR_INVALID_ARG, "encoder_ragged: u_active is NULL");
    return encoder_forward_impl(desc, layers, X, pattern_id, key_valid, sample_idx, u_active, final_g, final_b,
                                nullptr, Y, sel_out, score_out, workspace, workspace_bytes, stream);
}

extern "C" size_t sf_encoder_packed_workspace_bytes(const sf_desc *desc, const sf_compact_layer *layers, int32_t Tc)
{
    Dims D;
    EncWs w;
    if (Tc < 256 || Tc % 256 || read_desc(desc, D) || !layers || enc_ws(D, layers, nullptr, w, false, (size_t)Tc)) return 0;
    return w.bytes;
}

extern "C" int32_t sf_encoder_forward_packed(const sf_desc *desc, const sf_compact_layer *layers, const void *Xp,
                                             const sf_token_pack_plan *plan, const int32_t *pattern_id,
                                             const int32_t *sample_idx, const void *final_g, const void *final_b,
                                             void *Yp, int32_t *sel_out, float *score_out, void *workspace,
                                             size_t workspace_bytes, void *stream)
{
    if (!plan) return fail(SF_ERR_INVALID_ARG, "encoder_packed: plan is NULL");
    if (plan->Tc < 256 || plan->Tc % 256 || (int64_t)plan->Tc > ((int64_t)1 << 30))
        return fail(SF_ERR_INVALID_ARG, "encoder_packed: Tc must be a positive multiple of 256 (below 2^30)");
    if (!plan->row0 || !plan->ext || !plan->blk_pattern || !plan->valid_c || !plan->u_active)
        return fail(SF_ERR_INVALID_ARG, "encoder_packed: NULL pointer in the plan");
    return encoder_forward_impl(desc, layers, Xp, pattern_id, plan->valid_c, sample_idx, plan->u_active, final_g,
                                final_b, nullptr, Yp, sel_out, score_out, workspace, workspace_bytes, stream, nullptr,
                                nullptr, nullptr, nullptr, nullptr, nullptr, plan);
}

extern "C" size_t sf_encoder_fp8_workspace_bytes(const sf_desc *desc, const sf_compact_layer *layers)
{
    Dims D;
    EncWs w;
    if (read_desc(desc, D) || !layers || enc_ws(D, layers, nullptr, w, true)) return 0;
    return w.bytes;
}

extern "C" int32_t sf_encoder_forward_fp8(const sf_desc *desc, const sf_compact_layer *layers, const sf_ffn_fp8 *ffn8,
                                          const sf_proj_fp8 *proj8, const void *X, const int32_t *pattern_id,
                                          const uint8_t *key_valid, const int32_t *sample_idx, const void *final_g,
                                          const void *final_b, const int32_t *forced_sel, void *Y, int32_t *sel_out,
                                          float *score_out, uint8_t *xq_out, uint8_t *hq_out, uint8_t *aq_out,
                                          uint8_t *oq_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!ffn8 && !proj8) return fail(SF_ERR_INVALID_ARG, "encoder(fp8): ffn_host and proj_host are both NULL");
    return encoder_forward_impl(desc, layers, X, pattern_id, key_valid, sample_idx, nullptr, final_g, final_b,
                                forced_sel, Y, sel_out, score_out, workspace, workspace_bytes, stream, ffn8, xq_out,
                                hq_out, proj8, aq_out, oq_out);
}
