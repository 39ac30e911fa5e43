// SentryAttend (Sec. 4.4 of the paper): the steps that are not contractions --
// K/V statistics (mean key for the sparsity score, mean value = context
// vector), the top-U query choice, the lazy-row fill -- plus the plain fp32
// kernels and the dispatch.  The bf16 MFMA kernels are in attention_bf16.hip.
#include <mutex>

#include "attention.hpp"
#include "topk.hpp"

namespace sf {

// ---------------------------------------------------------------- statistics
// Partial column sums of K and V over one chunk of allowed keys.
// grid (chunks, B*nG), 256 threads; thread t owns column e = t % DHP.
template <class T>
__global__ __launch_bounds__(256) void kv_stats_partial_kernel(
    const T *__restrict__ K, sf_strides sk, const T *__restrict__ V, sf_strides sv, int64_t v_sj,
    int64_t v_se, const uint8_t *__restrict__ key_valid, int nG, int L, int dh, int DHP,
    float *__restrict__ part, const int32_t *__restrict__ row0, const int32_t *__restrict__ row0_v)
{
    __shared__ float red[2][256];
    const int bg = blockIdx.y, b = bg / nG, g = bg % nG;
    const int e = threadIdx.x % DHP, rg = threadIdx.x / DHP, nrg = 256 / DHP;
    const int j0 = blockIdx.x * STAT_CHUNK, j1 = min(L, j0 + STAT_CHUNK);
    const T *Kb = K + sample_offset(row0, b, sk) + (int64_t)g * sk.h;
    const T *Vb = V + sample_offset(row0_v, b, sv) + (int64_t)g * sv.h;      // a transposed V is b-strided
    const uint8_t *kv = key_valid ? key_valid + (int64_t)b * L : nullptr;
    float sk_ = 0.f, sv_ = 0.f;
    if (e < dh)
        for (int j = j0 + rg; j < j1; j += nrg) {
            if (kv && !kv[j]) continue;
            sk_ += to_f32(Kb[(int64_t)j * sk.l + e]);
            sv_ += to_f32(Vb[(int64_t)j * v_sj + (int64_t)e * v_se]);
        }
    red[0][threadIdx.x] = sk_;
    red[1][threadIdx.x] = sv_;
    __syncthreads();
    if (threadIdx.x < DHP && e < dh) {
        float a = 0.f, c = 0.f;
        for (int r = 0; r < nrg; ++r) { a += red[0][r * DHP + e]; c += red[1][r * DHP + e]; }
        float *o = part + (((int64_t)bg * gridDim.x + blockIdx.x) * 2) * dh;
        o[e] = a;
        o[dh + e] = c;
    }
}

// bf16 variant with 16-byte loads: K rows are dh-contiguous, V is read from
// its key-contiguous transposed layout [dh][Lp].  Same outputs as above.
// Every load of the chunk (validity bytes, K rows, V^T pieces) is issued before the first use, so a block pays one
// memory round trip instead of one per pass; validity is applied as a select afterwards (masked rows may hold
// anything).  The order of the additions is that of the pass-by-pass loop.
template <int DH>
__global__ __launch_bounds__(256) void kv_stats_partial_bf16_kernel(
    const h16 *__restrict__ K, sf_strides sk, const h16 *__restrict__ VT, sf_strides svt,
    const uint8_t *__restrict__ key_valid, int nG, int L, float *__restrict__ part,
    const int32_t *__restrict__ row0)
{
    constexpr int CH = DH / 8, RP = 256 / CH, TPR = 256 / DH;
    constexpr int NK = STAT_CHUNK / RP, NV = STAT_CHUNK / (TPR * 8);
    static_assert(STAT_CHUNK % RP == 0 && STAT_CHUNK % (TPR * 8) == 0 && STAT_CHUNK <= 256, "chunk shape");
    __shared__ float red[RP][DH];
    __shared__ uint8_t ok_s[STAT_CHUNK];
    const int bg = blockIdx.y, b = bg / nG, g = bg % nG, tid = threadIdx.x;
    const int j0 = blockIdx.x * STAT_CHUNK, j1 = min(L, j0 + STAT_CHUNK);
    const h16 *Kb = K + sample_offset(row0, b, sk) + (int64_t)g * sk.h;
    const h16 *Vb = VT + (int64_t)b * svt.b + (int64_t)g * svt.h;        // the transposed copy: always b-strided
    const uint8_t *kv = key_valid ? key_valid + (int64_t)b * L : nullptr;
    float *o = part + (((int64_t)bg * gridDim.x + blockIdx.x) * 2) * DH;

    const int r = tid / CH, c = tid % CH;          // K: row r of a pass, 16-byte chunk c
    const int e = tid / TPR, q = tid % TPR;        // V^T: row e, 8 keys at q*8 of a pass
    uint8_t okb = 0;
    if (tid < STAT_CHUNK) okb = j0 + tid < j1 && (!kv || kv[j0 + tid]);
    h16x8 kt[NK], vt[NV];
#pragma unroll
    for (int k = 0; k < NK; ++k) {
        const int j = j0 + r + RP * k;
        kt[k] = h16x8{};
        if (j < j1) kt[k] = *reinterpret_cast<const h16x8 *>(Kb + (int64_t)j * sk.l + c * 8);
    }
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int j = j0 + q * 8 + TPR * 8 * k;
        vt[k] = h16x8{};
        if (j < j1) vt[k] = *reinterpret_cast<const h16x8 *>(Vb + (int64_t)e * svt.l + j);   // j + 8 <= Lp
    }
    if (tid < STAT_CHUNK) ok_s[tid] = okb;
    __syncthreads();

    {   // column sums of K over the allowed keys of this chunk
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < NK; ++k)
            if (ok_s[r + RP * k]) {
#pragma unroll
                for (int t = 0; t < 8; ++t) acc[t] += (float)kt[k][t];
            }
#pragma unroll
        for (int t = 0; t < 8; ++t) red[r][c * 8 + t] = acc[t];
        __syncthreads();
        if (tid < DH) {
            float s = 0.f;
            for (int rr = 0; rr < RP; ++rr) s += red[rr][tid];
            o[tid] = s;
        }
    }
    {   // row sums of V^T over the allowed keys of this chunk
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k)
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (ok_s[q * 8 + TPR * 8 * k + u]) s += (float)vt[k][u];
#pragma unroll
        for (int w = 1; w < TPR; w <<= 1) s += __shfl_xor(s, w);
        if (q == 0) o[DH + e] = s;
    }
}

// stats[bg][0][:] = mean allowed key, stats[bg][1][:] = mean allowed value.
__global__ __launch_bounds__(256) void kv_stats_final_kernel(
    const float *__restrict__ part, int chunks, const uint8_t *__restrict__ key_valid, int nG, int L,
    int dh, float *__restrict__ stats, int32_t *__restrict__ n_valid, uint32_t *__restrict__ act_bits)
{
    __shared__ int red[4];
    const int bg = blockIdx.x, b = bg / nG;
    int c = 0;
    if (key_valid) {
        for (int j = threadIdx.x; j < L; j += 256) c += key_valid[(int64_t)b * L + j] != 0;
        c = block_sum<256>(c, red);
    } else {
        c = L;
    }
    if (threadIdx.x == 0 && bg % nG == 0) n_valid[b] = c;
    if (act_bits && bg % nG == 0)                 // the selection that follows sets the bits of the rows it picks
        for (int w = threadIdx.x; w < (L + 31) / 32; w += 256) act_bits[(int64_t)b * ((L + 31) / 32) + w] = 0u;
    const float inv = c > 0 ? 1.0f / (float)c : 0.f;
    for (int t = threadIdx.x; t < 2 * dh; t += 256) {
        float s = 0.f;
#pragma unroll 8
        for (int ch = 0; ch < chunks; ++ch) s += part[(((int64_t)bg * chunks + ch) * 2) * dh + t];      // loads in flight together
        stats[(int64_t)bg * 2 * dh + t] = s * inv;
    }
}

// ------------------------------------------------------------------- selection
// One block per (b, head): the U_eff = min(U, u_active[b], #allowed) queries with the
// highest score, ties to the lower index; emitted ascending.  score == NULL
// means "every allowed query" (used when U >= L).
template <int NT>
__global__ __launch_bounds__(NT) void select_kernel(
    const float *__restrict__ score, int scoreH, const uint8_t *__restrict__ key_valid, int nH, int L,
    int U, const int32_t *__restrict__ u_active, int32_t *__restrict__ sel, int selH, int32_t *__restrict__ slot,
    uint32_t *__restrict__ act_bits)
{
    extern __shared__ uint32_t keys[];
    __shared__ int scratch[TOPK_SCRATCH];
    __shared__ int red[NT / 64];    // not part of `scratch`: block_topk clears its histogram there right away
    const int bh = blockIdx.x, b = bh / nH, h = bh % nH;
    const uint8_t *kv = key_valid ? key_valid + (int64_t)b * L : nullptr;
    const float *M = score ? score + ((int64_t)b * scoreH + h) * L : nullptr;
    int32_t *sl = slot + (int64_t)bh * L;
    int32_t *se = sel + ((int64_t)b * selH + h) * U;
    int c = 0;
    for (int i = threadIdx.x; i < L; i += NT) {
        const bool ok = !kv || kv[i];
        // allowed queries get a key >= 1 (sortable_key(-inf) > 0), others key 0
        keys[i] = ok ? (M ? sortable_key(M[i]) : 1u) : 0u;
        c += ok;
    }
    const int n_ok = block_sum<NT>(c, red);        // also orders the LDS writes
    // u_active: this sample's own number of active queries (samples of different length in one batch)
    const int k = min(u_active ? min(max(u_active[b], 0), U) : U, n_ok);
    if (k == 0) {
        for (int i = threadIdx.x; i < L; i += NT) sl[i] = -1;
    } else {
        block_topk<NT>(keys, L, k, scratch, [&](int i, bool kept, int pos) {
            sl[i] = kept ? pos : -1;
            if (kept) {
                se[pos] = i;
                if (act_bits) atomicOr(&act_bits[(int64_t)b * ((L + 31) / 32) + (i >> 5)], 1u << (i & 31));
            }
        });
    }
    for (int r = k + threadIdx.x; r < U; r += NT) se[r] = -1;
}

// Caller-supplied active set: build the row -> slot map and copy the list.
__global__ __launch_bounds__(256) void forced_slot_kernel(const int32_t *__restrict__ forced, int forcedH,
                                                          int nH, int L, int U, int32_t *__restrict__ sel,
                                                          int selH, int32_t *__restrict__ slot,
                                                          uint32_t *__restrict__ act_bits)
{
    const int bh = blockIdx.x, b = bh / nH, h = bh % nH;
    int32_t *sl = slot + (int64_t)bh * L;
    for (int i = threadIdx.x; i < L; i += 256) sl[i] = -1;
    __syncthreads();
    for (int r = threadIdx.x; r < U; r += 256) {
        int q = forced[((int64_t)b * forcedH + h) * U + r];
        if (q < 0 || q >= L) q = -1;
        sel[((int64_t)b * selH + h) * U + r] = q;
        if (q >= 0) {
            sl[q] = r;
            if (act_bits) atomicOr(&act_bits[(int64_t)b * ((L + 31) / 32) + (q >> 5)], 1u << (q & 31));
        }
    }
}

// ------------------------------------------------------------------------ fill
// Every row that is not active takes its group's context vector.  One block
// per (sample, FILL_ROWS rows): the row -> slot map of those rows and the context
// vectors of all heads are staged in LDS (coalesced along the row index), then
// every thread writes VEC consecutive output elements at a time, rows of O
// contiguous.  Active rows are left alone.
constexpr int FILL_ROWS = 64;      // rows per block: enough stores per block to cover its two dependent loads

template <class T, int VEC>
__global__ __launch_bounds__(256) void fill_kernel(
    int nH, int nG, int L, int dh, const int32_t *__restrict__ slot,
    const int32_t *__restrict__ head_group, int hg_stride, const int32_t *__restrict__ pattern_id,
    const float *__restrict__ stats, T *__restrict__ O, int64_t ldo, const int32_t *__restrict__ row0,
    const int32_t *__restrict__ ext)
{
    extern __shared__ __attribute__((aligned(16))) char fsm[];
    float *ctx = reinterpret_cast<float *>(fsm);                 // [nH][dh]
    int32_t *sl = reinterpret_cast<int32_t *>(ctx + nH * dh);    // [nH][FILL_ROWS]
    const int b = blockIdx.y, i0 = blockIdx.x * FILL_ROWS;
    // packed samples: the rows the sample owns (its tokens and the padding behind them); rows at or beyond L have no
    // slot entry and are padding
    const int rows_b = ext ? ext[b] : L;
    if (i0 >= rows_b) return;
    const int p = pattern_id ? pattern_id[b] : 0;
    for (int t = threadIdx.x; t < nH * dh; t += 256) {
        const int h = t / dh, e = t % dh;
        const int g = head_group[(int64_t)p * hg_stride + h];
        ctx[t] = stats[(((int64_t)b * nG + g) * 2 + 1) * dh + e];
    }
    for (int t = threadIdx.x; t < nH * FILL_ROWS; t += 256) {
        const int h = t / FILL_ROWS, i = i0 + (t % FILL_ROWS);
        sl[t] = i < L ? slot[((int64_t)b * nH + h) * L + i] : -1;
    }
    __syncthreads();
    const int qv = dh / VEC, per_row = nH * qv;
    for (int c = threadIdx.x; c < FILL_ROWS * per_row; c += 256) {
        const int r = c / per_row, h = (c % per_row) / qv, e = (c % qv) * VEC;
        const int i = i0 + r;
        if (i >= rows_b) break;
        if (sl[h * FILL_ROWS + r] >= 0) continue;          // active row: written by the active pass / the merge
        float v[VEC];
#pragma unroll
        for (int t = 0; t < VEC; ++t) v[t] = ctx[h * dh + e + t];
        T *o = O + (sample_row(row0, b, L) + i) * ldo + (int64_t)h * dh + e;
        if constexpr (sizeof(T) == 2 && VEC == 8) {
            h16x8 ov;
#pragma unroll
            for (int t = 0; t < 8; ++t) ov[t] = (h16)v[t];
            *reinterpret_cast<h16x8 *>(o) = ov;             // ldo % 8 == 0 and 16-byte aligned O checked on the host
        } else {
#pragma unroll
            for (int t = 0; t < VEC; ++t) o[t] = from_f32<T>(v[t]);
        }
    }
}

// Merge of the key splits of the active pass: one wave per (sample, head,
// active slot).  Lane sp holds the (max, sum) pair of split sp (splits <= 64),
// the weights 2^(m_sp - m) are formed once, then lane e accumulates output
// dimension e over the splits (partials are [b, head, split, slot, dh]).
template <class T>
__global__ __launch_bounds__(256) void merge_splits_kernel(
    int nH, int L, int dh, int U, int Upad, int splits, int64_t n_waves, const int32_t *__restrict__ sel,
    int selH, const float *__restrict__ part_o, const float *__restrict__ part_ml, T *__restrict__ O,
    int64_t ldo, const int32_t *__restrict__ row0)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= n_waves) return;
    const int s = (int)(w % U);
    const int64_t bh = w / U;
    const int h = (int)(bh % nH);
    const int64_t b = bh / nH;
    const int64_t base = bh * splits;
    // an empty slot (fewer allowed queries than U) has no row and no partials: nothing to merge
    const int qi = sel[((int64_t)b * selH + h) * U + s];
    if (qi < 0) return;                                     // wave-uniform
    float ms = -INFINITY, ls = 0.f;
    if (lane < splits) {
        const int64_t q = (base + lane) * Upad + s;
        ms = part_ml[q * 2];
        ls = part_ml[q * 2 + 1];
    }
    float m = ms;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    const float wgt = (ms == -INFINITY) ? 0.f : exp2f(ms - m);
    float den = wgt * ls;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) den += __shfl_xor(den, o);
    const float inv = den > 0.f ? 1.0f / den : 0.f;
    T *orow = O + (sample_row(row0, (int)b, L) + qi) * ldo + (int64_t)h * dh;
    for (int e = lane; e < dh; e += 64) {
        float acc = 0.f;
        const float *po = part_o + (base * Upad + s) * dh + e;
#pragma unroll 4
        for (int sp = 0; sp < splits; ++sp) acc += __shfl(wgt, sp) * po[(int64_t)sp * Upad * dh];
        orow[e] = from_f32<T>(acc * inv);
    }
}

// V [B,nG,L,dh] -> VT [B,nG,dh,Lp] (bf16), 32x32 tiles through LDS.
__global__ __launch_bounds__(256) void transpose_v_kernel(const uint16_t *__restrict__ V, sf_strides sv, int nG,
                                                          int L, int dh, int Lp, uint16_t *__restrict__ VT,
                                                          const int32_t *__restrict__ row0)
{
    __shared__ uint16_t tile[32][33];
    const int bg = blockIdx.z, b = bg / nG, g = bg % nG;
    const int j0 = blockIdx.x * 32, e0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const uint16_t *Vb = V + sample_offset(row0, b, sv) + (int64_t)g * sv.h;
    for (int jj = ty; jj < 32; jj += 8) {
        const int j = j0 + jj, e = e0 + tx;
        tile[jj][tx] = (j < L && e < dh) ? Vb[(int64_t)j * sv.l + e] : (uint16_t)0;
    }
    __syncthreads();
    uint16_t *o = VT + (int64_t)bg * dh * Lp;
    for (int ee = ty; ee < 32; ee += 8) {
        const int e = e0 + ee, j = j0 + tx;
        if (e < dh && j < Lp) o[(int64_t)e * Lp + j] = tile[tx][ee];
    }
}

// ------------------------------------------------------------ plain fp32 path
// Sparsity score, one thread per query, over the Lk keys of K (validity key_mask [B,Lk] or NULL,
// n_keys[b] of them valid): the sample's own keys, or the gathered key sample.
__global__ __launch_bounds__(256) void score_f32_kernel(
    const float *__restrict__ Q, sf_strides sq, const float *__restrict__ K, sf_strides sk,
    const int32_t *__restrict__ head_group, int hg_stride, const int32_t *__restrict__ pattern_id,
    const uint8_t *__restrict__ query_valid, const uint8_t *__restrict__ key_mask,
    const int32_t *__restrict__ n_keys, int nH, int L, int Lk, int dh, float *__restrict__ score, int scoreH,
    const int32_t *__restrict__ row0, int keys_packed)
{
    const int bh = blockIdx.y, b = bh / nH, h = bh % nH;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= L) return;
    float *out = score + ((int64_t)b * scoreH + h) * L + i;
    if (query_valid && !query_valid[(int64_t)b * L + i]) { *out = -INFINITY; return; }
    if (n_keys[b] == 0) { *out = 0.f; return; }
    const uint8_t *km = key_mask ? key_mask + (int64_t)b * Lk : nullptr;
    const int g = head_group[(int64_t)(pattern_id ? pattern_id[b] : 0) * hg_stride + h];
    const float *q = Q + sample_offset(row0, b, sq) + (int64_t)h * sq.h + (int64_t)i * sq.l;
    // the gathered key sample lives in the workspace and is b-strided whatever the layout of K
    const float *Kb = K + sample_offset(keys_packed ? row0 : nullptr, b, sk) + (int64_t)g * sk.h;
    const float scale = 1.0f / sqrtf((float)dh);
    float mx = -INFINITY, sum = 0.f;
    for (int j = 0; j < Lk; ++j) {
        if (km && !km[j]) continue;
        const float *k = Kb + (int64_t)j * sk.l;
        float s = 0.f;
        for (int e = 0; e < dh; ++e) s = fmaf(q[e], k[e], s);
        s *= scale;
        mx = fmaxf(mx, s);
        sum += s;
    }
    *out = mx - sum / (float)n_keys[b];
}

// Key sample of the sparsity score: one block per (sample, group).  The sample is treated as a set
// (LDS bit words, integer atomics), intersected with the allowed keys, listed in ascending key order
// and gathered into Ks [B,nG,Sp,dh] (zero rows beyond the n_keys[b] listed keys), with the row validity
// ks_valid [B,Sp] and the mean listed key in ks_stats [(b*nG+g)*2*dh + e] (the layout of the K/V
// statistics; only the mean-key half is used).
template <class T>
__global__ __launch_bounds__(256) void gather_key_sample_kernel(
    const T *__restrict__ K, sf_strides sk, const uint8_t *__restrict__ key_valid,
    const int32_t *__restrict__ sample_idx, int n_sample, int nG, int L, int dh, int Sp,
    T *__restrict__ Ks, uint8_t *__restrict__ ks_valid, float *__restrict__ ks_stats,
    int32_t *__restrict__ n_keys, const int32_t *__restrict__ row0)
{
    extern __shared__ uint32_t gsm[];
    const int nwords = (L + 31) / 32;
    uint32_t *words = gsm;                                        // [nwords]
    int32_t *list = reinterpret_cast<int32_t *>(gsm + nwords);    // [Sp]
    __shared__ int nk_s;
    const int bg = blockIdx.x, b = bg / nG, g = bg % nG, tid = threadIdx.x;
    const uint8_t *kv = key_valid ? key_valid + (int64_t)b * L : nullptr;
    for (int w = tid; w < nwords; w += 256) words[w] = 0u;
    __syncthreads();
    for (int r = tid; r < n_sample; r += 256) {
        const int idx = sample_idx[(int64_t)b * n_sample + r];
        if (idx >= 0 && idx < L && (!kv || kv[idx])) atomicOr(&words[idx >> 5], 1u << (idx & 31));
    }
    __syncthreads();
    if (tid < 64) {                                               // ascending list of the set bits
        int base = 0;
        for (int w0 = 0; w0 < nwords; w0 += 64) {
            uint32_t w = (w0 + tid < nwords) ? words[w0 + tid] : 0u;
            const int pc = __popc(w);
            int incl = pc;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(incl, o);
                if (tid >= o) incl += t;
            }
            int pos = base + incl - pc;
            while (w) {
                const int bit = __ffs((int)w) - 1;
                list[pos++] = (w0 + tid) * 32 + bit;
                w &= w - 1u;
            }
            base += __shfl(incl, 63);
        }
        if (tid == 0) nk_s = base;
    }
    __syncthreads();
    const int nk = nk_s;                                          // <= n_sample <= Sp
    const T *Kb = K + sample_offset(row0, b, sk) + (int64_t)g * sk.h;
    T *out = Ks + (int64_t)bg * Sp * dh;
    for (int t = tid; t < Sp * dh; t += 256) {
        const int r = t / dh, e = t % dh;
        out[t] = r < nk ? Kb[(int64_t)list[r] * sk.l + e] : from_f32<T>(0.f);
    }
    if (g == 0) {
        for (int r = tid; r < Sp; r += 256) ks_valid[(int64_t)b * Sp + r] = r < nk ? 1 : 0;
        if (tid == 0) n_keys[b] = nk;
    }
    for (int e = tid; e < dh; e += 256) {
        float acc = 0.f;
        for (int r = 0; r < nk; ++r) acc += to_f32(Kb[(int64_t)list[r] * sk.l + e]);
        ks_stats[((int64_t)bg * 2) * dh + e] = nk ? acc / (float)nk : 0.f;
    }
}

// Active rows, Eq. (6): one 64-lane wave per (b, head, slot).
__global__ __launch_bounds__(64) void attend_f32_kernel(
    const float *__restrict__ Q, sf_strides sq, const float *__restrict__ K, sf_strides sk,
    const float *__restrict__ V, sf_strides sv, int64_t v_sj, int64_t v_se,
    const int32_t *__restrict__ head_group, int hg_stride, const int32_t *__restrict__ pattern_id,
    const uint8_t *__restrict__ key_valid, const int32_t *__restrict__ sel, int selH, int nH, int L, int dh,
    int U, float *__restrict__ O, int64_t ldo, const int32_t *__restrict__ row0)
{
    extern __shared__ float prob[];
    const int bh = blockIdx.y, b = bh / nH, h = bh % nH, lane = threadIdx.x;
    const int qi = sel[((int64_t)b * selH + h) * U + blockIdx.x];
    if (qi < 0) return;
    const uint8_t *kv = key_valid ? key_valid + (int64_t)b * L : nullptr;
    const int g = head_group[(int64_t)(pattern_id ? pattern_id[b] : 0) * hg_stride + h];
    const float *q = Q + sample_offset(row0, b, sq) + (int64_t)h * sq.h + (int64_t)qi * sq.l;
    const float *Kb = K + sample_offset(row0, b, sk) + (int64_t)g * sk.h;
    const float *Vb = V + sample_offset(row0, b, sv) + (int64_t)g * sv.h;
    const float scale = 1.0f / sqrtf((float)dh);
    float mx = -INFINITY;
    for (int j = lane; j < L; j += 64) {
        float s = -INFINITY;
        if (!kv || kv[j]) {
            const float *k = Kb + (int64_t)j * sk.l;
            s = 0.f;
            for (int e = 0; e < dh; ++e) s = fmaf(q[e], k[e], s);
            s *= scale;
        }
        prob[j] = s;
        mx = fmaxf(mx, s);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float den = 0.f;
    for (int j = lane; j < L; j += 64) {
        const float pj = prob[j] == -INFINITY ? 0.f : expf(prob[j] - mx);
        prob[j] = pj;
        den += pj;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) den += __shfl_xor(den, o);
    __syncthreads();
    const float inv = 1.0f / den;
    for (int e = lane; e < dh; e += 64) {
        float acc = 0.f;
        for (int j = 0; j < L; ++j) acc = fmaf(prob[j], Vb[(int64_t)j * v_sj + (int64_t)e * v_se], acc);
        O[(sample_row(row0, b, L) + qi) * ldo + (int64_t)h * dh + e] = acc * inv;
    }
}

// ------------------------------------------------------------------- planning
AttnPlan attn_plan(int dtype, const AttnArgs &a, void *ws)
{
    AttnPlan pl{};
    const bool sparse = a.U < a.L;
    pl.Upad = (int)align_up(a.U > 0 ? a.U : 1, 32);
    pl.Lp = (int)align_up(a.L, 8);
    pl.stat_chunks = ceil_div(a.L, STAT_CHUNK);
    pl.Sp = a.n_sample > 0 ? (int)align_up(a.n_sample, 64) : 0;
    pl.splits = 1;
    pl.keys_per_split = (int)align_up(a.L, 64);
    if (dtype == SF_BF16 && sparse && a.U > 0) {
        // the active pass has only B*nG independent (sample, group) problems: with fewer than one per compute unit
        // the keys are split until one workgroup per compute unit exists (256; the kernel keeps one workgroup per
        // compute unit resident, so 384 or 512 workgroups run in two rounds: measured at C5 with the key groups
        // inside a workgroup, active pass 36 us for 256 against 47 / 41 / 51 us for 384 / 512 / 1024 and 55 us for
        // 128), and only into pieces of at least four key tiles (C2, 384 keys: unsplit and without the merge launch
        // the step is 6 us shorter)
        const int64_t bg = (int64_t)a.B * a.nG;
        int want = bg >= 256 ? 1 : (int)((256 + bg - 1) / bg);
        const int max_splits = a.L / 256 > 0 ? a.L / 256 : 1;
        if (want > max_splits) want = max_splits;
        if (want > 64) want = 64;                     // the merge holds one split per lane
        if (want > 1) {
            pl.keys_per_split = (int)align_up(ceil_div(a.L, want), 64);
            pl.splits = ceil_div(a.L, pl.keys_per_split);
        }
    }
    Carver c(ws);
    const size_t BH = (size_t)a.B * a.nH, BG = (size_t)a.B * a.nG;
    pl.vt = (dtype == SF_BF16 && !a.v_transposed) ? c.take<uint16_t>(BG * a.dh * pl.Lp) : nullptr;
    pl.stat_part = c.take<float>(BG * pl.stat_chunks * 2 * a.dh);
    pl.stats = c.take<float>(BG * 2 * a.dh);
    pl.n_valid = c.take<int32_t>(a.B);
    pl.score = c.take<float>(BH * a.L);
    pl.sel = c.take<int32_t>(BH * (a.U > 0 ? a.U : 1));
    pl.slot = c.take<int32_t>(BH * a.L);
    if (pl.splits > 1) {
        pl.part_o = c.take<float>(BH * pl.Upad * pl.splits * a.dh);
        pl.part_ml = c.take<float>(BH * pl.Upad * pl.splits * 2);
    }
    if (pl.Sp > 0) {
        pl.ks = c.take<char>(BG * pl.Sp * a.dh * elem_size(dtype));
        pl.ks_valid = c.take<uint8_t>((size_t)a.B * pl.Sp);
        pl.ks_stats = c.take<float>(BG * 2 * a.dh);
        pl.n_keys = c.take<int32_t>(a.B);
    }
    pl.bytes = c.off;
    return pl;
}

int32_t attention_forward(int dtype, const AttnArgs &a, hipStream_t st)
{
    if (a.B <= 0) return SF_OK;
    if (a.L > 16384) return fail(SF_ERR_SHAPE, "sparse_gqa: L <= 16384 required");
    if (a.dh % 4 || a.ldo % 4) return fail(SF_ERR_SHAPE, "sparse_gqa: dh and ldo must be multiples of 4");
    if (dtype == SF_BF16) {
        if (a.dh != 32 && a.dh != 64 && a.dh != 128)
            return fail(SF_ERR_SHAPE, "sparse_gqa(bf16): dh must be 32, 64 or 128");
        if ((a.sq.b | a.sq.h | a.sq.l | a.sk.b | a.sk.h | a.sk.l | a.sv.b | a.sv.h | a.sv.l) % 8)
            return fail(SF_ERR_SHAPE, "sparse_gqa(bf16): strides must be multiples of 8 elements");
    } else if (a.dh > 256) {
        return fail(SF_ERR_SHAPE, "sparse_gqa(f32): dh <= 256 required");
    }
    // limits of the bf16 launchers (their 1-D grids), checked here so that nothing is enqueued when they fail
    if (dtype == SF_BF16 && a.nH > 64) return fail(SF_ERR_SHAPE, "sparse_gqa(bf16): at most 64 heads");
    if ((int64_t)a.B * a.nH * ceil_div(a.L, 32) * 64 > ((int64_t)1 << 30))
        return fail(SF_ERR_SHAPE, "sparse_gqa: too many work items (B * heads * L / 32 must stay below 2^24)");
    AttnPlan pl = attn_plan(dtype, a, a.ws);
    if (pl.bytes > 0 && (!a.ws || a.ws_bytes < pl.bytes || ((uintptr_t)a.ws & 255)))
        return fail(SF_ERR_WORKSPACE, "sparse_gqa: workspace of %zu bytes (256-byte aligned) required, got %zu",
                    pl.bytes, a.ws_bytes);

    const int BH = a.B * a.nH, BG = a.B * a.nG;
    // V as the kernels will read it
    const void *Vuse = a.V;
    sf_strides svu = a.sv;
    int vT = a.v_transposed;
    if (dtype == SF_BF16 && !a.v_transposed) {
        dim3 grid(ceil_div(pl.Lp, 32), ceil_div(a.dh, 32), BG);
        hipLaunchKernelGGL(transpose_v_kernel, grid, dim3(256), 0, st, (const uint16_t *)a.V, a.sv, a.nG,
                           a.L, a.dh, pl.Lp, (uint16_t *)pl.vt, a.row0);
        Vuse = pl.vt;
        svu.b = (int64_t)a.nG * a.dh * pl.Lp;
        svu.h = (int64_t)a.dh * pl.Lp;
        svu.l = pl.Lp;
        vT = 1;
    }
    const int64_t v_sj = vT ? 1 : svu.l, v_se = vT ? svu.l : 1;

    // 1. statistics: mean key (for the score's mean term) and context vector
    {
        int DHP = 4;
        while (DHP < a.dh) DHP *= 2;
        dim3 grid(pl.stat_chunks, BG);
        if (dtype == SF_BF16 && vT && a.dh == 32)
            hipLaunchKernelGGL(kv_stats_partial_bf16_kernel<32>, grid, dim3(256), 0, st, (const h16 *)a.K, a.sk,
                               (const h16 *)Vuse, svu, a.key_valid, a.nG, a.L, pl.stat_part, a.row0);
        else if (dtype == SF_BF16 && vT && a.dh == 64)
            hipLaunchKernelGGL(kv_stats_partial_bf16_kernel<64>, grid, dim3(256), 0, st, (const h16 *)a.K, a.sk,
                               (const h16 *)Vuse, svu, a.key_valid, a.nG, a.L, pl.stat_part, a.row0);
        else if (dtype == SF_BF16 && vT && a.dh == 128)
            hipLaunchKernelGGL(kv_stats_partial_bf16_kernel<128>, grid, dim3(256), 0, st, (const h16 *)a.K, a.sk,
                               (const h16 *)Vuse, svu, a.key_valid, a.nG, a.L, pl.stat_part, a.row0);
        else if (dtype == SF_BF16)
            hipLaunchKernelGGL(kv_stats_partial_kernel<h16>, grid, dim3(256), 0, st, (const h16 *)a.K,
                               a.sk, (const h16 *)Vuse, svu, v_sj, v_se, a.key_valid, a.nG, a.L, a.dh,
                               DHP, pl.stat_part, a.row0, vT ? nullptr : a.row0);
        else
            hipLaunchKernelGGL(kv_stats_partial_kernel<float>, grid, dim3(256), 0, st, (const float *)a.K,
                               a.sk, (const float *)Vuse, svu, v_sj, v_se, a.key_valid, a.nG, a.L, a.dh,
                               DHP, pl.stat_part, a.row0, vT ? nullptr : a.row0);
        hipLaunchKernelGGL(kv_stats_final_kernel, dim3(BG), dim3(256), 0, st, pl.stat_part, pl.stat_chunks,
                           a.key_valid, a.nG, a.L, a.dh, pl.stats, pl.n_valid, a.act_bits);
    }

    // 2. active set
    const int userH = a.selH > 0 ? a.selH : a.nH;
    int32_t *sel = a.sel_out ? a.sel_out : pl.sel;
    const int selH = a.sel_out ? userH : a.nH;
    if (a.forced_sel && a.U > 0) {
        hipLaunchKernelGGL(forced_slot_kernel, dim3(BH), dim3(256), 0, st, a.forced_sel, userH, a.nH, a.L, a.U,
                           sel, selH, pl.slot, a.act_bits);
    } else {
        const float *M = nullptr;
        int scoreH = a.nH;
        if (a.U > 0 && a.U < a.L) {
            float *score = a.score_out ? a.score_out : pl.score;
            scoreH = a.score_out ? userH : a.nH;
            // keys the score looks at: the sample's own keys, or the gathered key sample
            const void *Kx = a.K;
            sf_strides skx = a.sk;
            int Lk = a.L;
            const uint8_t *key_mask = a.key_valid;
            const float *kstats = pl.stats;
            const int32_t *nkeys = pl.n_valid;
            if (a.sample_idx && pl.Sp > 0) {
                const size_t gl = (size_t)ceil_div(a.L, 32) * 4 + (size_t)pl.Sp * 4;
                if (dtype == SF_BF16)
                    hipLaunchKernelGGL(gather_key_sample_kernel<h16>, dim3(BG), dim3(256), gl, st,
                                       (const h16 *)a.K, a.sk, a.key_valid, a.sample_idx, a.n_sample, a.nG, a.L,
                                       a.dh, pl.Sp, (h16 *)pl.ks, pl.ks_valid, pl.ks_stats, pl.n_keys, a.row0);
                else
                    hipLaunchKernelGGL(gather_key_sample_kernel<float>, dim3(BG), dim3(256), gl, st,
                                       (const float *)a.K, a.sk, a.key_valid, a.sample_idx, a.n_sample, a.nG, a.L,
                                       a.dh, pl.Sp, (float *)pl.ks, pl.ks_valid, pl.ks_stats, pl.n_keys, a.row0);
                Kx = pl.ks;
                skx.b = (int64_t)a.nG * pl.Sp * a.dh; skx.h = (int64_t)pl.Sp * a.dh; skx.l = a.dh;
                Lk = pl.Sp; key_mask = pl.ks_valid; kstats = pl.ks_stats; nkeys = pl.n_keys;
            }
            if (dtype == SF_BF16) {
                if (int32_t rc = score_bf16(a, Kx, skx, Lk, key_mask, kstats, score, scoreH, st)) return rc;
            } else {
                dim3 grid(ceil_div(a.L, 256), BH);
                hipLaunchKernelGGL(score_f32_kernel, grid, dim3(256), 0, st, (const float *)a.Q, a.sq,
                                   (const float *)Kx, skx, a.head_group, a.hg_stride, a.pattern_id,
                                   a.key_valid, key_mask, nkeys, a.nH, a.L, Lk, a.dh, score, scoreH, a.row0,
                                   Kx == a.K);
            }
            M = score;
        }
        // few blocks (one per sample and head): long rows get 1024 threads so that a radix pass is 4 keys per thread
        if (a.L >= 2048)
            hipLaunchKernelGGL(select_kernel<1024>, dim3(BH), dim3(1024), a.L * sizeof(uint32_t), st, M, scoreH,
                               a.key_valid, a.nH, a.L, a.U, a.u_active, sel, selH, pl.slot, a.act_bits);
        else
            hipLaunchKernelGGL(select_kernel<256>, dim3(BH), dim3(256), a.L * sizeof(uint32_t), st, M, scoreH,
                               a.key_valid, a.nH, a.L, a.U, a.u_active, sel, selH, pl.slot, a.act_bits);
    }

    // 3. active rows
    if (a.U > 0) {
        if (dtype == SF_BF16) {
            if (int32_t rc = attend_bf16(a, pl, Vuse, svu, sel, selH, st)) return rc;
        } else {
            dim3 grid(a.U, BH);
            hipLaunchKernelGGL(attend_f32_kernel, grid, dim3(64), a.L * sizeof(float), st, (const float *)a.Q,
                               a.sq, (const float *)a.K, a.sk, (const float *)Vuse, svu, v_sj, v_se,
                               a.head_group, a.hg_stride, a.pattern_id, a.key_valid, sel, selH, a.nH, a.L,
                               a.dh, a.U, (float *)a.O, a.ldo, a.row0);
        }
    }

    // 4. merge of the key splits, then the lazy rows
    if (pl.splits > 1) {
        const int64_t n_waves = (int64_t)BH * a.U;
        hipLaunchKernelGGL(merge_splits_kernel<h16>, dim3((unsigned)((n_waves + 3) / 4)), dim3(256), 0, st,
                           a.nH, a.L, a.dh, a.U, pl.Upad, pl.splits, n_waves, sel, selH, pl.part_o, pl.part_ml,
                           (h16 *)a.O, a.ldo, a.row0);
    }
    if (!a.skip_fill) {   // with U == L rows can still be lazy (fewer allowed rows than U)
        const bool v8 = dtype == SF_BF16 && a.dh % 8 == 0 && a.ldo % 8 == 0 && ((uintptr_t)a.O % 16 == 0);
        // packed samples: a sample may own up to 2 * 256 + L rows of padding behind its tokens
        dim3 grid(ceil_div(a.ext ? 2 * a.L + 512 : a.L, FILL_ROWS), a.B);
        const size_t fl = (size_t)a.nH * a.dh * 4 + (size_t)a.nH * FILL_ROWS * 4;
#define SF_FILL_ARGS grid, dim3(256), fl, st, a.nH, a.nG, a.L, a.dh, pl.slot, a.head_group, a.hg_stride, \
                     a.pattern_id, pl.stats
        if (dtype == SF_BF16 && v8) hipLaunchKernelGGL((fill_kernel<h16, 8>), SF_FILL_ARGS, (h16 *)a.O, a.ldo, a.row0, a.ext);
        else if (dtype == SF_BF16) hipLaunchKernelGGL((fill_kernel<h16, 4>), SF_FILL_ARGS, (h16 *)a.O, a.ldo, a.row0, a.ext);
        else hipLaunchKernelGGL((fill_kernel<float, 4>), SF_FILL_ARGS, (float *)a.O, a.ldo, a.row0, a.ext);
#undef SF_FILL_ARGS
    }
    return check_launch("sparse_gqa_forward");
}

}  // namespace sf

using namespace sf;

static int32_t make_attn_args(const sf_desc *desc, int32_t nH, int32_t nG, Dims &D, AttnArgs &a)
{
    if (int32_t rc = read_desc(desc, D)) return rc;
    if (nH < 1 || nG < 1) return fail(SF_ERR_INVALID_ARG, "sparse_gqa: nH and nG must be positive");
    a = AttnArgs{};
    a.B = D.B; a.nH = nH; a.nG = nG; a.L = D.L; a.dh = D.dh; a.U = D.U; a.n_sample = D.n_sample;
    return SF_OK;
}

extern "C" size_t sf_sparse_gqa_workspace_bytes(const sf_desc *desc, int32_t nH, int32_t nG)
{
    Dims D; AttnArgs a;
    if (make_attn_args(desc, nH, nG, D, a)) return 0;
    a.v_transposed = 0;       // the larger of the two cases
    return attn_plan(D.dtype, a, nullptr).bytes;
}

extern "C" int32_t sf_sparse_gqa_forward(const sf_desc *desc, int32_t nH, int32_t nG, const void *Q,
                                         sf_strides sq, const void *K, sf_strides sk, const void *V,
                                         sf_strides sv, int32_t v_transposed, const int32_t *head_group,
                                         const int32_t *pattern_id, const uint8_t *key_valid,
                                         const int32_t *sample_idx, const int32_t *forced_sel, void *O,
                                         int64_t ldo, int32_t *sel_out,
                                         float *score_out, void *workspace, size_t workspace_bytes,
                                         void *stream)
{
    Dims D; AttnArgs a;
    if (int32_t rc = make_attn_args(desc, nH, nG, D, a)) return rc;
    if (!Q || !K || !V || !head_group || !O) return fail(SF_ERR_INVALID_ARG, "sparse_gqa: NULL argument");
    if (ldo < (int64_t)nH * D.dh) return fail(SF_ERR_SHAPE, "sparse_gqa: ldo smaller than nH*dh");
    a.Q = Q; a.K = K; a.V = V; a.sq = sq; a.sk = sk; a.sv = sv; a.v_transposed = v_transposed != 0;
    a.head_group = head_group; a.hg_stride = nH; a.pattern_id = pattern_id; a.key_valid = key_valid;
    a.sample_idx = D.n_sample > 0 ? sample_idx : nullptr;
    a.forced_sel = forced_sel; a.O = O; a.ldo = ldo; a.sel_out = sel_out; a.score_out = score_out;
    a.ws = workspace; a.ws_bytes = workspace_bytes;
    return attention_forward(D.dtype, a, static_cast<hipStream_t>(stream));
}

// ---- sparse_gqa_forward for callers that cannot allocate --------------------------------------------------------
// The same launches as sf_sparse_gqa_forward with the workspace taken from a file-scope device array instead of a
// caller's buffer.  Every GPU the library runs on holds its own copy of the array at its own address until the
// process ends; the array's name is only a host-side handle, so its device address is looked up once per device
// (with that device current) and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[SF_STATIC_SCRATCH_BYTES];

static int32_t static_scratch(void **out)
{
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static void *per_device[MAX_DEV] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV)
        return fail(SF_ERR_HIP, "sparse_gqa_static: no current device (or device index >= %d)", MAX_DEV);
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(SF_ERR_HIP, "sparse_gqa_static: hipGetSymbolAddress failed on device %d: %s", dev,
                        hipGetErrorString(e));
        per_device[dev] = p;
    }
    *out = per_device[dev];
    return SF_OK;
}

extern "C" size_t sf_sparse_gqa_static_capacity(void) { return SF_STATIC_SCRATCH_BYTES; }

extern "C" int32_t sf_sparse_gqa_forward_static(const sf_desc *desc, int32_t nH, int32_t nG, const void *Q,
                                                sf_strides sq, const void *K, sf_strides sk, const void *V,
                                                sf_strides sv, int32_t v_transposed, const int32_t *head_group,
                                                const int32_t *pattern_id, const uint8_t *key_valid,
                                                const int32_t *sample_idx, const int32_t *forced_sel, void *O,
                                                int64_t ldo, int32_t *sel_out, float *score_out, void *stream)
{
    Dims D; AttnArgs a;
    if (int32_t rc = make_attn_args(desc, nH, nG, D, a)) return rc;
    a.v_transposed = v_transposed != 0;
    const size_t need = attn_plan(D.dtype, a, nullptr).bytes;
    if (need > SF_STATIC_SCRATCH_BYTES)
        return fail(SF_ERR_WORKSPACE,
                    "sparse_gqa_static: this problem needs %zu bytes of scratch, the built-in buffer holds %zu; use "
                    "sf_sparse_gqa_forward with a workspace of sf_sparse_gqa_workspace_bytes()",
                    need, (size_t)SF_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    if (int32_t rc = static_scratch(&ws)) return rc;
    // Nothing in the buffer has to start at zero: every piece (transposed V, K/V statistics, scores, active lists,
    // row -> slot map, key-split partials) is written in full by an earlier kernel of the same call before a later
    // one reads it, exactly as with a caller's uninitialised workspace.
    return sf_sparse_gqa_forward(desc, nH, nG, Q, sq, K, sk, V, sv, v_transposed, head_group, pattern_id, key_valid,
                                 sample_idx, forced_sel, O, ldo, sel_out, score_out, ws, SF_STATIC_SCRATCH_BYTES, stream);
}
