// Throughput variant of the bf16 MFMA GEMM (see gemm_bf16.hip for the role of
// the GEMM in the pruned encoder layer).  Requirements: K % 64 == 0.
//
// What is specific to gfx950 here:
//  * tiles go HBM/L2 -> LDS with direct-to-LDS loads (global_load_lds_dwordx4):
//    no staging registers, no ds_write; a wave fills 8 rows x 128 B per
//    instruction.  The LDS slot is fixed by the lane, so the XOR swizzle that
//    keeps the 16-byte fragment reads conflict-free is applied to the GLOBAL
//    address instead (lane -> logical chunk = physical chunk ^ (row & 7));
//  * out-of-range rows are clamped, not zero-filled: they only feed outputs
//    that are never stored;
//  * MFMA fragments are double-buffered in registers so the LDS reads of
//    k-step s+1 are in flight while the MFMAs of k-step s issue;
//  * workgroup ids are remapped so that each XCD (own L2) walks a contiguous
//    range of tiles, N fastest: the activation tile is fetched once per XCD and
//    the weight matrix stays resident in that L2;
//  * the epilogue pairs lane l with lane l+32 (v_permlane32_swap) so that each
//    lane owns 8 consecutive features of a token: 16-byte stores.
#include "gemm.hpp"

namespace sf {

constexpr int FBK = 64;
constexpr int N_XCD = 8;

__device__ __forceinline__ int fswz(int row, int chunk) { return row * FBK + ((chunk ^ (row & 7)) << 3); }

template <int ACT>
__device__ __forceinline__ float fact(float z)
{
    if (ACT == ACT_RELU) return z > 0.f ? z : 0.f;
    if (ACT == ACT_GELU) return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
    return z;
}

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

template <int WAVES_M, int WAVES_N, int TM, int TN, bool SWAP, int ACT>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_fast_kernel(GemmArgs a, int tiles_m, int tiles_n,
                                                                                 int total_tiles, int per_xcd)
{
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    constexpr int RG = (BM + BN) / 8;               // 8-row groups per K tile (one load instruction each)
    constexpr int LPW = RG / NW;                    // load instructions per wave per K tile
    static_assert(RG % NW == 0, "row groups must divide among the waves");

    extern __shared__ __attribute__((aligned(16))) char smem_raw[];
    __bf16 *smem = reinterpret_cast<__bf16 *>(smem_raw);      // [2][(BM+BN)*FBK]: X rows then W rows

    // XCD-aware tile order
    const int wid = blockIdx.x;
    const int w = (wid % N_XCD) * per_xcd + wid / N_XCD;
    if (w >= total_tiles) return;
    const int tn_i = w % tiles_n, tm_i = w / tiles_n;
    const int b = tm_i / tiles_m;
    const int m0 = (tm_i % tiles_m) * BM;
    const int nt0 = tn_i * BN;
    const int p = a.pattern_id ? a.pattern_id[b] : 0;

    const __bf16 *A = static_cast<const __bf16 *>(a.A) + ((int64_t)b * a.L) * a.lda;
    const __bf16 *W = static_cast<const __bf16 *>(a.W) + (int64_t)p * a.w_pstride + (int64_t)a.n0 * a.ldw;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int l32 = lane & 31, lhi = lane >> 5;

    // per-lane source pointers of this wave's load instructions (advanced by FBK per K tile)
    const __bf16 *src[LPW];
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
        const int rg = wave + j * NW;
        const int r = rg * 8 + (lane >> 3);          // row within [X rows | W rows]
        const int c = (lane & 7) ^ (r & 7);          // logical chunk that must land in physical chunk lane&7
        if (rg < BM / 8) {
            const int i = min(m0 + r, a.L - 1);
            src[j] = A + (int64_t)i * a.lda + c * 8;
        } else {
            const int n = min(nt0 + r - BM, a.N - 1);
            src[j] = W + (int64_t)n * a.ldw + c * 8;
        }
    }
    auto issue_loads = [&](int buf) {
        __bf16 *base = smem + buf * (BM + BN) * FBK;
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            const int rg = wave + j * NW;
            __builtin_amdgcn_global_load_lds((glb_void *)src[j], (lds_void *)(base + rg * 8 * FBK), 16, 0, 0);
            src[j] += FBK;
        }
    };

    constexpr int TP = SWAP ? TM : TN, TQ = SWAP ? TN : TM;
    f32x16 acc[TP][TQ];
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int nk = a.K / FBK;
    issue_loads(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) issue_loads((kt + 1) & 1);
        const __bf16 *xs = smem + (kt & 1) * (BM + BN) * FBK;
        const __bf16 *ws = xs + BM * FBK;
        bf16x8 xf[2][TM], wf[2][TN];
        auto load_frags = [&](int s, int slot) {
            const int chunk = s * 2 + lhi;
#pragma unroll
            for (int t = 0; t < TM; ++t)
                xf[slot][t] = *reinterpret_cast<const bf16x8 *>(xs + fswz((wm * TM + t) * 32 + l32, chunk));
#pragma unroll
            for (int t = 0; t < TN; ++t)
                wf[slot][t] = *reinterpret_cast<const bf16x8 *>(ws + fswz((wn * TN + t) * 32 + l32, chunk));
        };
        load_frags(0, 0);
#pragma unroll
        for (int s = 0; s < FBK / 16; ++s) {
            if (s + 1 < FBK / 16) load_frags(s + 1, (s + 1) & 1);
#pragma unroll
            for (int i = 0; i < TP; ++i)
#pragma unroll
                for (int j = 0; j < TQ; ++j) {
                    if (SWAP) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[s & 1][i], wf[s & 1][j], acc[i][j], 0, 0, 0);
                    else      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[s & 1][i], xf[s & 1][j], acc[i][j], 0, 0, 0);
                }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }

    // ---- epilogue -------------------------------------------------------------
    const __bf16 *bias = a.bias ? static_cast<const __bf16 *>(a.bias) + (int64_t)p * a.bias_pstride + a.n0 : nullptr;
    if (!SWAP) {
        // accumulator entry q*4+e of lane (l32, lhi): token l32, feature q*8 + lhi*4 + e.
        // After swapping halves, lanes < 32 own features [q0*8, q0*8+8) and lanes >= 32 own
        // [q1*8, q1*8+8) of the same token, for the pairs (q0,q1) = (0,1), (2,3).
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int i = m0 + (wm * TM + tm) * 32 + l32;
            const int64_t row = (int64_t)b * a.L + i;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
                for (int qp = 0; qp < 2; ++qp) {
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[tn][tm][(2 * qp) * 4 + e]),
                                                                        __float_as_uint(acc[tn][tm][(2 * qp + 1) * 4 + e]),
                                                                        false, false);
                        v[e] = __uint_as_float(r[0]);
                        v[4 + e] = __uint_as_float(r[1]);
                    }
                    const int n = nt0 + (wn * TN + tn) * 32 + (2 * qp + lhi) * 8;
                    if (i >= a.L || n >= a.N) continue;       // N % 8 == 0: a group of 8 is all in or all out
                    if (bias) {
                        const bf16x8 bv = *reinterpret_cast<const bf16x8 *>(bias + n);
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] += (float)bv[e];
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = fact<ACT>(v[e]);
                    if (a.R) {
                        const int64_t ro = row * a.ldr + a.r0 + n;
                        if (a.r_f32) {
                            const float *R = static_cast<const float *>(a.R) + ro;
                            const f32x4 r0 = *reinterpret_cast<const f32x4 *>(R), r1 = *reinterpret_cast<const f32x4 *>(R + 4);
#pragma unroll
                            for (int e = 0; e < 4; ++e) { v[e] += r0[e]; v[4 + e] += r1[e]; }
                        } else {
                            const bf16x8 rv = *reinterpret_cast<const bf16x8 *>(static_cast<const __bf16 *>(a.R) + ro);
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] += (float)rv[e];
                        }
                    }
                    const int64_t co = row * a.ldc + a.c0 + n;
                    if (a.c_f32) {
                        float *C = static_cast<float *>(a.C) + co;
                        f32x4 o0, o1;
#pragma unroll
                        for (int e = 0; e < 4; ++e) { o0[e] = v[e]; o1[e] = v[4 + e]; }
                        *reinterpret_cast<f32x4 *>(C) = o0;
                        *reinterpret_cast<f32x4 *>(C + 4) = o1;
                    } else {
                        bf16x8 o;
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] = (__bf16)v[e];
                        *reinterpret_cast<bf16x8 *>(static_cast<__bf16 *>(a.C) + co) = o;
                    }
                }
            }
        }
    } else {
        // transposed store: lane owns feature n and, after the swap, 8 consecutive tokens
        __bf16 *C = static_cast<__bf16 *>(a.C) + (int64_t)b * a.vt_b;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int n = nt0 + (wn * TN + tn) * 32 + l32;
            const float bv = (bias && n < a.N) ? (float)bias[n] : 0.f;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
                for (int qp = 0; qp < 2; ++qp) {
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[tm][tn][(2 * qp) * 4 + e]),
                                                                        __float_as_uint(acc[tm][tn][(2 * qp + 1) * 4 + e]),
                                                                        false, false);
                        v[e] = __uint_as_float(r[0]);
                        v[4 + e] = __uint_as_float(r[1]);
                    }
                    const int i = m0 + (wm * TM + tm) * 32 + (2 * qp + lhi) * 8;
                    if (n >= a.N || i >= a.L) continue;
                    bf16x8 o;
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = (__bf16)fact<ACT>(v[e] + bv);
                    __bf16 *dst = C + (int64_t)n * a.vt_n + i;
                    if (i + 7 < a.L) {
                        *reinterpret_cast<bf16x8 *>(dst) = o;       // vt_b, vt_n % 8 == 0 checked on the host
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (i + e < a.L) dst[e] = o[e];
                    }
                }
            }
        }
    }
}

template <int WAVES_M, int WAVES_N, int TM, int TN, bool SWAP, int ACT>
static int32_t launch_fast(const GemmArgs &a, hipStream_t st)
{
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    auto kern = gemm_bf16_fast_kernel<WAVES_M, WAVES_N, TM, TN, SWAP, ACT>;
    constexpr size_t lds = (size_t)2 * (BM + BN) * FBK * sizeof(__bf16);
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return fail(SF_ERR_HIP, "gemm: cannot reserve %zu bytes of LDS", lds);
        attr_set = true;
    }
    const int tiles_m = ceil_div(a.L, BM), tiles_n = ceil_div(a.N, BN);
    const int total = a.B * tiles_m * tiles_n;
    const int per_xcd = ceil_div(total, N_XCD);
    ProfScope prof(SF_KERNEL_GEMM, st);
    hipLaunchKernelGGL(kern, dim3(per_xcd * N_XCD), dim3(64 * WAVES_M * WAVES_N), lds, st, a, tiles_m, tiles_n,
                       total, per_xcd);
    return SF_OK;
}

// Returns SF_OK and sets `done` when the fast kernel took the problem.
int32_t gemm_bf16_fast(const GemmArgs &a, hipStream_t st, bool &done)
{
    done = false;
    if (a.K % FBK || a.K < FBK || a.N % 8 || a.n0 % 8 || a.lda % 8 || a.ldw % 8) return SF_OK;
    if (a.R && (a.ldr % 8 || a.r0 % 8)) return SF_OK;
    const bool swap = a.epi == EPI_VT;
    if (swap) {
        if (a.R || a.c_f32 || ((a.vt_b | a.vt_n) & 7)) return SF_OK;
    } else if (a.ldc % 8 || a.c0 % 8) {
        return SF_OK;
    }
    const int64_t rows = (int64_t)a.B * a.L;
    if (a.L < 128 || rows * a.N < (int64_t)128 * 128 * 64) return SF_OK;     // tiny problems: generic kernel
    done = true;
    const bool big = a.L >= 192 && a.N >= 192;
    if (swap) {
        if (a.act != ACT_NONE) { done = false; return SF_OK; }
        if (big) return launch_fast<2, 4, 4, 2, true, ACT_NONE>(a, st);
        return launch_fast<2, 2, 2, 2, true, ACT_NONE>(a, st);
    }
    switch (a.act) {
    case ACT_RELU:
        return big ? launch_fast<2, 4, 4, 2, false, ACT_RELU>(a, st) : launch_fast<2, 2, 2, 2, false, ACT_RELU>(a, st);
    case ACT_GELU:
        return big ? launch_fast<2, 4, 4, 2, false, ACT_GELU>(a, st) : launch_fast<2, 2, 2, 2, false, ACT_GELU>(a, st);
    default:
        return big ? launch_fast<2, 4, 4, 2, false, ACT_NONE>(a, st) : launch_fast<2, 2, 2, 2, false, ACT_NONE>(a, st);
    }
}

}  // namespace sf
