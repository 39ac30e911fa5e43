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
#include <type_traits>

#include <atomic>

#include "gemm.hpp"

namespace sf {

constexpr int FBK = 64;
constexpr int N_XCD = 8;

template <int ACT>
__device__ __forceinline__ float fact(float z)
{
    if (ACT == ACT_RELU) return z > 0.f ? z : 0.f;
    if (ACT == ACT_GELU) return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
    return z;
}

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

// LDS layout of a [rows][BKT] bf16 tile.  The LDS serves 16 lanes of a
// ds_read_b128 per cycle (256 bytes), so 16 consecutive rows of one logical
// 16-byte chunk must fall into 16 different 16-byte slots modulo 256 bytes:
// rows are packed into 256-byte super-rows and the slot is XOR-ed with the
// super-row number.
template <int BKT>
struct Lay {
    static constexpr int CH = BKT / 8;          // 16-byte chunks per row
    static constexpr int RPS = 16 / CH;         // rows per super-row
    __device__ __forceinline__ static int off(int row, int chunk)      // element offset
    {
        const int sr = row / RPS;
        const int pos = ((row % RPS) * CH + chunk) ^ (sr % CH);
        return sr * 128 + pos * 8;
    }
};

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// One workgroup per CU (its LDS tiles take most of the 160 KB), so a wave may use
// 512 / (waves per SIMD) registers: say so, or the accumulators spill.
template <int WAVES_M, int WAVES_N, int TM, int TN, int BKT, int NSTAGE, bool SWAP, int ACT>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N)
__attribute__((amdgpu_waves_per_eu(WAVES_M * WAVES_N / 4,
                                   (WAVES_M * WAVES_N * TM * TN >= 64) ? WAVES_M * WAVES_N / 4 : 2)))
void gemm_bf16_fast_kernel(GemmArgs a, int tiles_m, int tiles_n, int total_tiles, int per_xcd)
{
    using L = Lay<BKT>;
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    constexpr int ROWS_PER_LOAD = 4 * L::RPS;             // one load instruction fills 4 super-rows (1 KB)
    constexpr int LX = BM / ROWS_PER_LOAD / NW;           // load instructions per wave per K tile: X rows
    constexpr int LW = BN / ROWS_PER_LOAD / NW;           //                                          W rows
    constexpr int LPW = LX + LW;
    constexpr int STAGE = (BM + BN) * BKT;                // elements per stage
    static_assert(BM % (ROWS_PER_LOAD * NW) == 0 && BN % (ROWS_PER_LOAD * NW) == 0, "loads must divide among the waves");
    static_assert(NSTAGE >= 2 && NSTAGE <= 4 && (NSTAGE - 2) * LPW <= 63, "pipeline depth");

    extern __shared__ __attribute__((aligned(16))) char smem_raw[];
    h16 *smem = reinterpret_cast<h16 *>(smem_raw);      // [NSTAGE][X rows | W rows][BKT]

    // XCD-aware tile order
    const int wid = blockIdx.x;
    const int w = (wid % N_XCD) * per_xcd + wid / N_XCD;
    if (w >= total_tiles) return;
    const int tn_i = w % tiles_n, tm_i = w / tiles_n;
    const int b = tm_i / tiles_m;
    const int m0 = (tm_i % tiles_m) * BM;
    const int nt0 = tn_i * BN;
    const int p = a.pattern_id ? a.pattern_id[b] : 0;
    if (p < 0) return;                                             // sample not in use
    if (a.n_lim) a.N = min(a.N, a.n_lim[p]);
    if (a.k_lim) a.K = min(a.K, a.k_lim[p]);
    if (nt0 >= a.N) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: keeps LDS bases in SGPRs
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int l32 = lane & 31, lhi = lane >> 5;

    // Sources of this wave's load instructions: a uniform base that advances by BKT per K
    // tile plus a fixed per-lane byte offset.  Lane -> LDS slot is fixed (lane*16 bytes), so
    // the slot's (row, chunk) is decoded here; rows beyond the edge are clamped.
    const char *Ab = reinterpret_cast<const char *>(static_cast<const h16 *>(a.A) + ((int64_t)b * a.L + m0) * a.lda);
    const char *Wb = reinterpret_cast<const char *>(static_cast<const h16 *>(a.W) + (int64_t)p * a.w_pstride +
                                                    (int64_t)(a.n0 + nt0) * a.ldw);
    uint32_t xoff[LX], woff[LW];
    {
        const int srl = lane >> 4;                            // super-row within the instruction
        const int rows_x = min(BM, a.L - m0), rows_w = min(BN, a.N - nt0);
#pragma unroll
        for (int j = 0; j < LX; ++j) {
            const int sr = (wave + j * NW) * 4 + srl;
            const int t = (lane & 15) ^ (sr % L::CH);
            const int r = min(sr * L::RPS + t / L::CH, rows_x - 1);
            xoff[j] = (uint32_t)(r * (int)a.lda + (t % L::CH) * 8) * 2u;
        }
#pragma unroll
        for (int j = 0; j < LW; ++j) {
            const int sr = (wave + j * NW) * 4 + srl;
            const int t = (lane & 15) ^ (sr % L::CH);
            const int r = min(sr * L::RPS + t / L::CH, rows_w - 1);
            woff[j] = (uint32_t)(r * (int)a.ldw + (t % L::CH) * 8) * 2u;
        }
    }
    // load instruction j (0..LPW-1) of K tile `tile` into ring slot `stage`
    auto issue_load = [&](int j, int tile, int stage) {
        h16 *base = smem + stage * STAGE;
        const int64_t koff = (int64_t)tile * BKT * 2;
        if (j < LX) {
            __builtin_amdgcn_global_load_lds((glb_void *)(Ab + koff + xoff[j]),
                                             (lds_void *)(base + (wave + j * NW) * 512), 16, 0, 0);
        } else {
            const int jw = j - LX;
            __builtin_amdgcn_global_load_lds((glb_void *)(Wb + koff + woff[jw]),
                                             (lds_void *)(base + BM * BKT + (wave + jw * NW) * 512), 16, 0, 0);
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

    constexpr int KS = BKT / 16;                  // MFMA k-steps per K tile
    constexpr int LPS = LPW / KS;                 // load instructions issued per k-step
    static_assert(LPW % KS == 0, "loads must divide among the k-steps");

    // One K tile: the fragments of k-step s+1 are read while the MFMAs of k-step s issue, and
    // the direct-to-LDS loads of a younger tile are spread over the k-steps (a burst of loads at
    // the top of the iteration stalls instruction issue until the address unit has taken them).
    auto k_tile = [&](int kt, auto with_loads) {
        constexpr bool LOADS = decltype(with_loads)::value;
        const h16 *xs = smem + (kt % NSTAGE) * STAGE;
        const h16 *ws = xs + BM * BKT;
        const int load_tile = kt + NSTAGE - 1, load_stage = load_tile % NSTAGE;
        h16x8 xf[2][TM], wf[2][TN];
        auto load_frags = [&](int s, int slot) {
            const int chunk = s * 2 + lhi;
#pragma unroll
            for (int t = 0; t < TM; ++t)
                xf[slot][t] = *reinterpret_cast<const h16x8 *>(xs + L::off((wm * TM + t) * 32 + l32, chunk));
#pragma unroll
            for (int t = 0; t < TN; ++t)
                wf[slot][t] = *reinterpret_cast<const h16x8 *>(ws + L::off((wn * TN + t) * 32 + l32, chunk));
        };
        load_frags(0, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (s + 1 < KS) load_frags(s + 1, (s + 1) & 1);
            if (LOADS) {
#pragma unroll
                for (int j = 0; j < LPS; ++j) issue_load(s * LPS + j, load_tile, load_stage);
            }
#pragma unroll
            for (int i = 0; i < TP; ++i)
#pragma unroll
                for (int j = 0; j < TQ; ++j) {
                    if (SWAP) acc[i][j] = SF_MFMA16(xf[s & 1][i], wf[s & 1][j], acc[i][j], 0, 0, 0);
                    else      acc[i][j] = SF_MFMA16(wf[s & 1][i], xf[s & 1][j], acc[i][j], 0, 0, 0);
                }
            // pin the interleaving: MFMA, LDS read, MFMA, LDS read, ..., the global loads last
            constexpr int NMFMA = TP * TQ, NVM = LOADS ? LPS : 0;
            const int NDS = (s + 1 < KS) ? TM + TN : 0;
#pragma unroll
            for (int i = 0; i < NMFMA; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                         // one MFMA
                if (i < NDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);            // one LDS read
                if (i >= NMFMA - NVM) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // one global load
            }
        }
    };

    // NSTAGE-deep ring: tile kt+NSTAGE-1 is requested while tile kt is consumed
    const int nk = a.K / BKT;
    for (int t = 0; t < NSTAGE - 1 && t < nk; ++t) {
#pragma unroll
        for (int j = 0; j < LPW; ++j) issue_load(j, t, t);
    }
    const int n_main = nk - (NSTAGE - 1);         // iterations that still have a tile to request
    int kt = 0;
    for (; kt < n_main; ++kt) {
        wait_vmcnt<(NSTAGE - 2) * LPW>();         // tile kt has landed; NSTAGE-2 younger tiles stay in flight
        __syncthreads();                          // ... for every wave; and everyone is done with tile kt-1
        k_tile(kt, std::true_type{});
    }
    for (; kt < nk; ++kt) {
        const int younger = nk - 1 - kt;
        if (NSTAGE >= 4 && younger >= 2) wait_vmcnt<2 * LPW>();
        else if (NSTAGE >= 3 && younger >= 1) wait_vmcnt<LPW>();
        else wait_vmcnt<0>();
        __syncthreads();
        k_tile(kt, std::false_type{});
    }

    // ---- epilogue -------------------------------------------------------------
    const h16 *bias = a.bias ? static_cast<const h16 *>(a.bias) + (int64_t)p * a.bias_pstride + a.n0 : nullptr;
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
                        const h16x8 bv = *reinterpret_cast<const h16x8 *>(bias + n);
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
                            const h16x8 rv = *reinterpret_cast<const h16x8 *>(static_cast<const h16 *>(a.R) + ro);
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
                        h16x8 o;
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] = (h16)v[e];
                        *reinterpret_cast<h16x8 *>(static_cast<h16 *>(a.C) + co) = o;
                    }
                }
            }
        }
    } else {
        // transposed store: lane owns feature n and, after the swap, 8 consecutive tokens
        h16 *C = static_cast<h16 *>(a.C) + (int64_t)b * a.vt_b;
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
                    h16x8 o;
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = (h16)fact<ACT>(v[e] + bv);
                    h16 *dst = C + (int64_t)n * a.vt_n + i;
                    if (i + 7 < a.L) {
                        *reinterpret_cast<h16x8 *>(dst) = o;       // vt_b, vt_n % 8 == 0 checked on the host
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

template <int WAVES_M, int WAVES_N, int TM, int TN, int BKT, int NSTAGE, bool SWAP, int ACT>
static int32_t launch_fast(const GemmArgs &a, hipStream_t st)
{
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    auto kern = gemm_bf16_fast_kernel<WAVES_M, WAVES_N, TM, TN, BKT, NSTAGE, SWAP, ACT>;
    constexpr size_t lds = (size_t)NSTAGE * (BM + BN) * BKT * sizeof(h16);
    static std::atomic<bool> attr_set{false};     // per template instance; setting the attribute twice is harmless
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

#define SMALLCFG 2, 2, 2, 2, 64, 2

#define BIGCFG 2, 4, 4, 2, 64, 2
template <bool SWAP, int ACT>
static int32_t launch_big(const GemmArgs &a, hipStream_t st)
{
    return launch_fast<BIGCFG, SWAP, ACT>(a, st);
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
        if (big) return launch_big<true, ACT_NONE>(a, st);
        return launch_fast<SMALLCFG, true, ACT_NONE>(a, st);
    }
    switch (a.act) {
    case ACT_RELU:
        return big ? launch_big<false, ACT_RELU>(a, st) : launch_fast<SMALLCFG, false, ACT_RELU>(a, st);
    case ACT_GELU:
        return big ? launch_big<false, ACT_GELU>(a, st) : launch_fast<SMALLCFG, false, ACT_GELU>(a, st);
    default:
        return big ? launch_big<false, ACT_NONE>(a, st) : launch_fast<SMALLCFG, false, ACT_NONE>(a, st);
    }
}

}  // namespace sf
