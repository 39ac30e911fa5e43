// bf16 MFMA GEMM (fp32 accumulate) for the Q/K/V, output and FFN projections
// of the pruned encoder layer (Sec. 4.4 projections, Sec. 4.5 compacted
// weights).  Both operands are K-contiguous (token-major activations,
// unit-major weights), so every MFMA fragment is one 16-byte LDS read.
//
// Tiling: a workgroup owns a BM x BN output tile of ONE sample (rows never
// straddle samples, because the weight set depends on the sample's presence
// pattern); K is walked in steps of 64 through double-buffered, XOR-swizzled
// LDS tiles; each 64-lane wave owns a (BM/WAVES_M) x (BN/WAVES_N) sub-tile
// as 32x32x16 MFMA blocks.
//
// Orientation: with SWAP = false the MFMA "A" operand is the weight tile, so
// an accumulator lane holds one token and 4 consecutive features: row-major
// stores are 8-byte vectors.  With SWAP = true the roles flip and a lane holds
// one feature and 4 consecutive tokens: that is the store pattern of the
// transposed V layout the attention kernels read.
#include <atomic>

#include "gemm.hpp"

namespace sf {

constexpr int BK = 64;                 // bf16 elements per K step (128 bytes = 8 chunks of 16 B)

__device__ __forceinline__ int swz(int row, int chunk) { return row * BK + ((chunk ^ (row & 7)) << 3); }

__device__ __forceinline__ float apply_act(float z, int act)
{
    if (act == ACT_RELU) return z > 0.f ? z : 0.f;
    if (act == ACT_GELU) return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
    return z;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool SWAP>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_kernel(GemmArgs a)
{
    constexpr int NT = 64 * WAVES_M * WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int XCH = BM * 8 / NT, WCH = BN * 8 / NT;      // 16-byte chunks per thread per tile
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads mismatch");

    extern __shared__ __attribute__((aligned(16))) char smem_raw[];
    h16 *Xs = reinterpret_cast<h16 *>(smem_raw);             // [2][BM*BK]
    h16 *Ws = Xs + 2 * BM * BK;                                 // [2][BN*BK]

    const int tiles_m = (a.L + BM - 1) / BM;
    const int b = blockIdx.x / tiles_m;
    const int m0 = (blockIdx.x % tiles_m) * BM;
    const int nt0 = blockIdx.y * BN;                               // first feature of this tile (within launch)
    const int p = a.pattern_id ? a.pattern_id[b] : 0;
    if (p < 0) return;                                             // sample not in use
    if (a.n_lim) a.N = min(a.N, a.n_lim[p]);
    if (a.k_lim) a.K = min(a.K, a.k_lim[p]);
    if (nt0 >= a.N) return;

    const h16 *A = static_cast<const h16 *>(a.A) + ((int64_t)b * a.L) * a.lda;
    const h16 *W = static_cast<const h16 *>(a.W) + (int64_t)p * a.w_pstride + (int64_t)a.n0 * a.ldw;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int l32 = lane & 31, lhi = lane >> 5;

    uint4 xr[XCH], wr[WCH];
    const int lc = tid & 7;                 // chunk within the 128-byte row
    const int lr = tid >> 3;                // first row handled by this thread

    auto load_global = [&](int k0) {
        const int k = k0 + lc * 8;
        const bool kin = k < a.K;
#pragma unroll
        for (int j = 0; j < XCH; ++j) {
            const int r = lr + j * (NT / 8);
            const int i = m0 + r;
            xr[j] = (kin && i < a.L) ? *reinterpret_cast<const uint4 *>(A + (int64_t)i * a.lda + k)
                                     : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < WCH; ++j) {
            const int r = lr + j * (NT / 8);
            const int n = nt0 + r;
            wr[j] = (kin && n < a.N) ? *reinterpret_cast<const uint4 *>(W + (int64_t)n * a.ldw + k)
                                     : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_lds = [&](int buf) {
        h16 *xs = Xs + buf * BM * BK, *ws = Ws + buf * BN * BK;
#pragma unroll
        for (int j = 0; j < XCH; ++j) {
            const int r = lr + j * (NT / 8);
            *reinterpret_cast<uint4 *>(xs + swz(r, lc)) = xr[j];
        }
#pragma unroll
        for (int j = 0; j < WCH; ++j) {
            const int r = lr + j * (NT / 8);
            *reinterpret_cast<uint4 *>(ws + swz(r, lc)) = wr[j];
        }
    };

    // accumulators: [row-operand tile][col-operand tile]
    constexpr int TP = SWAP ? TM : TN, TQ = SWAP ? TN : TM;
    f32x16 acc[TP][TQ];
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int nk = (a.K + BK - 1) / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) load_global((kt + 1) * BK);
        const h16 *xs = Xs + (kt & 1) * BM * BK, *ws = Ws + (kt & 1) * BN * BK;
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            h16x8 xf[TM], wf[TN];
            const int chunk = s * 2 + lhi;
#pragma unroll
            for (int t = 0; t < TM; ++t)
                xf[t] = *reinterpret_cast<const h16x8 *>(xs + swz(wm * WTM + t * 32 + l32, chunk));
#pragma unroll
            for (int t = 0; t < TN; ++t)
                wf[t] = *reinterpret_cast<const h16x8 *>(ws + swz(wn * WTN + t * 32 + l32, chunk));
#pragma unroll
            for (int i = 0; i < TP; ++i)
#pragma unroll
                for (int j = 0; j < TQ; ++j) {
                    if (SWAP) acc[i][j] = SF_MFMA16(xf[i], wf[j], acc[i][j], 0, 0, 0);
                    else      acc[i][j] = SF_MFMA16(wf[i], xf[j], acc[i][j], 0, 0, 0);
                }
        }
        if (kt + 1 < nk) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue -------------------------------------------------------------
    const h16 *bias = a.bias ? static_cast<const h16 *>(a.bias) + (int64_t)p * a.bias_pstride + a.n0 : nullptr;
    if (!SWAP) {
        // lane: token i = m0 + wm*WTM + tm*32 + l32 ; features n = wn*WTN + tn*32 + q*8 + lhi*4 + {0..3}
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int i = m0 + wm * WTM + tm * 32 + l32;
            if (i >= a.L) continue;
            const int64_t row = (int64_t)b * a.L + i;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = nt0 + wn * WTN + tn * 32 + q * 8 + lhi * 4;
                    if (n >= a.N) continue;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[tn][tm][q * 4 + e];
                    if (bias) {
                        const h16x4 bv = *reinterpret_cast<const h16x4 *>(bias + n);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += (float)bv[e];
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = apply_act(v[e], a.act);
                    if (a.R) {
                        const int64_t ro = row * a.ldr + a.r0 + n;
                        if (a.r_f32) {
                            const f32x4 rv = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(a.R) + ro);
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] += rv[e];
                        } else {
                            const h16x4 rv = *reinterpret_cast<const h16x4 *>(static_cast<const h16 *>(a.R) + ro);
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] += (float)rv[e];
                        }
                    }
                    const int64_t co = row * a.ldc + a.c0 + n;
                    if (a.c_f32) {
                        f32x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = v[e];
                        *reinterpret_cast<f32x4 *>(static_cast<float *>(a.C) + co) = o;
                    } else {
                        h16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (h16)v[e];
                        *reinterpret_cast<h16x4 *>(static_cast<h16 *>(a.C) + co) = o;
                    }
                }
            }
        }
    } else {
        // lane: feature n = wn*WTN + tn*32 + l32 ; tokens i = m0 + wm*WTM + tm*32 + q*8 + lhi*4 + {0..3}
        h16 *C = static_cast<h16 *>(a.C) + (int64_t)b * a.vt_b;
        const bool vec_ok = ((a.vt_b | a.vt_n) & 3) == 0;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int n = nt0 + wn * WTN + tn * 32 + l32;
            if (n >= a.N) continue;
            const float bv = bias ? (float)bias[n] : 0.f;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int i = m0 + wm * WTM + tm * 32 + q * 8 + lhi * 4;
                    if (i >= a.L) continue;
                    h16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (h16)apply_act(acc[tm][tn][q * 4 + e] + bv, a.act);
                    h16 *dst = C + (int64_t)n * a.vt_n + i;
                    if (vec_ok && i + 3 < a.L) {
                        *reinterpret_cast<h16x4 *>(dst) = o;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (i + e < a.L) dst[e] = o[e];
                    }
                }
            }
        }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool SWAP>
static int32_t launch_cfg(const GemmArgs &a, hipStream_t st)
{
    auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, SWAP>;
    constexpr size_t lds = (size_t)2 * (BM + BN) * BK * sizeof(h16);
    static std::atomic<bool> attr_set{false};     // per template instance; setting the attribute twice is harmless
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return fail(SF_ERR_HIP, "gemm: cannot reserve %zu bytes of LDS", lds);
        attr_set = true;
    }
    dim3 grid(ceil_div(a.L, BM) * a.B, ceil_div(a.N, BN));
    ProfScope prof(SF_KERNEL_GEMM, st);
    hipLaunchKernelGGL(kern, grid, dim3(64 * WAVES_M * WAVES_N), lds, st, a);
    return SF_OK;
}

int32_t gemm_bf16_fast(const GemmArgs &a, hipStream_t st, bool &done);
int32_t gemm_bf16_ws(const GemmArgs &a, hipStream_t st, bool &done);
bool gemm_bf16_ws_eligible(const GemmArgs &a);

bool gemm_takes_row_map(int dtype, const GemmArgs &a) { return dtype == SF_BF16 && gemm_bf16_ws_eligible(a); }
bool gemm_takes_vt_split(int dtype, const GemmArgs &a)
{
    return dtype == SF_BF16 && gemm_bf16_ws_eligible(a) && a.vt_from > 0 && a.vt_from < a.N && a.vt_from % 8 == 0 &&
           a.vt_b % 8 == 0 && a.vt_n % 8 == 0 && !a.R && !a.c_f32 && !a.n_lim;
}

int32_t gemm_bf16(const GemmArgs &a, hipStream_t st)
{
    if (a.B <= 0 || a.N <= 0) return SF_OK;
    if (a.VT && !gemm_takes_vt_split(SF_BF16, a)) return fail(SF_ERR_UNSUPPORTED, "gemm(bf16): transposed column range on a problem the large-tile kernel does not take");
    if (a.row_map && !gemm_bf16_ws_eligible(a)) return fail(SF_ERR_UNSUPPORTED, "gemm(bf16): row_map on a problem the large-tile kernel does not take");
    {
        bool done = false;
        if (int32_t rc = gemm_bf16_ws(a, st, done)) return rc;
        if (done) return SF_OK;
        if (int32_t rc = gemm_bf16_fast(a, st, done)) return rc;
        if (done) return SF_OK;
    }
    if (a.K % 8 || a.lda % 8 || a.ldw % 8 || a.N % 4 || a.n0 % 4 || (a.R && (a.ldr % 4 || a.r0 % 4)) ||
        (a.epi == EPI_ROWMAJOR && (a.ldc % 4 || a.c0 % 4)))
        return fail(SF_ERR_SHAPE, "gemm(bf16): K, leading dimensions and column origins must be multiples of 8/4");
    const bool swap = a.epi == EPI_VT;
    if (swap && (a.R || a.c_f32)) return fail(SF_ERR_UNSUPPORTED, "gemm(bf16): residual / fp32 output with transposed store");
    const int64_t rows = (int64_t)a.B * a.L;
    const bool big = a.L >= 192 && a.N >= 192 && rows * a.N >= (int64_t)256 * 256 * 256;
    if (swap) {
        if (big) return launch_cfg<256, 256, 2, 2, true>(a, st);
        return launch_cfg<128, 128, 2, 2, true>(a, st);
    }
    if (big) return launch_cfg<256, 256, 2, 2, false>(a, st);
    return launch_cfg<128, 128, 2, 2, false>(a, st);
}

}  // namespace sf
