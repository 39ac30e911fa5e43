// Wave-specialised bf16 MFMA GEMM for the large projections of the pruned
// encoder layer (K % 64 == 0, row-major output; see gemm_bf16.hip for the role
// of the GEMM and gemm.hpp for the arguments).
//
// Measured on gfx950: a wave that issues direct-to-LDS loads between its MFMAs
// stalls in instruction issue while the address unit takes the loads, and the
// matrix pipe drains.  So the 256x256 output tile is computed by 8 MFMA waves
// (2 x 4, 128 x 64 each, 128 accumulator registers) while 4 separate loader
// waves do nothing but feed the double-buffered LDS ring with
// global_load_lds_dwordx4 (12 waves = 3 per SIMD, <= 168 registers each).
//
//  * LDS layout: 256-byte super-rows (two 128-byte K rows) with the 16-byte slot
//    XOR-ed by the super-row number: the LDS serves 16 lanes of a ds_read_b128
//    per cycle and this keeps any 16 consecutive rows of one chunk conflict-free.
//    The direct loads land at lane*16 bytes, so the swizzle is applied to the
//    global address.
//  * Edge rows are clamped (they only feed outputs that are never stored).
//  * Tile order is XCD-aware: each XCD (own L2) walks a contiguous range of
//    tiles, N fastest.
//  * Epilogue: bias and activation in registers, then each wave transposes its
//    sub-tile through its private 16 KB of the (now free) LDS ring so that
//    every global store instruction writes 8 rows x 128 contiguous bytes (the
//    residual is read with the same pattern).
#include <type_traits>

#include "gemm.hpp"

namespace sf {

namespace {

constexpr int BM = 256, BN = 256, BKT = 64;
constexpr int NCW = 8, NLW = 4;                 // compute waves, loader waves
constexpr int WAVES_N = 4;                      // compute waves: 2 (M) x 4 (N)
constexpr int TM = 4, TN = 2;                   // 32x32 MFMA tiles per compute wave
constexpr int STAGE = (BM + BN) * BKT;          // bf16 elements per ring slot (64 KB)
constexpr int N_XCD = 8;

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

// element offset of (row, 16-byte chunk) in a [rows][64] bf16 tile
__device__ __forceinline__ int lay(int row, int chunk)
{
    const int sr = row >> 1;
    return sr * 128 + ((((row & 1) << 3) | chunk) ^ (sr & 7)) * 8;
}

template <int ACT>
__device__ __forceinline__ float activate(float z)
{
    if (ACT == ACT_RELU) return z > 0.f ? z : 0.f;
    if (ACT == ACT_GELU) return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
    return z;
}

template <int ACT>
__global__ __launch_bounds__(64 * (NCW + NLW)) __attribute__((amdgpu_waves_per_eu(3, 3)))
void gemm_bf16_ws_kernel(GemmArgs a, int tiles_m, int tiles_n, int total_tiles, int per_xcd)
{
    extern __shared__ __attribute__((aligned(16))) char smem_raw[];
    __bf16 *smem = reinterpret_cast<__bf16 *>(smem_raw);      // [2][X rows | W rows][64]

    const int wid = blockIdx.x;
    const int w = (wid % N_XCD) * per_xcd + wid / N_XCD;
    if (w >= total_tiles) return;
    const int tn_i = w % tiles_n, tm_i = w / tiles_n;
    const int b = tm_i / tiles_m;
    const int m0 = (tm_i % tiles_m) * BM;
    const int nt0 = tn_i * BN;
    const int p = a.pattern_id ? a.pattern_id[b] : 0;
    const int nk = a.K / BKT;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    if (wave >= NCW) {
        // ------------------------------------------------------------ loader wave
        const int lw = wave - NCW;
        constexpr int LPW = (BM / 8) / NLW;       // 8 X-instructions and 8 W-instructions per loader wave
        const char *Ab = reinterpret_cast<const char *>(static_cast<const __bf16 *>(a.A) + ((int64_t)b * a.L + m0) * a.lda);
        const char *Wb = reinterpret_cast<const char *>(static_cast<const __bf16 *>(a.W) + (int64_t)p * a.w_pstride +
                                                        (int64_t)(a.n0 + nt0) * a.ldw);
        const int rows_x = min(BM, a.L - m0), rows_w = min(BN, a.N - nt0);
        uint32_t xoff[LPW], woff[LPW];
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            const int sr = (lw * LPW + j) * 4 + (lane >> 4);      // super-row of this lane's 16-byte slot
            const int t = (lane & 15) ^ (sr & 7);
            const int r = sr * 2 + (t >> 3), c = t & 7;
            xoff[j] = (uint32_t)(min(r, rows_x - 1) * (int)a.lda + c * 8) * 2u;
            woff[j] = (uint32_t)(min(r, rows_w - 1) * (int)a.ldw + c * 8) * 2u;
        }
        auto issue = [&](int tile) {
            __bf16 *base = smem + (tile & 1) * STAGE;
            const int64_t koff = (int64_t)tile * BKT * 2;
#pragma unroll
            for (int j = 0; j < LPW; ++j) {
                __builtin_amdgcn_global_load_lds((glb_void *)(Ab + koff + xoff[j]),
                                                 (lds_void *)(base + (lw * LPW + j) * 512), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((glb_void *)(Wb + koff + woff[j]),
                                                 (lds_void *)(base + BM * BKT + (lw * LPW + j) * 512), 16, 0, 0);
            }
        };
        issue(0);
        for (int kt = 0; kt < nk; ++kt) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // tile kt has landed
            __syncthreads();                                      // barrier kt: tile kt visible, slot of tile kt-1 free
            if (kt + 1 < nk) issue(kt + 1);
        }
        __syncthreads();                                          // matches the barrier before the epilogue
        return;
    }

    // ---------------------------------------------------------------- MFMA wave
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int l32 = lane & 31, lhi = lane >> 5;
    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();                                          // barrier kt
        const __bf16 *xs = smem + (kt & 1) * STAGE;
        const __bf16 *ws = xs + BM * BKT;
        bf16x8 xf[2][TM], wf[2][TN];
        auto load_frags = [&](int s, int slot) {
            const int chunk = s * 2 + lhi;
#pragma unroll
            for (int t = 0; t < TM; ++t)
                xf[slot][t] = *reinterpret_cast<const bf16x8 *>(xs + lay((wm * TM + t) * 32 + l32, chunk));
#pragma unroll
            for (int t = 0; t < TN; ++t)
                wf[slot][t] = *reinterpret_cast<const bf16x8 *>(ws + lay((wn * TN + t) * 32 + l32, chunk));
        };
        load_frags(0, 0);
#pragma unroll
        for (int s = 0; s < BKT / 16; ++s) {
            if (s + 1 < BKT / 16) load_frags(s + 1, (s + 1) & 1);
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[s & 1][i], xf[s & 1][j], acc[i][j], 0, 0, 0);
            // MFMA, LDS read, MFMA, LDS read, ...: the reads of k-step s+1 ride under the MFMAs of k-step s
            const int NDS = (s + 1 < BKT / 16) ? TM + TN : 0;
#pragma unroll
            for (int i = 0; i < TM * TN; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (i < NDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
    }
    __syncthreads();          // every MFMA wave is done reading the ring: its LDS can be reused

    // ------------------------------------------------------------------ epilogue
    // Accumulator entry q*4+e of lane (l32, lhi) of tile (tn, tm): token tm*32 + l32, feature
    // tn*32 + q*8 + lhi*4 + e.  v_permlane32_swap pairs lane l with l+32 so that lanes < 32 own
    // features [q0*8, q0*8+8) and lanes >= 32 own [q1*8, q1*8+8), (q0, q1) = (0,1), (2,3).
    const __bf16 *bias = a.bias ? static_cast<const __bf16 *>(a.bias) + (int64_t)p * a.bias_pstride + a.n0 : nullptr;
    char *stg = smem_raw + wave * 16384;                           // this wave's private staging area
    const int ncol0 = nt0 + wn * 64;                               // first feature of the wave's sub-tile
    const int mrow0 = m0 + wm * 128;                               // first token of the wave's sub-tile
    const int64_t grow0 = (int64_t)b * a.L;

    if (!a.c_f32 && !a.R) {
        // bf16 output, no residual: stage the whole 128 x 64 sub-tile as bf16 rows of 128 bytes
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
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
                    const int c = tn * 4 + qp * 2 + lhi;               // 16-byte chunk = 8 features
                    if (bias) {
                        const int n = min(ncol0 + c * 8, a.N - 8);     // clamped: out-of-range chunks are not stored
                        const bf16x8 bv = *reinterpret_cast<const bf16x8 *>(bias + n);
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] += (float)bv[e];
                    }
                    bf16x8 o;
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = (__bf16)activate<ACT>(v[e]);
                    *reinterpret_cast<bf16x8 *>(reinterpret_cast<__bf16 *>(stg) + lay(tm * 32 + l32, c)) = o;
                }
        // rows out: 8 lanes x 16 bytes = one 128-byte row, 8 rows per instruction
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int r = j * 8 + (lane >> 3), c = lane & 7;
            const bf16x8 o = *reinterpret_cast<const bf16x8 *>(reinterpret_cast<const __bf16 *>(stg) + lay(r, c));
            const int i = mrow0 + r, n = ncol0 + c * 8;
            if (i < a.L && n < a.N)
                *reinterpret_cast<bf16x8 *>(static_cast<__bf16 *>(a.C) + (grow0 + i) * a.ldc + a.c0 + n) = o;
        }
    } else {
        // residual and/or fp32 output: stage fp32, 32 features (128 bytes per row) at a time
        float *stf = reinterpret_cast<float *>(stg);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
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
                    const int f0 = (qp * 2 + lhi) * 8;                 // first of this lane's 8 features within the 32
                    if (bias) {
                        const int n = min(ncol0 + tn * 32 + f0, a.N - 8);
                        const bf16x8 bv = *reinterpret_cast<const bf16x8 *>(bias + n);
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] += (float)bv[e];
                    }
                    f32x4 o0, o1;
#pragma unroll
                    for (int e = 0; e < 4; ++e) { o0[e] = activate<ACT>(v[e]); o1[e] = activate<ACT>(v[4 + e]); }
                    // a 16-byte chunk holds 4 floats: this lane fills chunks f0/4 and f0/4 + 1
                    *reinterpret_cast<f32x4 *>(stf + lay(tm * 32 + l32, f0 / 4) / 2) = o0;
                    *reinterpret_cast<f32x4 *>(stf + lay(tm * 32 + l32, f0 / 4 + 1) / 2) = o1;
                }
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int r = j * 8 + (lane >> 3), c = lane & 7;
                f32x4 v = *reinterpret_cast<const f32x4 *>(stf + lay(r, c) / 2);
                const int i = mrow0 + r, n = ncol0 + tn * 32 + c * 4;
                if (i < a.L && n < a.N) {
                    if (a.R) {
                        const int64_t ro = (grow0 + i) * a.ldr + a.r0 + n;
                        if (a.r_f32) {
                            const f32x4 rv = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(a.R) + ro);
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] += rv[e];
                        } else {
                            const bf16x4 rv = *reinterpret_cast<const bf16x4 *>(static_cast<const __bf16 *>(a.R) + ro);
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] += (float)rv[e];
                        }
                    }
                    const int64_t co = (grow0 + i) * a.ldc + a.c0 + n;
                    if (a.c_f32) {
                        *reinterpret_cast<f32x4 *>(static_cast<float *>(a.C) + co) = v;
                    } else {
                        bf16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (__bf16)v[e];
                        *reinterpret_cast<bf16x4 *>(static_cast<__bf16 *>(a.C) + co) = o;
                    }
                }
            }
        }
    }
}

}  // namespace

template <int ACT>
static int32_t launch_ws(const GemmArgs &a, hipStream_t st)
{
    auto kern = gemm_bf16_ws_kernel<ACT>;
    constexpr size_t lds = (size_t)2 * STAGE * sizeof(__bf16);
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
    hipLaunchKernelGGL(kern, dim3(per_xcd * N_XCD), dim3(64 * (NCW + NLW)), lds, st, a, tiles_m, tiles_n, total, per_xcd);
    return SF_OK;
}

// Takes the problem (sets `done`) when it is large, row-major and K % 64 == 0.
int32_t gemm_bf16_ws(const GemmArgs &a, hipStream_t st, bool &done)
{
    done = false;
    if (a.epi != EPI_ROWMAJOR || a.K % BKT || a.K < BKT || a.N % 8 || a.n0 % 8 || a.lda % 8 || a.ldw % 8 ||
        a.ldc % 8 || a.c0 % 8 || (a.R && (a.ldr % 8 || a.r0 % 8)))
        return SF_OK;
    if (a.L < 192 || a.N < 192) return SF_OK;
    if ((int64_t)a.L * a.lda * 2 >= ((int64_t)1 << 32) || (int64_t)a.N * a.ldw * 2 >= ((int64_t)1 << 32)) return SF_OK;
    done = true;
    switch (a.act) {
    case ACT_RELU: return launch_ws<ACT_RELU>(a, st);
    case ACT_GELU: return launch_ws<ACT_GELU>(a, st);
    default: return launch_ws<ACT_NONE>(a, st);
    }
}

}  // namespace sf
