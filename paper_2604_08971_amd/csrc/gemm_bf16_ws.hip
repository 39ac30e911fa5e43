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
//  * The ring is asymmetric: the activation operand X is streamed once from
//    HBM (a cold miss per line, a few microseconds under load) while the weight
//    tile is re-read from L2 by every row block.  X therefore gets three 32 KB
//    slots and is fetched two K tiles ahead, W gets two slots and is fetched
//    one tile ahead: 160 KB, all of a CU's LDS.
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
constexpr int XSLOT = BM * BKT, WSLOT = BN * BKT;  // bf16 elements per X / W ring slot (32 KB each)
constexpr int NXS = 3, NWS = 2;                 // ring slots: X two tiles ahead, W one tile ahead
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
    __bf16 *smem = reinterpret_cast<__bf16 *>(smem_raw);      // [NXS][X rows][64] | [NWS][W rows][64]

    const int wid = blockIdx.x;
    int tn_i, tm_i;
    if (a.xcd_rows) {
        // tile row r goes to XCD r % 8: rows of unequal cost spread evenly over the XCDs
        const int s = wid / N_XCD;
        tn_i = s % tiles_n;
        tm_i = (s / tiles_n) * N_XCD + wid % N_XCD;
        if (tm_i * tiles_n >= total_tiles) return;
    } else {
        const int w = (wid % N_XCD) * per_xcd + wid / N_XCD;
        if (w >= total_tiles) return;
        tn_i = w % tiles_n;
        tm_i = w / tiles_n;
    }
    const int b = tm_i / tiles_m;
    const int m0 = (tm_i % tiles_m) * BM;
    const int nt0 = tn_i * BN;
    const int p = a.pattern_id ? a.pattern_id[b] : 0;
    if (p < 0) return;                                             // sample not in use
    if (a.n_lim) a.N = min(a.N, a.n_lim[p]);
    if (a.k_lim) a.K = min(a.K, a.k_lim[p]);
    if (nt0 >= a.N) return;
    const int nk = a.K / BKT;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    if (wave >= NCW) {
        // ------------------------------------------------------------ loader wave
        const int lw = wave - NCW;
        constexpr int LPW = (BM / 8) / NLW;       // 8 X-instructions and 8 W-instructions per loader wave
        const char *Ab = reinterpret_cast<const char *>(static_cast<const __bf16 *>(a.A) +
                                                        (a.row_map ? (int64_t)0 : ((int64_t)b * a.L + m0) * a.lda));
        const int32_t *rmap = a.row_map ? a.row_map + (int64_t)b * a.L + m0 : nullptr;
        const char *Wb = reinterpret_cast<const char *>(static_cast<const __bf16 *>(a.W) + (int64_t)p * a.w_pstride +
                                                        (int64_t)(a.n0 + nt0) * a.ldw);
        const int rows_x = min(BM, a.L - m0), rows_w = min(BN, a.N - nt0);
        uint32_t xoff[LPW], woff[LPW];
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            const int sr = (lw * LPW + j) * 4 + (lane >> 4);      // super-row of this lane's 16-byte slot
            const int t = (lane & 15) ^ (sr & 7);
            const int r = sr * 2 + (t >> 3), c = t & 7;
            const int rx = min(r, rows_x - 1);
            xoff[j] = ((uint32_t)(rmap ? rmap[rx] : rx) * (uint32_t)a.lda + (uint32_t)(c * 8)) * 2u;
            woff[j] = (uint32_t)(min(r, rows_w - 1) * (int)a.ldw + c * 8) * 2u;
        }
        auto issue_x = [&](int tile) {
            __bf16 *base = smem + (tile % NXS) * XSLOT;
            const int64_t koff = (int64_t)tile * BKT * 2;
#pragma unroll
            for (int j = 0; j < LPW; ++j)
                __builtin_amdgcn_global_load_lds((glb_void *)(Ab + koff + xoff[j]),
                                                 (lds_void *)(base + (lw * LPW + j) * 512), 16, 0, 0);
        };
        auto issue_w = [&](int tile) {
            __bf16 *base = smem + NXS * XSLOT + (tile % NWS) * WSLOT;
            const int64_t koff = (int64_t)tile * BKT * 2;
#pragma unroll
            for (int j = 0; j < LPW; ++j)
                __builtin_amdgcn_global_load_lds((glb_void *)(Wb + koff + woff[j]),
                                                 (lds_void *)(base + (lw * LPW + j) * 512), 16, 0, 0);
        };
        // Loads complete in issue order.  Order kept: X(0) W(0) X(1) | W(1) X(2) | W(2) X(3) | ...
        // so at barrier kt only the LPW loads of X(kt+1) may still be in flight.
        issue_x(0);
        issue_w(0);
        if (nk > 1) issue_x(1);
        for (int kt = 0; kt < nk; ++kt) {
            if (kt + 1 < nk) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPW) : "memory");   // X(kt), W(kt) landed
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            // bare barrier: __syncthreads() carries a fence that would wait for the loads still in flight
            __builtin_amdgcn_s_barrier();     // barrier kt: tile kt visible; slots of X(kt-1), W(kt-1) free
            asm volatile("" ::: "memory");
            if (kt + 1 < nk) issue_w(kt + 1);
            if (kt + 2 < nk) issue_x(kt + 2);
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

    // Byte address in LDS of this lane's fragment (k-step 0, MFMA tile 0) inside an X / W slot.  In the
    // layout of lay(), MFMA tile t adds t * 4096 bytes and k-step s flips bits 5..6 (XOR with s << 5).
    const uint32_t xlane = (uint32_t)lay(wm * TM * 32 + l32, lhi) * 2u;
    const uint32_t wlane = (uint32_t)(NXS * XSLOT) * 2u + (uint32_t)lay(wn * TN * 32 + l32, lhi) * 2u;
    static_assert(TN == 2 && TM == 4 && BKT == 64, "the interleaving below is written for 2 x 4 MFMA tiles per wave");
    uint32_t xslot = 0, wslot = 0;          // byte offsets of the ring slots of tile kt
    for (int kt = 0; kt < nk; ++kt) {
        // bare barrier: no global memory traffic of this wave needs ordering here
        __builtin_amdgcn_s_barrier();                             // barrier kt
        asm volatile("" ::: "memory");
        const uint32_t xb = xlane + xslot, wb = wlane + wslot;
        xslot = (xslot + XSLOT * 2 == NXS * XSLOT * 2) ? 0u : xslot + XSLOT * 2;
        wslot = (wslot + WSLOT * 2 == NWS * WSLOT * 2) ? 0u : wslot + WSLOT * 2;
        // Fragment registers are scarce next to 128 accumulators: the W fragments are double-buffered,
        // the X fragments are single-buffered and X fragment j of the next k-step is read right after
        // its last use in this k-step, so every read has about six MFMAs of cover.  The order below is
        // kept as written (sched_barrier), one address register per operand and k-step.
        bf16x8 xf[TM], wf[2][TN];
        auto rd = [&](uint32_t addr) { return *reinterpret_cast<const bf16x8 *>(smem_raw + addr); };
        {
            wf[0][0] = rd(wb); wf[0][1] = rd(wb + 4096);
#pragma unroll
            for (int t = 0; t < TM; ++t) xf[t] = rd(xb + t * 4096);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < BKT / 16; ++s) {
            const bool more = s + 1 < BKT / 16;
            const uint32_t xa = xb ^ ((uint32_t)(s + 1) << 5), wa = wb ^ ((uint32_t)(s + 1) << 5);
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[s & 1][0], xf[j], acc[0][j], 0, 0, 0);
                acc[1][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[s & 1][1], xf[j], acc[1][j], 0, 0, 0);
                if (more) {
                    xf[j] = rd(xa + j * 4096);
                    if (j < TN) wf[(s + 1) & 1][j] = rd(wa + j * 4096);
                }
                __builtin_amdgcn_sched_barrier(0);      // keep exactly this order: MFMA MFMA read(s)
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
                // streamed out: the output is far larger than L2 and must not push the weights out of it
                __builtin_nontemporal_store(o, reinterpret_cast<bf16x8 *>(static_cast<__bf16 *>(a.C) + (grow0 + i) * a.ldc + a.c0 + n));
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
            // rows out: 8 lanes x 16 bytes = 128 bytes of one row, 8 rows per instruction.  The residual
            // reads of the whole pass are issued first (the accumulators just staged have freed the
            // registers), so their latency is paid once per pass and not once per row group.
            const int er = lane >> 3, ec = lane & 7;
            const int n = ncol0 + tn * 32 + ec * 4;
            auto finish = [&](int j, f32x4 v) {
                const int i = mrow0 + j * 8 + er;
                if (i < a.L && n < a.N) {
                    const int64_t co = (grow0 + i) * a.ldc + a.c0 + n;
                    if (a.c_f32) {
                        __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(static_cast<float *>(a.C) + co));
                    } else {
                        bf16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (__bf16)v[e];
                        __builtin_nontemporal_store(o, reinterpret_cast<bf16x4 *>(static_cast<__bf16 *>(a.C) + co));
                    }
                }
            };
            if (a.R && a.r_f32) {
                f32x4 rr[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int i = min(mrow0 + j * 8 + er, a.L - 1);          // clamped: never stored when out of range
                    const int64_t ro = (grow0 + i) * a.ldr + a.r0 + min(n, a.N - 4);
                    rr[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(static_cast<const float *>(a.R) + ro));
                }
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    f32x4 v = *reinterpret_cast<const f32x4 *>(stf + lay(j * 8 + er, ec) / 2);
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += rr[j][e];
                    finish(j, v);
                }
            } else if (a.R) {
                bf16x4 rr[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int i = min(mrow0 + j * 8 + er, a.L - 1);
                    const int64_t ro = (grow0 + i) * a.ldr + a.r0 + min(n, a.N - 4);
                    rr[j] = __builtin_nontemporal_load(reinterpret_cast<const bf16x4 *>(static_cast<const __bf16 *>(a.R) + ro));
                }
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    f32x4 v = *reinterpret_cast<const f32x4 *>(stf + lay(j * 8 + er, ec) / 2);
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += (float)rr[j][e];
                    finish(j, v);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    finish(j, *reinterpret_cast<const f32x4 *>(stf + lay(j * 8 + er, ec) / 2));
            }
        }
    }
}

}  // namespace

template <int ACT>
static int32_t launch_ws(const GemmArgs &a, hipStream_t st)
{
    auto kern = gemm_bf16_ws_kernel<ACT>;
    constexpr size_t lds = ((size_t)NXS * XSLOT + (size_t)NWS * WSLOT) * sizeof(__bf16);     // 160 KB
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return fail(SF_ERR_HIP, "gemm: cannot reserve %zu bytes of LDS", lds);
        attr_set = true;
    }
    const int tiles_m = ceil_div(a.L, BM), tiles_n = ceil_div(a.N, BN);
    const int total = a.B * tiles_m * tiles_n;
    const int per_xcd = a.xcd_rows ? ceil_div(a.B * tiles_m, N_XCD) * tiles_n : ceil_div(total, N_XCD);
    ProfScope prof(SF_KERNEL_GEMM, st);
    hipLaunchKernelGGL(kern, dim3(per_xcd * N_XCD), dim3(64 * (NCW + NLW)), lds, st, a, tiles_m, tiles_n, total, per_xcd);
    return SF_OK;
}

// Large, row-major, K % 64 == 0.
bool gemm_bf16_ws_eligible(const GemmArgs &a)
{
    if (a.epi != EPI_ROWMAJOR || a.K % BKT || a.K < BKT || a.N % 8 || a.n0 % 8 || a.lda % 8 || a.ldw % 8 ||
        a.ldc % 8 || a.c0 % 8 || (a.R && (a.ldr % 8 || a.r0 % 8)))
        return false;
    if (a.L < 192 || a.N < 192) return false;
    if ((int64_t)a.L * a.lda * 2 >= ((int64_t)1 << 32) || (int64_t)a.N * a.ldw * 2 >= ((int64_t)1 << 32)) return false;
    return true;
}

// Takes the problem (sets `done`) when it is eligible.
int32_t gemm_bf16_ws(const GemmArgs &a, hipStream_t st, bool &done)
{
    done = false;
    if (!gemm_bf16_ws_eligible(a)) return SF_OK;
    done = true;
    switch (a.act) {
    case ACT_RELU: return launch_ws<ACT_RELU>(a, st);
    case ACT_GELU: return launch_ws<ACT_GELU>(a, st);
    default: return launch_ws<ACT_NONE>(a, st);
    }
}

}  // namespace sf
