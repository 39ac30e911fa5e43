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
//  * Persistent: one workgroup per compute unit walks its share of the output
//    tiles.  Each XCD (own L2) owns a contiguous range of the tile list (N
//    fastest) and its workgroups take the tiles of that range round-robin, so
//    the tiles in flight on an XCD are neighbours.  The loader waves run on
//    across output tiles: while the MFMA waves are in the epilogue of tile i the
//    first K tiles of tile i+1 are already landing, no workgroup launch, first-
//    load latency or store drain sits between two tiles.  (Measured on the FFN
//    up-projection: a workgroup per tile spent 9 of 29 microseconds per tile
//    outside the K loop, 1.9 of them in the launch alone.)
//  * Epilogue: the accumulators start at the bias, activation and rounding run
//    in registers, then each wave transposes its sub-tile through a private
//    8 KB piece of the two ring slots of the step consumed last (the other
//    slots already hold the next tile) so that every global store instruction
//    writes 8 rows x 128 contiguous bytes (the residual is read with the same
//    pattern).  Two MFMA waves share a SIMD, so the epilogue is bound by its
//    instruction count: no lane exchange, packed conversions, integer ReLU.
#include <algorithm>
#include <type_traits>

#include <atomic>

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
    // integer max on the bit pattern: one instruction, -0 and negatives give +0, no canonicalisation pass
    if (ACT == ACT_RELU) return __int_as_float(max(__float_as_int(z), 0));
    if (ACT == ACT_GELU) return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
    return z;
}

// One output tile of the walk below
struct Tile { int b, m0, nt0, p, N, nk, vt; };

// The tiles of this workgroup, in order.  The launch has the same number of workgroups on every XCD
// (workgroup w runs on XCD w % 8); an XCD owns `per_xcd` tile slots: a contiguous range of the tile list
// (N fastest), or with xcd_rows the tile rows r with r % 8 == XCD.  The workgroups of an XCD take its
// slots round-robin, so at any time they work on neighbouring tiles (shared W tiles and X rows in that
// XCD's L2).  Slots past the end, samples with a negative pattern and tiles beyond the pattern's own
// width are skipped.  Every wave of the workgroup calls this with the same arguments, so loader and MFMA
// waves see the same sequence.
template <int KSTEP>
__device__ __forceinline__ bool next_tile(const GemmArgs &a, int tiles_m, int tiles_n, int total_tiles, int per_xcd,
                                          int stride, int &s, Tile &t)
{
    const int xcd = blockIdx.x % N_XCD;
    for (; s < per_xcd; s += stride) {
        int tn_i, tm_i;
        if (a.xcd_rows) {
            tn_i = s % tiles_n;
            tm_i = (s / tiles_n) * N_XCD + xcd;
            if (tm_i * tiles_n >= total_tiles) continue;
        } else {
            const int w = xcd * per_xcd + s;
            if (w >= total_tiles) continue;
            tn_i = w % tiles_n;
            tm_i = w / tiles_n;
            // when the workgroups of an XCD are a multiple of the tiles per row, a workgroup would meet the same
            // column in every round: rotate the columns from round to round (tiles of unequal cost then spread
            // over all workgroups).  Only when the XCD's range starts on a row boundary too: then the tiles of a
            // row lie in one round of one XCD and the rotation permutes them; a row that straddles two rounds or
            // two XCDs would get one column twice and another not at all.
            if (stride % tiles_n == 0 && per_xcd % tiles_n == 0) tn_i = (tn_i + s / stride) % tiles_n;
        }
        t.b = tm_i / tiles_m;
        t.m0 = (tm_i % tiles_m) * BM;
        t.p = a.pattern_id ? a.pattern_id[t.b] : 0;
        if (t.p < 0) continue;                                     // sample not in use
        if (a.VT) {
            // two column ranges, each with its own tiles: [0, vt_from) row-major, [vt_from, N) transposed
            const int ta = (a.vt_from + BN - 1) / BN;
            t.vt = tn_i >= ta;
            t.nt0 = t.vt ? a.vt_from + (tn_i - ta) * BN : tn_i * BN;
            t.N = t.vt ? a.N : a.vt_from;
        } else {
            t.vt = 0;
            t.nt0 = tn_i * BN;
            t.N = a.n_lim ? min(a.N, a.n_lim[t.p]) : a.N;
        }
        if (t.nt0 >= t.N) continue;
        t.nk = (a.k_lim ? min(a.K, a.k_lim[t.p]) : a.K) / KSTEP;
        if (t.nk < 1) continue;
        s += stride;
        return true;
    }
    return false;
}

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

// F8: A and W hold E4M3 codes (one byte per element).  A K tile is still 128 bytes of a row, i.e. 128 elements,
// so the loaders, the LDS ring and its layout are those of the bf16 kernel byte for byte; the MFMA waves issue
// v_mfma_f32_32x32x64_f8f6f4 (twice the multiply-adds per matrix-pipe cycle of the bf16 instruction, 32 bytes of a
// row per lane and instruction).  Which 64 of the 128 k of a row an instruction sees only has to agree between
// the two operands: lane (l32, lhi) takes 16-byte chunks 4m + lhi and 4m + 2 + lhi for instruction m, the two
// reads the bf16 loop issues for k-steps 2m and 2m + 1.
template <int ACT, bool F8>
__device__ __forceinline__ void ws_body(const GemmArgs a, int tiles_m, int tiles_n, int total_tiles, int per_xcd)
{
    extern __shared__ __attribute__((aligned(16))) char smem_raw[];
    h16 *smem = reinterpret_cast<h16 *>(smem_raw);      // [NXS][X rows][128 bytes] | [NWS][W rows][128 bytes]
    constexpr int ESZ = F8 ? 1 : 2;                           // bytes per element of A and W
    constexpr int KSTEP = 128 / ESZ;                          // elements of K per ring slot

    const int stride = gridDim.x / N_XCD;                     // workgroups per XCD
    const int s0 = blockIdx.x / N_XCD;                        // this workgroup's first slot
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    if (wave >= NCW) {
        // ------------------------------------------------------------ loader wave
        // Three walks over the same tile sequence: the K tiles of X being requested (two steps ahead of
        // the MFMA waves), those of W (one step ahead) and the step being consumed.  A "step" is one K
        // tile of one output tile; the ring and the barrier protocol run on across output tiles, so the
        // first K tiles of the next output tile arrive while the MFMA waves are still in their epilogue.
        const int lw = wave - NCW;
        constexpr int LPW = (BM / 8) / NLW;       // 8 X-instructions and 8 W-instructions per loader wave
        int sx = s0, sw = s0, sc = s0;
        Tile tx, tw, tc;
        bool vx, vw;
        const char *xbase = nullptr, *wbase = nullptr;
        uint32_t xoff[LPW], woff[LPW];
        int ktx = 0, ktw = 0, xs = 0, wsl = 0;
        auto open_x = [&]() {
            vx = next_tile<KSTEP>(a, tiles_m, tiles_n, total_tiles, per_xcd, stride, sx, tx);
            ktx = 0;
            if (!vx) return;
            xbase = static_cast<const char *>(a.A) +
                    (a.row_map ? (int64_t)0 : ((int64_t)tx.b * a.L + tx.m0) * a.lda) * ESZ;
            const int32_t *rmap = a.row_map ? a.row_map + (int64_t)tx.b * a.L + tx.m0 : nullptr;
            const int rows_x = min(BM, a.L - tx.m0);
#pragma unroll
            for (int j = 0; j < LPW; ++j) {
                const int sr = (lw * LPW + j) * 4 + (lane >> 4);      // super-row of this lane's 16-byte slot
                const int t = (lane & 15) ^ (sr & 7);
                const int r = sr * 2 + (t >> 3), c = t & 7;
                const int rx = min(r, rows_x - 1);
                xoff[j] = (uint32_t)(rmap ? rmap[rx] : rx) * (uint32_t)a.lda * (uint32_t)ESZ + (uint32_t)(c * 16);
            }
        };
        auto open_w = [&]() {
            vw = next_tile<KSTEP>(a, tiles_m, tiles_n, total_tiles, per_xcd, stride, sw, tw);
            ktw = 0;
            if (!vw) return;
            wbase = static_cast<const char *>(a.W) + ((int64_t)tw.p * a.w_pstride + (int64_t)(a.n0 + tw.nt0) * a.ldw) * ESZ;
            const int rows_w = min(BN, tw.N - tw.nt0);
#pragma unroll
            for (int j = 0; j < LPW; ++j) {
                const int sr = (lw * LPW + j) * 4 + (lane >> 4);
                const int t = (lane & 15) ^ (sr & 7);
                const int r = sr * 2 + (t >> 3), c = t & 7;
                woff[j] = (uint32_t)(min(r, rows_w - 1) * (int)a.ldw) * (uint32_t)ESZ + (uint32_t)(c * 16);
            }
        };
        auto issue_x = [&]() {
            h16 *base = smem + xs * XSLOT;
            const int64_t koff = (int64_t)ktx * 128;
#pragma unroll
            for (int j = 0; j < LPW; ++j)
                __builtin_amdgcn_global_load_lds((glb_void *)(xbase + koff + xoff[j]),
                                                 (lds_void *)(base + (lw * LPW + j) * 512), 16, 0, 0);
            xs = xs + 1 == NXS ? 0 : xs + 1;
            if (++ktx == tx.nk) open_x();
        };
        auto issue_w = [&]() {
            h16 *base = smem + NXS * XSLOT + wsl * WSLOT;
            const int64_t koff = (int64_t)ktw * 128;
#pragma unroll
            for (int j = 0; j < LPW; ++j)
                __builtin_amdgcn_global_load_lds((glb_void *)(wbase + koff + woff[j]),
                                                 (lds_void *)(base + (lw * LPW + j) * 512), 16, 0, 0);
            wsl = wsl + 1 == NWS ? 0 : wsl + 1;
            if (++ktw == tw.nk) open_w();
        };
        open_x();
        open_w();
        // Loads complete in issue order.  Order kept: X(0) W(0) X(1) | W(1) X(2) | W(2) X(3) | ...
        // so at barrier g only the LPW loads of X(g+1) may still be in flight.
        bool x_ahead = false;
        if (vx) issue_x();
        if (vw) issue_w();
        if (vx) { issue_x(); x_ahead = true; }
        while (next_tile<KSTEP>(a, tiles_m, tiles_n, total_tiles, per_xcd, stride, sc, tc)) {
            for (int kt = 0; kt < tc.nk; ++kt) {
                if (x_ahead) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPW) : "memory");   // X(g), W(g) landed
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                // bare barrier: __syncthreads() carries a fence that would wait for the loads still in flight
                __builtin_amdgcn_s_barrier();     // barrier g: step g visible; slots of X(g-1), W(g-1) free
                asm volatile("" ::: "memory");
                if (vw) issue_w();
                x_ahead = vx;
                if (vx) issue_x();
            }
            __builtin_amdgcn_s_barrier();         // matches the barrier before the epilogue
            asm volatile("" ::: "memory");
        }
        return;
    }

    // ---------------------------------------------------------------- MFMA wave
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int l32 = lane & 31, lhi = lane >> 5;
    // Byte address in LDS of this lane's fragment (k-step 0, MFMA tile 0) inside an X / W slot.  In the
    // layout of lay(), MFMA tile t adds t * 4096 bytes and k-step s flips bits 5..6 (XOR with s << 5).
    const uint32_t xlane = (uint32_t)lay(wm * TM * 32 + l32, lhi) * 2u;
    const uint32_t wlane = (uint32_t)(NXS * XSLOT) * 2u + (uint32_t)lay(wn * TN * 32 + l32, lhi) * 2u;
    // Transposed column range: the same instruction stream with the operand roles exchanged.  The two-fragment
    // ("A") side reads token rows, the four-fragment ("B") side reads feature rows, so the wave covers 64 tokens x
    // 128 features (waves 4 x 2) and an accumulator lane owns one feature and 4 consecutive tokens.
    const int wmv = wave & 3, wnv = wave >> 2;
    const uint32_t xlane_vt = (uint32_t)lay(wmv * TN * 32 + l32, lhi) * 2u;                                   // A side, in an X slot
    const uint32_t wlane_vt = (uint32_t)(NXS * XSLOT) * 2u + (uint32_t)lay(wnv * TM * 32 + l32, lhi) * 2u;    // B side, in a W slot
    static_assert(TN == 2 && TM == 4 && BKT == 64, "the interleaving below is written for 2 x 4 MFMA tiles per wave");
    uint32_t xslot = 0, wslot = 0;          // byte offsets of the ring slots of the next step
    int sm = s0;
    Tile tl;
    while (next_tile<KSTEP>(a, tiles_m, tiles_n, total_tiles, per_xcd, stride, sm, tl)) {
    // The accumulators start at the bias (fp32), so the epilogue has no bias pass.  Entry q*4+e of lane
    // (l32, lhi) of MFMA tile (tn, tm) is feature tn*32 + q*8 + lhi*4 + e.  The lane number goes through an
    // opaque copy so that these per-tile values are not hoisted out of the tile loop into long-lived registers.
    f32x16 acc[TN][TM];
    {
        int lb = lane;
        asm volatile("" : "+v"(lb));
        const h16 *bias = a.bias ? static_cast<const h16 *>(a.bias) + (int64_t)tl.p * a.bias_pstride + a.n0 : nullptr;
        // F8: the sum of code products is multiplied by out_scale in the epilogue, so the bias enters divided by it
        const float bscale = F8 ? 1.0f / a.out_scale : 1.0f;
        if (!F8 && tl.vt) {
            // every entry of MFMA tile (tn, tm) of this lane belongs to feature wnv*128 + tm*32 + l32
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int n = min(tl.nt0 + wnv * 128 + j * 32 + (lb & 31), tl.N - 1);   // clamped: never stored
                const float f = bias ? (float)bias[n] : 0.f;
#pragma unroll
                for (int i = 0; i < TN; ++i)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] = f;
            }
        } else
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                h16x4 bv = {};
                if (bias) {
                    const int n = min(tl.nt0 + wn * 64 + i * 32 + q * 8 + (lb >> 5) * 4, tl.N - 4);   // clamped: never stored
                    bv = *reinterpret_cast<const h16x4 *>(bias + n);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float f = F8 ? (float)bv[e] * bscale : (float)bv[e];
#pragma unroll
                    for (int j = 0; j < TM; ++j) acc[i][j][q * 4 + e] = f;
                }
            }
    }
    uint32_t xdone = 0, wdone = 0;          // slots of the step consumed last: free during the epilogue
    int kt = 0;
    do {                                    // next_tile() hands out tiles with nk >= 1 only
        // bare barrier: no global memory traffic of this wave needs ordering here
        __builtin_amdgcn_s_barrier();                             // barrier of this step
        asm volatile("" ::: "memory");
        // xb: base of the four-fragment side, wb: base of the two-fragment side
        const uint32_t xb = !F8 && tl.vt ? wlane_vt + wslot : xlane + xslot, wb = !F8 && tl.vt ? xlane_vt + xslot : wlane + wslot;
        xdone = xslot;
        wdone = wslot;
        xslot = (xslot + XSLOT * 2 == NXS * XSLOT * 2) ? 0u : xslot + XSLOT * 2;
        wslot = (wslot + WSLOT * 2 == NWS * WSLOT * 2) ? 0u : wslot + WSLOT * 2;
        // Fragment registers are scarce next to 128 accumulators: the W fragments are double-buffered,
        // the X fragments are single-buffered and X fragment j of the next k-step is read right after
        // its last use in this k-step, so every read has about six MFMAs of cover.  The order below is
        // kept as written (sched_barrier), one address register per operand and k-step.
        if constexpr (F8) {
            // Two instructions of K = 64 per (MFMA tile, ring slot), 8 registers per operand.  Next to the 128
            // accumulators there is room for three operands only: the two W fragments of instruction m stay
            // resident, the X fragment is a single buffer refilled right after the second instruction that
            // uses it has issued.  The wait for that read is covered by the other MFMA wave of the SIMD.
            auto rd32 = [&](uint32_t base, int m) {
                const i32x4 lo = *reinterpret_cast<const i32x4 *>(smem_raw + (base ^ ((uint32_t)(2 * m) << 5)));
                const i32x4 hi = *reinterpret_cast<const i32x4 *>(smem_raw + (base ^ ((uint32_t)(2 * m + 1) << 5)));
                return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            };
            i32x8 xv, wv[2];
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                wv[0] = rd32(wb, m); wv[1] = rd32(wb + 4096, m);
                xv = rd32(xb, m);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    acc[0][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wv[0], xv, acc[0][j], 0, 0, 0, 0, 0, 0);
                    acc[1][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wv[1], xv, acc[1][j], 0, 0, 0, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (j + 1 < TM) xv = rd32(xb + (uint32_t)(j + 1) * 4096u, m);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else {
        h16x8 xf[TM], wf[2][TN];
        auto rd = [&](uint32_t addr) { return *reinterpret_cast<const h16x8 *>(smem_raw + addr); };
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
                acc[0][j] = SF_MFMA16(wf[s & 1][0], xf[j], acc[0][j], 0, 0, 0);
                acc[1][j] = SF_MFMA16(wf[s & 1][1], xf[j], acc[1][j], 0, 0, 0);
                if (more) {
                    xf[j] = rd(xa + j * 4096);
                    if (j < TN) wf[(s + 1) & 1][j] = rd(wa + j * 4096);
                }
                __builtin_amdgcn_sched_barrier(0);      // keep exactly this order: MFMA MFMA read(s)
            }
        }
        }
    } while (++kt < tl.nk);
    // Every MFMA wave is done reading the step consumed last (its fragments went into MFMAs that have
    // issued): the two slots of that step are free until the loaders are let past the next step's
    // barrier, and hold the staging areas of the epilogue; the other slots already hold the next tile.
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // ------------------------------------------------------------------ epilogue
    // Accumulator entry q*4+e of lane (l32, lhi) of tile (tn, tm): token tm*32 + l32, feature
    // tn*32 + q*8 + lhi*4 + e.  v_permlane32_swap pairs lane l with l+32 so that lanes < 32 own
    // features [q0*8, q0*8+8) and lanes >= 32 own [q1*8, q1*8+8), (q0, q1) = (0,1), (2,3).
    // The lane-dependent indices are recomputed per tile from an opaque copy of the lane number: hoisted
    // out of the tile loop they would have to live across the K loop, i.e. in scratch.  The epilogue is
    // bound by its instruction count (two MFMA waves share a SIMD), so addresses advance by uniform strides.
    int le = lane;
    asm volatile("" : "+v"(le));
    const int l32e = le & 31, lhie = le >> 5;
    const int Np = tl.N;
    // this wave's private 8 KB staging area: 64 rows of 128 bytes
    char *stg = smem_raw + (wave < 4 ? xdone + (uint32_t)wave * 8192u
                                     : (uint32_t)(NXS * XSLOT) * 2u + wdone + (uint32_t)(wave - 4) * 8192u);
    const int ncol0 = tl.nt0 + wn * 64;                            // first feature of the wave's sub-tile
    const int mrow0 = tl.m0 + wm * 128;                            // first token of the wave's sub-tile
    const int64_t grow0 = (int64_t)tl.b * a.L;
    const bool inside = mrow0 + 128 <= a.L && ncol0 + 64 <= Np;   // uniform: the whole sub-tile exists, no per-row checks

    const float os = F8 ? a.out_scale : 1.0f;                      // F8: value = sum of code products x out_scale
    bool stored = false;
    if constexpr (F8) {
        if (a.c_f8) {
            // E4M3 codes out (the quantised hidden activations): code = E4M3(act(value) * c_scale), saturating.
            // The whole 128 x 64 sub-tile is staged at once: staged row r (128 bytes) holds the 64 codes of token r
            // and, in its upper half, those of token r + 64.  A lane owns 4 consecutive features per (tile, q):
            // two packed conversions make one dword.
            stored = true;
            const float cs = a.c_scale;
            const uint32_t wbase8 = (uint32_t)lay(l32e, 0) * 2u + (uint32_t)lhie * 4u;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float t[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float z = activate<ACT>(acc[tn][tm][q * 4 + e] * os) * cs;
                            t[e] = __builtin_amdgcn_fmed3f(z, -448.f, 448.f);
                        }
                        int w = 0;
                        w = __builtin_amdgcn_cvt_pk_fp8_f32(t[0], t[1], w, false);
                        w = __builtin_amdgcn_cvt_pk_fp8_f32(t[2], t[3], w, true);
                        const uint32_t chunk = (uint32_t)((tm >> 1) * 4 + tn * 2 + (q >> 1));
                        *reinterpret_cast<int *>(stg + ((wbase8 ^ (chunk << 4)) + (uint32_t)(tm & 1) * 4096u + (uint32_t)(q & 1) * 8u)) = w;
                    }
            int lo = le;
            asm volatile("" : "+v"(lo));
            const int er = lo >> 3, ec = lo & 7;
            const int tok0 = er + (ec >> 2) * 64;                  // token of this lane in row group 0
            const int rows_left = a.L - mrow0 - tok0;
            const bool col_ok = ncol0 + (ec & 3) * 16 < Np;
            uint8_t *cp = static_cast<uint8_t *>(a.C) + (grow0 + mrow0 + tok0) * a.ldc + a.c0 + ncol0 + (ec & 3) * 16;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const i32x4 o = *reinterpret_cast<const i32x4 *>(reinterpret_cast<const h16 *>(stg) + lay(j * 8 + er, ec));
                if (inside || (col_ok && j * 8 < rows_left))
                    __builtin_nontemporal_store(o, reinterpret_cast<i32x4 *>(cp + (int64_t)(j * 8) * a.ldc));
            }
        }
    }
    if (stored) {
    } else if ((!F8 && tl.vt) || (!a.c_f32 && !a.R)) {
        // bf16 output, no residual: stage 64 x 64 of the 128 x 64 sub-tile at a time as bf16 rows of 128 bytes.
        // (Transposed column range: the same code with tokens and features exchanged - a staged row is a feature
        // and holds 64 tokens - and the rows go to VT[b, n - vt_from, i].)
        // A lane owns 4 consecutive features per (tile, q): they go to LDS as one 8-byte write, with no lane
        // exchange.  In lay() the chunk index only flips bits 4..6 of the byte address, so one base address
        // per lane serves all chunks (XOR) and both 32-row halves (+4096 bytes).
        const uint32_t wbase = (uint32_t)lay(l32e, 0) * 2u + (uint32_t)lhie * 8u;
        typedef short i16x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int th = 0; th < 2; ++th)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int tm = half * 2 + th;
                        // round first, then (ReLU) clamp the packed values with 16-bit integer maxima: the
                        // sign of a bf16 is its top bit and rounding never changes the sign
                        float vf[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if constexpr (F8) vf[e] = ACT == ACT_RELU ? acc[tn][tm][q * 4 + e] * os : activate<ACT>(acc[tn][tm][q * 4 + e] * os);
                            else vf[e] = ACT == ACT_RELU ? acc[tn][tm][q * 4 + e] : activate<ACT>(acc[tn][tm][q * 4 + e]);
                        // one packed conversion per pair (written out: the compiler converts the elements of
                        // an accumulator tuple one by one and merges them with a byte permute)
                        uint2 pw;
                        pw.x = pack2_h16(vf[0], vf[1]);
                        pw.y = pack2_h16(vf[2], vf[3]);
                        i16x4 m = __builtin_bit_cast(i16x4, pw);
                        if (ACT == ACT_RELU) {
                            const i16x4 z = {0, 0, 0, 0};
                            m = __builtin_elementwise_max(m, z);
                        }
                        const uint2 o = __builtin_bit_cast(uint2, m);
                        *reinterpret_cast<uint2 *>(stg + ((wbase ^ ((uint32_t)(tn * 4 + q) << 4)) + (uint32_t)th * 4096u)) = o;
                    }
            // rows out: 8 lanes x 16 bytes = one 128-byte row, 8 rows per instruction.  The lane's output
            // address is formed here, after the staging pass (again from an opaque copy of the lane number):
            // formed before it, the 64-bit pointer lives through the pass with all 128 accumulators and is
            // spilled, and scratch traffic goes to memory (measured: +12 % bytes written by this kernel).
            int lo = le;
            asm volatile("" : "+v"(lo));
            const int er = lo >> 3, ec = lo & 7;
            const int rows_left = a.L - mrow0 - er;
            const bool col_ok = ncol0 + ec * 8 < Np;
            h16 *cp = static_cast<h16 *>(a.C) + (grow0 + mrow0 + er) * a.ldc + a.c0 + ncol0 + ec * 8;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = half * 64 + j * 8;                            // uniform
                const h16x8 o = *reinterpret_cast<const h16x8 *>(reinterpret_cast<const h16 *>(stg) + lay(j * 8 + er, ec));
                if (!F8 && tl.vt) {
                    const int n = tl.nt0 + wnv * 128 + r + er, i = tl.m0 + wmv * 64 + ec * 8;
                    h16 *dst = static_cast<h16 *>(a.VT) + (int64_t)tl.b * a.vt_b + (int64_t)(n - a.vt_from) * a.vt_n + i;
                    if (n < Np && i + 7 < a.L) {
                        __builtin_nontemporal_store(o, reinterpret_cast<h16x8 *>(dst));
                    } else if (n < Np) {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (i + e < a.L) dst[e] = o[e];
                    }
                } else if (inside || (col_ok && r < rows_left))
                    // streamed out: the output is far larger than L2 and must not push the weights out of it
                    __builtin_nontemporal_store(o, reinterpret_cast<h16x8 *>(cp + (int64_t)r * a.ldc));
            }
        }
    } else {
        // residual and/or fp32 output: stage fp32, 64 tokens x 32 features (128 bytes per row) at a time
        float *stf = reinterpret_cast<float *>(stg);
        // byte address of chunk lhi of row l32 in the staging tile; chunk c flips address bits 4..6 (see lay())
        const uint32_t wbase32 = (uint32_t)lay(l32e, lhie) * 2u;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
#pragma unroll
                for (int th = 0; th < 2; ++th)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        // the lane's 4 consecutive features of (tile, q) are one 16-byte chunk of the fp32 row:
                        // chunk q*2 + lhi, written as it is (no lane exchange)
                        const int tm = half * 2 + th;
                        f32x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = activate<ACT>(F8 ? acc[tn][tm][q * 4 + e] * os : acc[tn][tm][q * 4 + e]);
                        *reinterpret_cast<f32x4 *>(stg + ((wbase32 ^ ((uint32_t)(q * 2) << 4)) + (uint32_t)th * 4096u)) = o;
                    }
                // rows out: 8 lanes x 16 bytes = 128 bytes of one row, 8 rows per instruction.  The residual
                // reads of the whole pass are issued first, so their latency is paid once per pass and not
                // once per row group.  (Addresses formed after the staging pass, see the bf16 path.)
                int lo = le;
                asm volatile("" : "+v"(lo));
                const int er = lo >> 3, ec = lo & 7;
                const int rows_left = a.L - mrow0 - er;
                const int n = ncol0 + tn * 32 + ec * 4;
                const bool col_ok = n < Np;
                const int64_t co0 = (grow0 + mrow0 + er) * a.ldc + a.c0 + n;      // output element of row er
                const int64_t ro0 = (grow0 + min(mrow0 + er, a.L - 1)) * a.ldr + a.r0 + min(n, Np - 4);   // clamped: never stored when out of range
                auto finish = [&](int j, f32x4 v) {
                    const int r = half * 64 + j * 8;                        // uniform
                    if (inside || (col_ok && r < rows_left)) {
                        const int64_t co = co0 + (int64_t)r * a.ldc;
                        if (a.c_f32) {
                            __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(static_cast<float *>(a.C) + co));
                        } else {
                            h16x4 o;
#pragma unroll
                            for (int e = 0; e < 4; ++e) o[e] = (h16)v[e];
                            __builtin_nontemporal_store(o, reinterpret_cast<h16x4 *>(static_cast<h16 *>(a.C) + co));
                        }
                    }
                };
                // rows beyond the sample read the clamped row again (never stored)
                auto rrow = [&](int j) { return ro0 + (int64_t)min(half * 64 + j * 8, max(rows_left - 1, 0)) * a.ldr; };
                if (a.R && a.r_f32) {
                    f32x4 rr[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        rr[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(static_cast<const float *>(a.R) + rrow(j)));
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        f32x4 v = *reinterpret_cast<const f32x4 *>(stf + lay(j * 8 + er, ec) / 2);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += rr[j][e];
                        finish(j, v);
                    }
                } else if (a.R) {
                    h16x4 rr[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        rr[j] = __builtin_nontemporal_load(reinterpret_cast<const h16x4 *>(static_cast<const h16 *>(a.R) + rrow(j)));
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        f32x4 v = *reinterpret_cast<const f32x4 *>(stf + lay(j * 8 + er, ec) / 2);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += (float)rr[j][e];
                        finish(j, v);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        finish(j, *reinterpret_cast<const f32x4 *>(stf + lay(j * 8 + er, ec) / 2));
                }
            }
        }
    }
    }   // tile loop
}

template <int ACT>
__global__ __launch_bounds__(64 * (NCW + NLW)) __attribute__((amdgpu_waves_per_eu(3, 3)))
void gemm_bf16_ws_kernel(GemmArgs a, int tiles_m, int tiles_n, int total_tiles, int per_xcd)
{
    ws_body<ACT, false>(a, tiles_m, tiles_n, total_tiles, per_xcd);
}

template <int ACT>
__global__ __launch_bounds__(64 * (NCW + NLW)) __attribute__((amdgpu_waves_per_eu(3, 3)))
void gemm_fp8_ws_kernel(GemmArgs a, int tiles_m, int tiles_n, int total_tiles, int per_xcd)
{
    ws_body<ACT, true>(a, tiles_m, tiles_n, total_tiles, per_xcd);
}

}  // namespace

template <int ACT, bool F8>
static int32_t launch_ws(const GemmArgs &a, hipStream_t st)
{
    auto kern = F8 ? gemm_fp8_ws_kernel<ACT> : gemm_bf16_ws_kernel<ACT>;
    constexpr size_t lds = ((size_t)NXS * XSLOT + (size_t)NWS * WSLOT) * sizeof(h16);     // 160 KB
    static std::atomic<bool> attr_set{false};     // per template instance; setting the attribute twice is harmless
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return fail(SF_ERR_HIP, "gemm: cannot reserve %zu bytes of LDS", lds);
        attr_set = true;
    }
    const int tiles_m = ceil_div(a.L, BM);
    const int tiles_n = a.VT ? ceil_div(a.vt_from, BN) + ceil_div(a.N - a.vt_from, BN) : ceil_div(a.N, BN);
    const int total = a.B * tiles_m * tiles_n;
    const int per_xcd = a.xcd_rows ? ceil_div(a.B * tiles_m, N_XCD) * tiles_n : ceil_div(total, N_XCD);
    // persistent: one workgroup per compute unit (160 KB of LDS each), the same number on every XCD
    static std::atomic<int> cus{0};
    if (!cus) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < N_XCD)
            n = 256;
        cus = n;
    }
    const int wg_per_xcd = std::min(cus / N_XCD, per_xcd);
    ProfScope prof(SF_KERNEL_GEMM, st);
    hipLaunchKernelGGL(kern, dim3(wg_per_xcd * N_XCD), dim3(64 * (NCW + NLW)), lds, st, a, tiles_m, tiles_n, total, per_xcd);
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
    case ACT_RELU: return launch_ws<ACT_RELU, false>(a, st);
    case ACT_GELU: return launch_ws<ACT_GELU, false>(a, st);
    default: return launch_ws<ACT_NONE, false>(a, st);
    }
}

// E4M3 x E4M3 GEMM (a.f8): the persistent kernel is the only implementation.
//   value[b*L+i, n] = out_scale * sum_k dec(A[..]) dec(W[..]) + bias
// written as bf16 (with activation), as fp32 / with a residual like the bf16 GEMM, or (c_f8) as E4M3 codes of
// act(value) * c_scale with ldc in bytes.
int32_t gemm_fp8(const GemmArgs &a, hipStream_t st)
{
    if (a.B <= 0 || a.N <= 0) return SF_OK;
    if (a.epi != EPI_ROWMAJOR || a.VT || a.row_map)
        return fail(SF_ERR_UNSUPPORTED, "gemm(fp8): row-major output without row map only");
    if (a.K % 128 || a.K < 128 || a.lda % 16 || a.ldw % 16 || a.N % 16 || a.n0 % 16 || a.c0 % 16 ||
        a.ldc % (a.c_f8 ? 16 : 8) || (a.R && (a.ldr % 8 || a.r0 % 8)))
        return fail(SF_ERR_SHAPE, "gemm(fp8): K %% 128 == 0, N %% 16 == 0 and 16-byte aligned rows required");
    if (a.L < 192 || a.N < 192)
        return fail(SF_ERR_UNSUPPORTED, "gemm(fp8): at least 192 rows per sample and 192 output features required (got %d, %d)",
                    a.L, a.N);
    if ((int64_t)a.L * a.lda >= ((int64_t)1 << 32) || (int64_t)a.N * a.ldw >= ((int64_t)1 << 32))
        return fail(SF_ERR_SHAPE, "gemm(fp8): a sample of A and a pattern of W must stay below 4 GiB");
    if (!(a.out_scale > 0.f) || (a.c_f8 && (!(a.c_scale > 0.f) || a.R || a.c_f32)))
        return fail(SF_ERR_INVALID_ARG, "gemm(fp8): scales must be positive; code output takes no residual");
    switch (a.act) {
    case ACT_RELU: return launch_ws<ACT_RELU, true>(a, st);
    case ACT_GELU: return launch_ws<ACT_GELU, true>(a, st);
    default: return launch_ws<ACT_NONE, true>(a, st);
    }
}

}  // namespace sf
