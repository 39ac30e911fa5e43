// Pieces shared by the 256 x 256 x 64 bf16 MFMA GEMM kernels (gemm_bf16_ws.hip,
// gemm_bf16_w4.hip): tile constants, the swizzled LDS layout, the activation and
// the epilogue of one wave's 128-token x 64-feature sub-tile.
#pragma once

#include "gemm.hpp"

namespace sf {
namespace gemm_tile {

constexpr int BM = 256, BN = 256, BKT = 64;
constexpr int XSLOT = BM * BKT, WSLOT = BN * BKT;  // bf16 elements per X / W ring slot (32 KB each)
constexpr int NXS = 3, NWS = 2;                 // ring slots: X two tiles ahead, W one tile ahead
constexpr int N_XCD = 8;
constexpr int TM = 4;                           // 32-token MFMA tiles per wave sub-tile (128 tokens)

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

// element offset of (row, 16-byte chunk) in a [rows][64] bf16 tile: 256-byte super-rows (two
// 128-byte K rows) with the 16-byte slot XOR-ed by the super-row number
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

// Epilogue of one wave's sub-tile of 128 tokens (first token mrow0 of sample rows grow0..) x 64
// features (first feature ncol0): acc[tn][tm] is the 32x32x16 MFMA accumulator of features
// tn*32.., tokens tm*32.. with the weight tile as the MFMA "A" operand.
// Accumulator entry q*4+e of lane (l32, lhi): token tm*32 + l32, feature tn*32 + q*8 + lhi*4 + e.
// v_permlane32_swap pairs lane l with l+32 so that lanes < 32 own features [q0*8, q0*8+8) and
// lanes >= 32 own [q1*8, q1*8+8), (q0, q1) = (0,1), (2,3).  Bias and activation are applied in
// registers, then the wave transposes the sub-tile through its private 16 KB of LDS (`stg`) so
// that every global store instruction writes 8 rows x 128 contiguous bytes (the residual is read
// with the same pattern).  Calls of one wave on the same `stg` need no barrier in between: the
// LDS serves a wave's accesses in order.
template <int ACT>
__device__ __forceinline__ void epilogue_128x64(const GemmArgs &a, const f32x16 (&acc)[2][TM], char *stg,
                                                const __bf16 *bias, int ncol0, int mrow0, int64_t grow0, int lane)
{
    constexpr int TN = 2;
    const int l32 = lane & 31, lhi = lane >> 5;
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

}  // namespace gemm_tile
}  // namespace sf
