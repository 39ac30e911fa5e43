// Block-wide exact top-k selection over keys held in LDS, with the tie rule
// "higher key first, then lower index".  Used for the gate-score keep sets
// (Sec. 4.5) and for the top-U query choice of SentryAttend (Sec. 4.4).
//
// The k-th largest key is found by a 4-pass radix select (8 bits per pass, a
// 256-bin LDS histogram with integer atomics: the counts, hence the result,
// do not depend on the order of the atomics).  The kept indices are then
// emitted in ascending order from contiguous per-thread index ranges with two
// block-wide prefix sums.
#pragma once

#include "common.hpp"

namespace sf {

constexpr int TOPK_SCRATCH = 256 + 16 + 2;      // ints of LDS scratch block_topk needs

// Sum of one int per thread over the block; every thread gets the total.
// `red` is LDS scratch of at least NT/64 ints.
template <int NT>
__device__ __forceinline__ int block_sum(int v, int *red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    int t = 0;
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) t += red[i];
    return t;
}

// Exclusive prefix sum of one int per thread in thread order; `total` gets the
// block total.  `red` is LDS scratch of at least NT/64 ints.
template <int NT>
__device__ __forceinline__ int block_excl_scan(int v, int *red, int &total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(x, o);
        if (lane >= o) x += t;
    }
    __syncthreads();
    if (lane == 63) red[w] = x;
    __syncthreads();
    int off = 0, t = 0;
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) {
        const int c = red[i];
        if (i < w) off += c;
        t += c;
    }
    total = t;
    return off + x - v;
}

// keys[0..n) in LDS (already synchronised).  Selects the k largest
// (1 <= k <= n).  For every index i, in ascending order within a thread,
// calls emit(i, kept, pos) where pos is the rank of i among the kept indices
// (ascending index order) when kept.  Must be called by all NT threads;
// `scratch` is LDS of TOPK_SCRATCH ints.
template <int NT, class Emit>
__device__ void block_topk(const uint32_t *keys, int n, int k, int *scratch, Emit emit)
{
    int *hist = scratch, *red = scratch + 256, *res = scratch + 256 + 16;
    const int tid = threadIdx.x, lane = tid & 63;
    __syncthreads();        // nobody may still be reading `scratch` (or writing `keys`) from before the call

    // k-th largest key T, most significant byte first
    uint32_t prefix = 0, mask = 0;
    int kk = k;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        for (int j = tid; j < 256; j += NT) hist[j] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += NT) {
            const uint32_t key = keys[i];
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        if (tid < 64) {
            // lane owns bins 4*lane .. 4*lane+3; find the bin holding the kk-th largest candidate
            int h[4], local = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { h[j] = hist[4 * lane + j]; local += h[j]; }
            int incl = local;                       // becomes the sum over lanes >= lane
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_down(incl, o);
                if (lane + o < 64) incl += t;
            }
            int run = incl - local;                 // candidates in strictly higher bins
#pragma unroll
            for (int j = 3; j >= 0; --j) {
                if (run < kk && run + h[j] >= kk) { res[0] = 4 * lane + j; res[1] = kk - run; }
                run += h[j];
            }
        }
        __syncthreads();
        prefix |= (uint32_t)res[0] << shift;
        mask |= 255u << shift;
        kk = res[1];
        __syncthreads();                            // res is rewritten in the next pass
    }
    const uint32_t T = prefix;
    const int need = kk;                            // how many keys == T are kept (lowest indices)

    // emit in ascending index order: thread t owns indices [t*E, (t+1)*E)
    const int E = (n + NT - 1) / NT;
    const int i0 = min(n, tid * E), i1 = min(n, i0 + E);
    int c_gt = 0, c_eq = 0;
    for (int i = i0; i < i1; ++i) { const uint32_t key = keys[i]; c_gt += key > T; c_eq += key == T; }
    int tot;
    const int eq_before = block_excl_scan<NT>(c_eq, red, tot);
    const int eq_kept = max(0, min(c_eq, need - eq_before));
    int pos = block_excl_scan<NT>(c_gt + eq_kept, red, tot);
    int eqr = eq_before;
    for (int i = i0; i < i1; ++i) {
        const uint32_t key = keys[i];
        const bool eq = key == T;
        const bool kept = key > T || (eq && eqr < need);
        eqr += eq;
        emit(i, kept, pos);
        pos += kept;
    }
}

}  // namespace sf
