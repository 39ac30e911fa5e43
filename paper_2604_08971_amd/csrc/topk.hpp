// Block-wide exact top-k selection over keys held in LDS, with the tie rule
// "higher key first, then lower index".  Used for the gate-score keep sets
// (Sec. 4.5) and for the top-U query choice of SentryAttend (Sec. 4.4).
#pragma once

#include "common.hpp"

namespace sf {

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

// Exclusive prefix count of a 0/1 flag in thread order; `total` gets the block
// total.  `red` is LDS scratch of at least NT/64 ints.
template <int NT>
__device__ __forceinline__ int block_excl_count(bool flag, int *red, int &total)
{
    const unsigned long long bal = __ballot(flag);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int below = __popcll(bal & ((1ull << lane) - 1ull));
    __syncthreads();
    if (lane == 0) red[w] = __popcll(bal);
    __syncthreads();
    int off = 0, t = 0;
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) {
        const int c = red[i];
        if (i < w) off += c;
        t += c;
    }
    total = t;
    return off + below;
}

// keys[0..n) in LDS (already synchronised).  Selects the k largest
// (1 <= k <= n).  For every index i, in ascending order within a thread,
// calls emit(i, kept, pos) where pos is the rank of i among the kept indices
// (ascending index order) when kept.  Must be called by all NT threads.
template <int NT, class Emit>
__device__ void block_topk(const uint32_t *keys, int n, int k, int *red, Emit emit)
{
    // k-th largest key: the largest T with #{key >= T} >= k, built bit by bit
    uint32_t T = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        int c = 0;
        for (int i = threadIdx.x; i < n; i += NT) c += keys[i] >= cand;
        if (block_sum<NT>(c, red) >= k) T = cand;
    }
    int c = 0;
    for (int i = threadIdx.x; i < n; i += NT) c += keys[i] > T;
    const int need = k - block_sum<NT>(c, red);     // how many keys == T are kept (lowest indices)

    int eq_base = 0, kept_base = 0;
    for (int i0 = 0; i0 < n; i0 += NT) {
        const int i = i0 + threadIdx.x;
        const bool in = i < n;
        const uint32_t key = in ? keys[i] : 0u;
        const bool eq = in && key == T;
        int eq_total, kept_total;
        const int eq_rank = eq_base + block_excl_count<NT>(eq, red, eq_total);
        const bool kept = in && (key > T || (eq && eq_rank < need));
        const int pos = kept_base + block_excl_count<NT>(kept, red, kept_total);
        if (in) emit(i, kept, pos);
        eq_base += eq_total;
        kept_base += kept_total;
    }
}

}  // namespace sf
