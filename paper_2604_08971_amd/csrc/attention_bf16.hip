// SentryAttend on bf16 MFMA (Sec. 4.4 of the paper, Eq. (6)).
//
// Both kernels compute the TRANSPOSED score tile S^T = K_tile . Q^T with
// 32x32x16 MFMAs, so that one accumulator lane owns ONE query (column
// lane % 32) and 16 of the tile's 32 keys.  Everything the softmax needs per
// query (running max, running sum, rescaling of the output accumulator) then
// lives in that lane; only one exchange with lane ^ 32 (the other 16 keys of
// the same query) is needed per tile.  The output is accumulated transposed
// as well, O^T = V^T . P^T, so P goes from accumulator registers straight
// into the MFMA "B" operand without leaving the lane; V is read from a
// [dh, L] (key-contiguous) layout so that its fragments are plain vector
// loads too.  K and V^T tiles are staged in LDS once per workgroup and shared
// by all waves, i.e. by all heads of the K/V group.
#include "attention.hpp"

namespace sf {

constexpr int NWAVE = 4;
constexpr int BKEY = 64;          // keys per LDS tile (two 32-key MFMA blocks)
constexpr int PAD = 8;            // bf16 elements of row padding (16 bytes) against bank conflicts
constexpr float LOG2E = 1.4426950408889634f;
constexpr float RESCALE_LOG2 = 8.0f;    // slack of the softmax reference below the running maximum, in powers of two
#define SF_SCORE_OCC __attribute__((amdgpu_waves_per_eu(4, 4)))

// Bit j%32 of word j/32 = key j of sample b is allowed (0 beyond L).
__device__ __forceinline__ void build_mask_words(const uint8_t *kv, int L, uint32_t *words, int nwords)
{
    // one position per lane, the words from the wave's ballot: a single round of byte loads for the whole block
    // (a lane that assembled a word by itself paid 32 loads one after the other)
    const int lane = threadIdx.x & 63;
    for (int j0 = 0; j0 < nwords * 32; j0 += (int)blockDim.x) {      // the same trip count for every wave
        const int j = j0 + (int)threadIdx.x;
        const bool ok = j < L && (!kv || kv[j]);
        const unsigned long long bal = __ballot(ok);
        const int w = j >> 5;
        if ((lane & 31) == 0 && w < nwords) words[w] = (uint32_t)(bal >> (lane & 32));
    }
}

// List of the 64-key tiles of [jbeg, jend) that contain at least one allowed key (ascending),
// built by the first wave; returns the count through *n_tiles.  Needs `words` complete.
__device__ __forceinline__ void build_tile_list(const uint32_t *words, int nwords, int jbeg, int jend,
                                                uint16_t *tiles, int *n_tiles)
{
    if (threadIdx.x < 64) {
        int base = 0;
        for (int t0 = jbeg / BKEY; t0 * BKEY < jend; t0 += 64) {
            const int t = t0 + (int)threadIdx.x;
            bool live = false;
            if (t * BKEY < jend) {
                const uint32_t w0 = words[2 * t], w1 = (2 * t + 1 < nwords) ? words[2 * t + 1] : 0u;
                live = (w0 | w1) != 0u;
            }
            const unsigned long long bal = __ballot(live);
            if (live) tiles[base + __popcll(bal & ((1ull << threadIdx.x) - 1ull))] = (uint16_t)t;
            base += __popcll(bal);
        }
        if (threadIdx.x == 0) *n_tiles = base;
    }
}

// K tile chunks of this thread -> registers (rows at or beyond L are zero); NT
// threads share a tile.  j0 must be wave-uniform: the tile base stays scalar
// and each lane adds a 32-bit offset that does not change from tile to tile.
template <int DH, int NT>
struct KTile {
    static constexpr int CH = DH / 8, TOTAL = BKEY * CH, N = (TOTAL + NT - 1) / NT;
    static __device__ __forceinline__ void fetch(const h16 *Kb, int64_t sl, int j0, int L, uint4 (&r)[N])
    {
        const char *base = reinterpret_cast<const char *>(Kb + (int64_t)j0 * sl);
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int c = threadIdx.x + u * NT;
            const int row = c / CH, cc = c % CH;
            const uint32_t off = (uint32_t)row * (uint32_t)sl * 2u + (uint32_t)cc * 16u;   // < 64 rows * row stride bytes
            r[u] = ((TOTAL % NT == 0 || c < TOTAL) && j0 + row < L)
                       ? *reinterpret_cast<const uint4 *>(base + off) : make_uint4(0, 0, 0, 0);
        }
    }
    static __device__ __forceinline__ void put(const uint4 (&r)[N], h16 *Ks)
    {
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int c = threadIdx.x + u * NT;
            if (TOTAL % NT == 0 || c < TOTAL)
                *reinterpret_cast<uint4 *>(Ks + (c / CH) * (DH + PAD) + (c % CH) * 8) = r[u];
        }
    }
};

// ------------------------------------------------------------- sparsity score
// M_i = max_j s_ij - mean_j s_ij over allowed keys.  The max comes from the
// streamed S^T tiles; the mean is q_i . mean_key (computed once per group),
// which is the same number up to fp32 rounding.
// 1-D grid over (query block, sample*head) items, query block fastest; each
// wave owns QBS blocks of 32 queries.  The launch index is folded so that all
// query blocks of one (sample, head) - and of the neighbouring heads, which
// mostly share the K/V group - run on one XCD and find K in its L2.  K tiles
// are double-buffered in LDS and the next tile is prefetched into registers
// while the current one is multiplied, so one barrier per tile suffices.
template <int DH, int QBS>
__global__ __launch_bounds__(NWAVE * 64) SF_SCORE_OCC void score_bf16_kernel(
    const h16 *__restrict__ Q, sf_strides sq, const h16 *__restrict__ K, sf_strides sk,
    const int32_t *__restrict__ head_group, int hg_stride, const int32_t *__restrict__ pattern_id,
    const uint8_t *__restrict__ query_valid, const uint8_t *__restrict__ key_mask,
    const float *__restrict__ stats, int nH, int nG, int L, int Lk, float *__restrict__ score, int scoreH,
    int qblocks, int n_items, const int32_t *__restrict__ row0, const int32_t *__restrict__ row0_k)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    h16 *Ks = reinterpret_cast<h16 *>(smem);                              // [2][BKEY][DH+PAD]
    float *kbar = reinterpret_cast<float *>(Ks + 2 * BKEY * (DH + PAD));        // [DH]
    uint32_t *words = reinterpret_cast<uint32_t *>(kbar + DH);                  // [ceil(Lk/32)]
    uint16_t *tiles = reinterpret_cast<uint16_t *>(words + (Lk + 31) / 32);     // [ceil(Lk/64)]
    __shared__ int n_tiles;

    const int item = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
    if (item >= n_items) return;                          // uniform
    const int qblk = item % qblocks, bh = item / qblocks, b = bh / nH, h = bh % nH;
    const int g = head_group[(int64_t)(pattern_id ? pattern_id[b] : 0) * hg_stride + h];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lhi = lane >> 5;
    const uint8_t *kv = query_valid ? query_valid + (int64_t)b * L : nullptr;
    const int nwords = (Lk + 31) / 32;
    build_mask_words(key_mask ? key_mask + (int64_t)b * Lk : nullptr, Lk, words, nwords);
    if (threadIdx.x < DH) kbar[threadIdx.x] = stats[((int64_t)b * nG + g) * 2 * DH + threadIdx.x];

    // packed samples: Q (and K, unless it is the gathered key sample of the workspace) start at the sample's own row
    const h16 *Qb = Q + sample_offset(row0, b, sq) + (int64_t)h * sq.h;
    const h16 *Kb = K + sample_offset(row0_k, b, sk) + (int64_t)g * sk.h;
    const int q0 = (qblk * NWAVE + wave) * QBS * 32;

    h16x8 qf[QBS][DH / 16];
    float rmax[QBS];
#pragma unroll
    for (int qq = 0; qq < QBS; ++qq) {
        const int i = min(q0 + qq * 32 + l32, L - 1);
#pragma unroll
        for (int kk = 0; kk < DH / 16; ++kk)
            qf[qq][kk] = *reinterpret_cast<const h16x8 *>(Qb + (int64_t)i * sq.l + kk * 16 + lhi * 8);
        rmax[qq] = -INFINITY;
    }
    __syncthreads();
    build_tile_list(words, nwords, 0, Lk, tiles, &n_tiles);
    __syncthreads();
    const int nt = n_tiles;

    using KT_ = KTile<DH, NWAVE * 64>;
    uint4 kreg[KT_::N];
    auto tile_j0 = [&](int it) { return __builtin_amdgcn_readfirstlane((int)tiles[it]) * BKEY; };   // same for every lane
    if (nt > 0) KT_::fetch(Kb, sk.l, tile_j0(0), Lk, kreg);
    for (int it = 0; it < nt; ++it) {
        const int j0 = tile_j0(it);
        h16 *Kt = Ks + (it & 1) * BKEY * (DH + PAD);
        KT_::put(kreg, Kt);
        __syncthreads();        // tile `it` visible; everyone is done with tile it-1 (the other buffer)
        if (it + 1 < nt) KT_::fetch(Kb, sk.l, tile_j0(it + 1), Lk, kreg);
        // the mask words are the same for every lane: keep them scalar
        const uint32_t w0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)words[j0 / 32]);
        const uint32_t w1 = (j0 / 32 + 1 < nwords) ? (uint32_t)__builtin_amdgcn_readfirstlane((int)words[j0 / 32 + 1]) : 0u;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const uint32_t w = kb ? w1 : w0;
            if (w == 0u) continue;
            h16x8 kf[DH / 16];
#pragma unroll
            for (int kk = 0; kk < DH / 16; ++kk)
                kf[kk] = *reinterpret_cast<const h16x8 *>(Kt + (kb * 32 + l32) * (DH + PAD) + kk * 16 + lhi * 8);
            if (w == 0xffffffffu) {                 // scalar branch: the usual tile, no masking
#pragma unroll
                for (int qq = 0; qq < QBS; ++qq) {
                    f32x16 s;
#pragma unroll
                    for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
                    for (int kk = 0; kk < DH / 16; ++kk)
                        s = SF_MFMA16(kf[kk], qf[qq][kk], s, 0, 0, 0);
                    float m = rmax[qq];
#pragma unroll
                    for (int e = 0; e < 16; e += 2) m = fmaxf(fmaxf(m, s[e]), s[e + 1]);
                    rmax[qq] = m;
                }
            } else {
                const uint32_t wl = w >> (lhi * 4);
#pragma unroll
                for (int qq = 0; qq < QBS; ++qq) {
                    f32x16 s;
#pragma unroll
                    for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
                    for (int kk = 0; kk < DH / 16; ++kk)
                        s = SF_MFMA16(kf[kk], qf[qq][kk], s, 0, 0, 0);
                    float m = rmax[qq];
#pragma unroll
                    for (int e = 0; e < 16; ++e)       // key row of s[e]: (e/4)*8 + lhi*4 + e%4
                        m = fmaxf(m, ((wl >> ((e / 4) * 8 + (e % 4))) & 1u) ? s[e] : -INFINITY);
                    rmax[qq] = m;
                }
            }
        }
    }

    const float scale = 1.0f / sqrtf((float)DH);
#pragma unroll
    for (int qq = 0; qq < QBS; ++qq) {
        float m = fmaxf(rmax[qq], __shfl_xor(rmax[qq], 32));
        float dot = 0.f;
#pragma unroll
        for (int kk = 0; kk < DH / 16; ++kk)
#pragma unroll
            for (int e = 0; e < 8; ++e) dot = fmaf((float)qf[qq][kk][e], kbar[kk * 16 + lhi * 8 + e], dot);
        dot += __shfl_xor(dot, 32);
        const int i = q0 + qq * 32 + l32;
        if (lhi == 0 && i < L) {
            const bool ok = !kv || kv[i];
            score[((int64_t)b * scoreH + h) * L + i] = !ok ? -INFINITY : nt == 0 ? 0.f : (m - dot) * scale;   // no key: 0
        }
    }
}

// v_permlane32_swap exchanges lanes 32..63 of its first operand with lanes 0..31 of its second: fed the same value
// twice, lane l then holds v[l % 32] in the first result and v[32 + l % 32] in the second - the values of the two
// lanes that share a query.
__device__ __forceinline__ float both_halves_max(float v)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float both_halves_sum(float v)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// ---------------------------------------------------------------- active pass
// A "pair" is (head of the group, block of 32 active queries).  A workgroup of
// AWAVE waves serves one (sample, K/V group, key split): each wave owns QB
// pairs and all waves share the K / V^T tiles staged in LDS; a group with more
// pairs than AWAVE*QB is served in several passes over the key range.
// 1-D grid; the launch index is folded so that consecutive work items (the
// pair chunks of one (sample, group), which read the same K/V) run on the same
// XCD and share its L2, and the items are spread evenly over the XCDs.
constexpr int AWAVE = 8;

// (139 registers at dh = 64: one workgroup per compute unit.  Capping the allocation at 128 registers so that two fit
// was faster where the launch has more workgroups than compute units - C5 active pass 40 -> 33.5 us, C3 66 -> 49.5 us -
// but the build with its eight spilled registers gave wrong rows whenever a pass left waves without a pair, with or
// without the key groups and with or without a second workgroup on the compute unit; no cause was found in the
// source, so that build is not used.)
// NW = waves per workgroup.  Four instead of eight where a (sample, group) has at most four pairs: the same registers
// per wave then leave room for three workgroups per compute unit, and no wave is without a pair.
template <int DH, int QB, int NW>
__global__ __launch_bounds__(NW * 64) void attend_bf16_kernel(
    const h16 *__restrict__ Q, sf_strides sq, const h16 *__restrict__ K, sf_strides sk,
    const h16 *__restrict__ VT, sf_strides svt, const int32_t *__restrict__ head_group, int hg_stride,
    const int32_t *__restrict__ pattern_id, const uint8_t *__restrict__ key_valid,
    const int32_t *__restrict__ sel, int selH, int nH, int nG, int BG, int chunks, int L, int Lp, int U,
    int Upad, int splits, int keys_per_split, h16 *__restrict__ O, int64_t ldo,
    float *__restrict__ part_o, float *__restrict__ part_ml, const int32_t *__restrict__ row0)
{
    constexpr int NT = NW * 64;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int KT = BKEY * (DH + PAD), VT_ = DH * (BKEY + PAD);          // elements of one K / V^T tile
    h16 *Ks = reinterpret_cast<h16 *>(smem);                         // [2][BKEY][DH+PAD]
    h16 *Vs = Ks + 2 * KT;                                              // [2][DH][BKEY+PAD]
    uint32_t *words = reinterpret_cast<uint32_t *>(Vs + 2 * VT_);          // [ceil(L/32)]
    uint16_t *tiles = reinterpret_cast<uint16_t *>(words + (L + 31) / 32); // [ceil(L/64)]
    __shared__ int heads[64];
    __shared__ int n_heads, n_tiles;

    // launch index -> work item: XCD x (launch index % 8) takes the x-th eighth of the items
    const int per_xcd = gridDim.x / 8;
    const int item = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (item >= chunks * BG * splits) return;             // uniform
    const int chunk = item % chunks, bg = (item / chunks) % BG, sp = item / (chunks * BG);
    const int b = bg / nG, g = bg % nG;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lhi = lane >> 5;
    const int32_t *hg = head_group + (int64_t)(pattern_id ? pattern_id[b] : 0) * hg_stride;

    if (wave == 0) {                      // ordered list of the group's heads (nH <= 64)
        const bool mine = lane < nH && hg[lane] == g;
        const unsigned long long bal = __ballot(mine);
        if (mine) heads[__popcll(bal & ((1ull << lane) - 1ull))] = lane;
        if (lane == 0) n_heads = __popcll(bal);
    }
    const uint8_t *kv = key_valid ? key_valid + (int64_t)b * L : nullptr;
    const int nwords = (L + 31) / 32;
    build_mask_words(kv, L, words, nwords);
    const int jbeg = sp * keys_per_split, jend = min(L, jbeg + keys_per_split);
    __syncthreads();
    build_tile_list(words, nwords, jbeg, jend, tiles, &n_tiles);
    __syncthreads();
    const int nt = n_tiles;
    const int nqb = Upad / 32;
    const int npairs = n_heads * nqb;

    const h16 *Kb = K + sample_offset(row0, b, sk) + (int64_t)g * sk.h;
    const h16 *Vb = VT + (int64_t)b * svt.b + (int64_t)g * svt.h;        // the transposed V is always b-strided
    const float sc = LOG2E / sqrtf((float)DH);

    // V^T tile chunks of this thread -> registers; keys at or beyond L are zeroed
    constexpr int VTOTAL = DH * (BKEY / 8), NV = (VTOTAL + NT - 1) / NT;
    auto fetch_v = [&](int j0, uint4 (&r)[NV]) {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int c = threadIdx.x + u * NT;
            const int e = c / (BKEY / 8), cc = c % (BKEY / 8);
            const int j = j0 + cc * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if ((VTOTAL % NT == 0 || c < VTOTAL) && j < Lp) {
                const uint32_t off = (uint32_t)e * (uint32_t)svt.l * 2u + (uint32_t)cc * 16u;   // < dh rows of Lp keys
                v = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(Vb + j0) + off);
            }
            r[u] = v;          // (keys at or beyond L are zeroed when the chunk is written to LDS: touching the value
                               // here would make the wave wait for the load it has just issued)
        }
    };
    auto put_v = [&](const uint4 (&r)[NV], h16 *Vt, int j0) {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int c = threadIdx.x + u * NT;
            if (VTOTAL % NT == 0 || c < VTOTAL) {
                uint4 v = r[u];
                const int j = j0 + (c % (BKEY / 8)) * 8;
                if (j + 8 > L) {                       // last tile of a ragged row only
                    uint16_t *hv = reinterpret_cast<uint16_t *>(&v);
#pragma unroll
                    for (int t = 0; t < 8; ++t)
                        if (j + t >= L) hv[t] = 0;
                }
                *reinterpret_cast<uint4 *>(Vt + (c / (BKEY / 8)) * (BKEY + PAD) + (c % (BKEY / 8)) * 8) = v;
            }
        }
    };
    using KT_ = KTile<DH, NT>;
    auto tile_j0 = [&](int it) { return __builtin_amdgcn_readfirstlane((int)tiles[it]) * BKEY; };   // same for every lane

    for (int pair0 = chunk * (NW * QB); pair0 < npairs; pair0 += chunks * (NW * QB)) {
        // When this pass has pairs for at most half of the waves (few active rows: U = c*ceil(ln L) gives one or two
        // blocks of 32 per head), the others would only help with the staging: instead KG groups of waves take the
        // same pairs and every KG-th key tile each, and their partial results are merged through LDS at the end.
        int kg = 1;
        {
            const int waves_used = (min(npairs - pair0, NW * QB) + QB - 1) / QB;
            // only where the launch is short of workgroups (the host split the keys for that reason): with a
            // (sample, group) problem per compute unit or more the idle waves cost nothing and the merge does
            while (splits > 1 && waves_used * kg * 2 <= NW) kg *= 2;
        }
        const int pslots = NW / kg;                  // waves that hold distinct pairs
        const int pw = wave % pslots, kgi = wave / pslots;
        int head[QB], qidx[QB], slot[QB];
        h16x8 qf[QB][DH / 16];
#pragma unroll
        for (int qq = 0; qq < QB; ++qq) {
            const int pi = pair0 + pw * QB + qq;
            head[qq] = -1; qidx[qq] = -1; slot[qq] = 0;
            if (pi < npairs) {
                head[qq] = heads[pi / nqb];
                slot[qq] = (pi % nqb) * 32 + l32;
                if (slot[qq] < U) qidx[qq] = sel[((int64_t)b * selH + head[qq]) * U + slot[qq]];
            }
            const h16 *qrow = Q + sample_offset(row0, b, sq) + (int64_t)max(head[qq], 0) * sq.h +
                                 (int64_t)max(qidx[qq], 0) * sq.l;
#pragma unroll
            for (int kk = 0; kk < DH / 16; ++kk)
                qf[qq][kk] = *reinterpret_cast<const h16x8 *>(qrow + kk * 16 + lhi * 8);
        }
        const bool idle = pair0 + pw * QB >= npairs;          // wave-uniform: no pair at all

        f32x16 oacc[QB][DH / 32];
        float m_run[QB], l_run[QB];
#pragma unroll
        for (int qq = 0; qq < QB; ++qq) {
            m_run[qq] = -INFINITY; l_run[qq] = 0.f;
#pragma unroll
            for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[qq][db][e] = 0.f;
        }

        uint4 kreg[KT_::N], vreg[NV];
        if (nt > 0) { KT_::fetch(Kb, sk.l, tile_j0(0), L, kreg); fetch_v(tile_j0(0), vreg); }

        for (int it = 0; it < nt; ++it) {
            const int j0 = tile_j0(it);
            h16 *Kt = Ks + (it & 1) * KT, *Vt = Vs + (it & 1) * VT_;
            KT_::put(kreg, Kt);
            put_v(vreg, Vt, j0);
            __syncthreads();        // tile `it` visible; everyone is done with tile it-1 (the other buffers)
            if (it + 1 < nt) { const int jn = tile_j0(it + 1); KT_::fetch(Kb, sk.l, jn, L, kreg); fetch_v(jn, vreg); }
            if (idle || (it & (kg - 1)) != kgi) continue;          // not this wave's tile
            const uint32_t w0 = words[j0 / 32], w1 = (j0 / 32 + 1 < nwords) ? words[j0 / 32 + 1] : 0u;
            // the same for every lane: a tile with all 64 keys allowed skips the masking
            const bool all_allowed = (uint32_t)__builtin_amdgcn_readfirstlane((int)(w0 & w1)) == 0xffffffffu;

            // S^T blocks for the two 32-key halves
            f32x16 s[QB][2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                h16x8 kf[DH / 16];
#pragma unroll
                for (int kk = 0; kk < DH / 16; ++kk)
                    kf[kk] = *reinterpret_cast<const h16x8 *>(Kt + (kb * 32 + l32) * (DH + PAD) + kk * 16 + lhi * 8);
#pragma unroll
                for (int qq = 0; qq < QB; ++qq) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) s[qq][kb][e] = 0.f;
#pragma unroll
                    for (int kk = 0; kk < DH / 16; ++kk)
                        s[qq][kb] = SF_MFMA16(kf[kk], qf[qq][kk], s[qq][kb], 0, 0, 0);
                }
            }

            // online softmax per query (per lane), log2 domain
            h16x8 pf[QB][4];
#pragma unroll
            for (int qq = 0; qq < QB; ++qq) {
                if (!all_allowed) {
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb) {
                        const uint32_t wl = (kb ? w1 : w0) >> (lhi * 4);
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            if (!((wl >> ((e / 4) * 8 + (e % 4))) & 1u)) s[qq][kb][e] = -INFINITY;
                    }
                }
                float mt = fmaxf(fmaxf(s[qq][0][0], s[qq][0][1]), s[qq][1][0]);
                mt = fmaxf(fmaxf(mt, s[qq][1][1]), s[qq][0][2]);
#pragma unroll
                for (int e = 3; e < 15; e += 2) mt = fmaxf(fmaxf(mt, s[qq][0][e]), s[qq][0][e + 1]);
#pragma unroll
                for (int e = 2; e < 16; e += 2) mt = fmaxf(fmaxf(mt, s[qq][1][e]), s[qq][1][e + 1]);
                mt = fmaxf(mt, s[qq][0][15]) * sc;         // sc > 0: max and scaling commute
                mt = both_halves_max(mt);                  // the other 16 keys of each 32-key block sit in lane ^ 32
                // The reference m_run of the exponentials only has to stay within 2^RESCALE_LOG2 of the true running
                // maximum (sums and outputs are relative to the same reference, so the result does not depend on
                // it): it moves, and the accumulators are rescaled, only when some query of the wave needs it.
                // After the first tiles of a row that is rare, which removes the rescaling from the common path.
                if (__builtin_expect(__builtin_amdgcn_ballot_w64(mt > m_run[qq] + RESCALE_LOG2) != 0ull, 0)) {
                    const float m_new = fmaxf(m_run[qq], mt);
                    const float alpha = __builtin_amdgcn_exp2f(m_run[qq] - (m_new == -INFINITY ? 0.f : m_new));
                    m_run[qq] = m_new;
                    l_run[qq] *= alpha;
#pragma unroll
                    for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                        for (int e = 0; e < 16; ++e) oacc[qq][db][e] *= alpha;
                }
                const float nm = m_run[qq] == -INFINITY ? 0.f : -m_run[qq];
                float rs0 = 0.f, rs1 = 0.f;
                // k-step t covers keys 16t..16t+15; this lane supplies keys
                // {16t + lhi*4 + 0..3, 16t + 8 + lhi*4 + 0..3} = accumulator entries (t%2)*8 + 0..7 of block t/2
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; e += 2) {
                        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[qq][kb][e], sc, nm));
                        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[qq][kb][e + 1], sc, nm));
                        rs0 += p0;
                        rs1 += p1;
                        reinterpret_cast<uint32_t *>(&pf[qq][kb * 2 + e / 8])[(e % 8) / 2] = pack2_h16(p0, p1);
                    }
                l_run[qq] += rs0 + rs1;
            }

            // O^T += V^T . P^T
#pragma unroll
            for (int db = 0; db < DH / 32; ++db) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const h16 *vrow = Vt + (db * 32 + l32) * (BKEY + PAD) + t * 16 + lhi * 4;
                    const h16x4 lo = *reinterpret_cast<const h16x4 *>(vrow);
                    const h16x4 hi = *reinterpret_cast<const h16x4 *>(vrow + 8);
                    h16x8 vf;
#pragma unroll
                    for (int e = 0; e < 4; ++e) { vf[e] = lo[e]; vf[4 + e] = hi[e]; }
#pragma unroll
                    for (int qq = 0; qq < QB; ++qq)
                        oacc[qq][db] = SF_MFMA16(vf, pf[qq][t], oacc[qq][db], 0, 0, 0);
                }
            }
        }

        // merge of the key groups: in log2(KG) rounds the upper half of the groups hands its running reference, sum
        // and accumulator over through the tile buffers (free now) and the lower half folds them into its own
        if (kg > 1) {
            float *mrg = reinterpret_cast<float *>(smem);              // [writer wave][QB * (DH/2 + 2)][64 lanes]
            constexpr int PER = QB * ((DH / 32) * 16 + 2);
            static_assert((NW / 2) * PER * 64 * 4 <= 2 * KT * 2 + 2 * VT_ * 2, "merge scratch must fit in the tile buffers");
            for (int step = kg / 2; step >= 1; step /= 2) {
                __syncthreads();                                       // tile buffers (or the last round's slots) are free
                if (kgi >= step && kgi < 2 * step) {
                    float *dst = mrg + (size_t)(wave - step * pslots) * PER * 64 + lane;
#pragma unroll
                    for (int qq = 0; qq < QB; ++qq) {
#pragma unroll
                        for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                            for (int e = 0; e < 16; ++e) dst[((qq * (DH / 32) + db) * 16 + e) * 64] = oacc[qq][db][e];
                        dst[(QB * (DH / 32) * 16 + qq * 2) * 64] = m_run[qq];
                        dst[(QB * (DH / 32) * 16 + qq * 2 + 1) * 64] = l_run[qq];
                    }
                }
                __syncthreads();
                if (kgi < step) {
                    const float *src = mrg + (size_t)wave * PER * 64 + lane;
#pragma unroll
                    for (int qq = 0; qq < QB; ++qq) {
                        const float m_o = src[(QB * (DH / 32) * 16 + qq * 2) * 64], l_o = src[(QB * (DH / 32) * 16 + qq * 2 + 1) * 64];
                        const float m_new = fmaxf(m_run[qq], m_o);
                        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                        const float a_me = __builtin_amdgcn_exp2f(m_run[qq] - m_safe), a_o = __builtin_amdgcn_exp2f(m_o - m_safe);
                        m_run[qq] = m_new;
                        l_run[qq] = l_run[qq] * a_me + l_o * a_o;
#pragma unroll
                        for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                            for (int e = 0; e < 16; ++e)
                                oacc[qq][db][e] = oacc[qq][db][e] * a_me + src[((qq * (DH / 32) + db) * 16 + e) * 64] * a_o;
                    }
                }
            }
        }

        // lane owns query l32 and output dims db*32 + ig*8 + lhi*4 + {0..3}
#pragma unroll
        for (int qq = 0; qq < QB; ++qq) {
            const float l_tot = both_halves_sum(l_run[qq]);
            if (qidx[qq] < 0 || kgi != 0) continue;
            if (splits <= 1) {
                const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
                h16 *orow = O + (sample_row(row0, b, L) + qidx[qq]) * ldo + (int64_t)head[qq] * DH;
#pragma unroll
                for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                    for (int ig = 0; ig < 4; ++ig) {
                        h16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (h16)(oacc[qq][db][ig * 4 + e] * inv);
                        *reinterpret_cast<h16x4 *>(orow + db * 32 + ig * 8 + lhi * 4) = o;
                    }
            } else {
                const int64_t base = (((int64_t)b * nH + head[qq]) * splits + sp) * Upad + slot[qq];   // [b, head, split, slot]
                float *po = part_o + base * DH;
#pragma unroll
                for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                    for (int ig = 0; ig < 4; ++ig) {
                        f32x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = oacc[qq][db][ig * 4 + e];
                        *reinterpret_cast<f32x4 *>(po + db * 32 + ig * 8 + lhi * 4) = o;
                    }
                if (lhi == 0) {
                    part_ml[base * 2] = m_run[qq];
                    part_ml[base * 2 + 1] = l_tot;
                }
            }
        }
        __syncthreads();            // the next pass restages both tile buffers
    }
}

// ------------------------------------------------- active pass, many active rows (dense-like patterns)
// Two pairs per wave as above, but the two waves of a SIMD are kept in OPPOSITE phases.  Measured on the plain loop
// (dense pattern, 16 x 8 heads x 4096^2): matrix-pipe work, softmax and tile staging took 430 + 220 + 125 us and
// added up to the kernel's 775 us - nothing overlapped, because after the tile's barrier both waves of a SIMD issue
// their MFMAs at the same time (the pipe alternates between them), then both run their softmax on the one vector
// ALU.  Here waves 0-3 (group 0) and waves 4-7 (group 1; wave w runs on SIMD w % 4) alternate between two clusters
// separated by workgroup barriers, group 1 one cluster behind group 0:
//     V(t): softmax of S(t) -> P(t) on the vector ALU, plus the group's share of the tile staging
//     M(t): P(t) V(t) and S(t+1) = K(t+1) Q^T on the matrix pipe
// so in every slot between two barriers one wave of each SIMD is in V and the other in M.  S(t+1) overwrites the
// registers of S(t), which V(t) has turned into P(t), so the register budget is that of the plain loop.
// Staging: group 0 writes V(t) during its V(t) cluster, group 1 writes K(t+2) during its V(t) cluster; each lands in
// a buffer whose last readers finished two slots earlier and is first read one slot later.
template <int DH>
__global__ __launch_bounds__(AWAVE * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attend_pp_bf16_kernel(
    const h16 *__restrict__ Q, sf_strides sq, const h16 *__restrict__ K, sf_strides sk,
    const h16 *__restrict__ VT, sf_strides svt, const int32_t *__restrict__ head_group, int hg_stride,
    const int32_t *__restrict__ pattern_id, const uint8_t *__restrict__ key_valid,
    const int32_t *__restrict__ sel, int selH, int nH, int nG, int BG, int chunks, int L, int Lp, int U,
    int Upad, int splits, int keys_per_split, h16 *__restrict__ O, int64_t ldo,
    float *__restrict__ part_o, float *__restrict__ part_ml, const int32_t *__restrict__ row0)
{
    constexpr int QB = 2, GT = (AWAVE / 2) * 64;                         // threads of a wave group
    static_assert(AWAVE == 8, "two groups of four waves, one wave of each per SIMD");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int KT = BKEY * (DH + PAD), VT_ = DH * (BKEY + PAD);          // elements of one K / V^T tile
    h16 *Ks = reinterpret_cast<h16 *>(smem);                         // [2][BKEY][DH+PAD]
    h16 *Vs = Ks + 2 * KT;                                              // [2][DH][BKEY+PAD]
    uint32_t *words = reinterpret_cast<uint32_t *>(Vs + 2 * VT_);          // [ceil(L/32)]
    uint16_t *tiles = reinterpret_cast<uint16_t *>(words + (L + 31) / 32); // [ceil(L/64)]
    __shared__ int heads[64];
    __shared__ int n_heads, n_tiles;

    const int per_xcd = gridDim.x / 8;
    const int item = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (item >= chunks * BG * splits) return;             // uniform
    const int chunk = item % chunks, bg = (item / chunks) % BG, sp = item / (chunks * BG);
    const int b = bg / nG, g = bg % nG;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lhi = lane >> 5;
    const int grp = __builtin_amdgcn_readfirstlane(wave >> 2), gtid = threadIdx.x & (GT - 1);
    const int32_t *hg = head_group + (int64_t)(pattern_id ? pattern_id[b] : 0) * hg_stride;

    if (wave == 0) {                      // ordered list of the group's heads (nH <= 64)
        const bool mine = lane < nH && hg[lane] == g;
        const unsigned long long bal = __ballot(mine);
        if (mine) heads[__popcll(bal & ((1ull << lane) - 1ull))] = lane;
        if (lane == 0) n_heads = __popcll(bal);
    }
    const uint8_t *kv = key_valid ? key_valid + (int64_t)b * L : nullptr;
    const int nwords = (L + 31) / 32;
    build_mask_words(kv, L, words, nwords);
    const int jbeg = sp * keys_per_split, jend = min(L, jbeg + keys_per_split);
    __syncthreads();
    build_tile_list(words, nwords, jbeg, jend, tiles, &n_tiles);
    __syncthreads();
    const int nt = n_tiles;
    const int nqb = Upad / 32;
    const int npairs = n_heads * nqb;

    const h16 *Kb = K + sample_offset(row0, b, sk) + (int64_t)g * sk.h;
    const h16 *Vb = VT + (int64_t)b * svt.b + (int64_t)g * svt.h;        // the transposed V is always b-strided
    const float sc = LOG2E / sqrtf((float)DH);

    // Tile chunks (16 bytes) of one thread of a group -> registers -> LDS.  K rows at or beyond L and V^T keys at or
    // beyond L are zero.  The thread's offsets are re-formed from an opaque copy of its index at every use: kept
    // live across the loop they are spilled, and a reload from scratch inside the loop is a vector-memory operation
    // whose wait also waits for the tile loads just issued (measured: 1200 clocks per tile in the fetch alone).
    constexpr int KCH = DH / 8, KTOTAL = BKEY * KCH, NK = (KTOTAL + GT - 1) / GT;
    constexpr int VTOTAL = DH * (BKEY / 8), NV = (VTOTAL + GT - 1) / GT;
    auto fetch_k = [&](int j0, uint4 (&r)[NK]) {
        int gt = gtid;
        asm volatile("" : "+v"(gt));      // re-formed at every use, see below
        const char *base = reinterpret_cast<const char *>(Kb + (int64_t)j0 * sk.l);
#pragma unroll
        for (int u = 0; u < NK; ++u) {
            const int c = gt + u * GT;
            const int row = c / KCH, cc = c % KCH;
            const uint32_t off = (uint32_t)row * (uint32_t)sk.l * 2u + (uint32_t)cc * 16u;
            r[u] = ((KTOTAL % GT == 0 || c < KTOTAL) && j0 + row < L)
                       ? *reinterpret_cast<const uint4 *>(base + off) : make_uint4(0, 0, 0, 0);
        }
    };
    auto put_k = [&](const uint4 (&r)[NK], h16 *Kt) {
        int gt = gtid;
        asm volatile("" : "+v"(gt));      // re-formed at every use, see below
#pragma unroll
        for (int u = 0; u < NK; ++u) {
            const int c = gt + u * GT;
            if (KTOTAL % GT == 0 || c < KTOTAL)
                *reinterpret_cast<uint4 *>(Kt + (c / KCH) * (DH + PAD) + (c % KCH) * 8) = r[u];
        }
    };
    auto fetch_v = [&](int j0, uint4 (&r)[NV]) {
        int gt = gtid;
        asm volatile("" : "+v"(gt));      // re-formed at every use, see below
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int c = gt + u * GT;
            const int e = c / (BKEY / 8), cc = c % (BKEY / 8);
            const int j = j0 + cc * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if ((VTOTAL % GT == 0 || c < VTOTAL) && j < Lp) {
                const uint32_t off = (uint32_t)e * (uint32_t)svt.l * 2u + (uint32_t)cc * 16u;   // < dh rows of Lp keys
                v = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(Vb + j0) + off);
            }
            r[u] = v;          // (keys at or beyond L are zeroed when the chunk is written to LDS: touching the value
                               // here would make the wave wait for the load it has just issued)
        }
    };
    auto put_v = [&](const uint4 (&r)[NV], h16 *Vt, int j0) {
        int gt = gtid;
        asm volatile("" : "+v"(gt));      // re-formed at every use, see below
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int c = gt + u * GT;
            if (VTOTAL % GT == 0 || c < VTOTAL) {
                uint4 v = r[u];
                const int j = j0 + (c % (BKEY / 8)) * 8;
                if (j + 8 > L) {                       // last tile of a ragged row only
                    uint16_t *hv = reinterpret_cast<uint16_t *>(&v);
#pragma unroll
                    for (int t = 0; t < 8; ++t)
                        if (j + t >= L) hv[t] = 0;
                }
                // chunk cc holds keys 8cc..8cc+7 of the row; inside every group of 16 keys the LDS order is
                // [0-3, 8-11, 4-7, 12-15], so that the 8 keys a lane supplies per MFMA are 16 contiguous bytes
                const int cc = c % (BKEY / 8);
                h16 *dst = Vt + (c / (BKEY / 8)) * (BKEY + PAD) + (cc >> 1) * 16 + (cc & 1) * 4;
                *reinterpret_cast<uint2 *>(dst) = make_uint2(v.x, v.y);
                *reinterpret_cast<uint2 *>(dst + 8) = make_uint2(v.z, v.w);
            }
        }
    };
    auto tile_j0 = [&](int it) { return __builtin_amdgcn_readfirstlane((int)tiles[it]) * BKEY; };   // same for every lane

    for (int pair0 = chunk * (AWAVE * QB); pair0 < npairs; pair0 += chunks * (AWAVE * QB)) {
        int head[QB], qidx[QB], slot[QB];
        h16x8 qf[QB][DH / 16];
#pragma unroll
        for (int qq = 0; qq < QB; ++qq) {
            const int pi = pair0 + wave * QB + qq;
            head[qq] = -1; qidx[qq] = -1; slot[qq] = 0;
            if (pi < npairs) {
                head[qq] = heads[pi / nqb];
                slot[qq] = (pi % nqb) * 32 + l32;
                if (slot[qq] < U) qidx[qq] = sel[((int64_t)b * selH + head[qq]) * U + slot[qq]];
            }
            const h16 *qrow = Q + sample_offset(row0, b, sq) + (int64_t)max(head[qq], 0) * sq.h +
                                 (int64_t)max(qidx[qq], 0) * sq.l;
#pragma unroll
            for (int kk = 0; kk < DH / 16; ++kk)
                qf[qq][kk] = *reinterpret_cast<const h16x8 *>(qrow + kk * 16 + lhi * 8);
        }
        const bool idle = pair0 + wave * QB >= npairs;        // wave-uniform: no pair at all (still stages and syncs)

        f32x16 oacc[QB][DH / 32];
        float m_run[QB], l_run[QB];
#pragma unroll
        for (int qq = 0; qq < QB; ++qq) {
            m_run[qq] = -INFINITY; l_run[qq] = 0.f;
#pragma unroll
            for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[qq][db][e] = 0.f;
        }
        f32x16 s[QB][2];
        h16x8 pf[QB][4];

        // S^T of both pairs for the 64 keys of a K tile (every K fragment serves both pairs)
        auto s_tile = [&](const h16 *Kt) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                h16x8 kf[DH / 16];
#pragma unroll
                for (int kk = 0; kk < DH / 16; ++kk)
                    kf[kk] = *reinterpret_cast<const h16x8 *>(Kt + (kb * 32 + l32) * (DH + PAD) + kk * 16 + lhi * 8);
#pragma unroll
                for (int qq = 0; qq < QB; ++qq) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) s[qq][kb][e] = 0.f;
#pragma unroll
                    for (int kk = 0; kk < DH / 16; ++kk)
                        s[qq][kb] = SF_MFMA16(kf[kk], qf[qq][kk], s[qq][kb], 0, 0, 0);
                }
            }
        };
        // O^T += V^T . P^T of both pairs
        auto pv_tile = [&](const h16 *Vt) {
#pragma unroll
            for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    // keys {16t + lhi*4 + 0..3, 16t + 8 + lhi*4 + 0..3}: one 16-byte read in the staged key order
                    const h16x8 vf = *reinterpret_cast<const h16x8 *>(Vt + (db * 32 + l32) * (BKEY + PAD) + t * 16 + lhi * 8);
#pragma unroll
                    for (int qq = 0; qq < QB; ++qq)
                        oacc[qq][db] = SF_MFMA16(vf, pf[qq][t], oacc[qq][db], 0, 0, 0);
                }
        };
        // softmax of S(t) -> P(t); updates the running reference / sum / output scale of both pairs
        auto softmax_tile = [&](int j0) {
            const uint32_t w0 = words[j0 / 32], w1 = (j0 / 32 + 1 < nwords) ? words[j0 / 32 + 1] : 0u;
            const bool all_allowed = (uint32_t)__builtin_amdgcn_readfirstlane((int)(w0 & w1)) == 0xffffffffu;
#pragma unroll
            for (int qq = 0; qq < QB; ++qq) {
                if (!all_allowed) {
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb) {
                        const uint32_t wl = (kb ? w1 : w0) >> (lhi * 4);
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            if (!((wl >> ((e / 4) * 8 + (e % 4))) & 1u)) s[qq][kb][e] = -INFINITY;
                    }
                }
                float mt = fmaxf(fmaxf(s[qq][0][0], s[qq][0][1]), s[qq][1][0]);
                mt = fmaxf(fmaxf(mt, s[qq][1][1]), s[qq][0][2]);
#pragma unroll
                for (int e = 3; e < 15; e += 2) mt = fmaxf(fmaxf(mt, s[qq][0][e]), s[qq][0][e + 1]);
#pragma unroll
                for (int e = 2; e < 16; e += 2) mt = fmaxf(fmaxf(mt, s[qq][1][e]), s[qq][1][e + 1]);
                mt = fmaxf(mt, s[qq][0][15]) * sc;         // sc > 0: max and scaling commute
                mt = both_halves_max(mt);
                // the reference moves only when some query needs it (see attend_bf16_kernel)
                if (__builtin_expect(__builtin_amdgcn_ballot_w64(mt > m_run[qq] + RESCALE_LOG2) != 0ull, 0)) {
                    const float m_new = fmaxf(m_run[qq], mt);
                    const float alpha = __builtin_amdgcn_exp2f(m_run[qq] - (m_new == -INFINITY ? 0.f : m_new));
                    m_run[qq] = m_new;
                    l_run[qq] *= alpha;
#pragma unroll
                    for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                        for (int e = 0; e < 16; ++e) oacc[qq][db][e] *= alpha;
                }
                const float nm = m_run[qq] == -INFINITY ? 0.f : -m_run[qq];
                float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; e += 2) {
                        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[qq][kb][e], sc, nm));
                        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[qq][kb][e + 1], sc, nm));
                        rs0 += p0;
                        rs1 += p1;
                        reinterpret_cast<uint32_t *>(&pf[qq][kb * 2 + e / 8])[(e % 8) / 2] = pack2_h16(p0, p1);
                    }
                l_run[qq] += rs0 + rs1;
            }
        };

        if (nt > 0) {
            // K(0) and V(0) by group 0, K(1) by group 1; V(1) waits in group 0's registers, K(2) in group 1's
            uint4 kreg[NK], vreg[NV];
            if (grp == 0) {
                fetch_k(tile_j0(0), kreg);
                fetch_v(tile_j0(0), vreg);
                put_k(kreg, Ks);
                put_v(vreg, Vs, tile_j0(0));
                fetch_v(tile_j0(min(1, nt - 1)), vreg);
            } else {
                fetch_k(tile_j0(min(1, nt - 1)), kreg);
                put_k(kreg, Ks + KT);
                fetch_k(tile_j0(min(2, nt - 1)), kreg);
            }
            __syncthreads();
            if (!idle) s_tile(Ks);
            if (grp == 1) __syncthreads();                    // group 1 runs one cluster behind
            for (int it = 0; it < nt; ++it) {
                // The tile numbers of this iteration, read at the top of the V cluster where the vector ALU work hides
                // the LDS round trip.  Beyond the last tile the index is clamped: the staging and the S^T block of
                // the last iterations are then redundant (they land in buffers nobody reads again), which keeps the
                // M cluster free of data-dependent branches.
                const int j_cur = tile_j0(it), j1 = tile_j0(min(it + 1, nt - 1));
                const int j_far = tile_j0(min(it + 2 + grp, nt - 1));
                // ---- cluster V(it): vector ALU only
                if (!idle) softmax_tile(j_cur);
                __syncthreads();
                // ---- cluster M(it): matrix pipe, and the group's share of the staging (the buffers written here had
                // their last readers one slot ago).  (Raising this wave's priority for the cluster changed nothing.)
                if (grp == 0) {
                    put_v(vreg, Vs + ((it + 1) & 1) * VT_, j1);                     // V(it+1) over V(it-1)
                    fetch_v(j_far, vreg);                                           // V(it+2)
                } else {
                    put_k(kreg, Ks + (it & 1) * KT);                                // K(it+2) over K(it)
                    fetch_k(j_far, kreg);                                           // K(it+3)
                }
                if (!idle) {
                    pv_tile(Vs + (it & 1) * VT_);
                    s_tile(Ks + ((it + 1) & 1) * KT);
                }
                __syncthreads();
            }
            if (grp == 0) __syncthreads();                    // as many barriers as group 1
        }

        // lane owns query l32 and output dims db*32 + ig*8 + lhi*4 + {0..3}
#pragma unroll
        for (int qq = 0; qq < QB; ++qq) {
            const float l_tot = both_halves_sum(l_run[qq]);
            if (qidx[qq] < 0) continue;
            if (splits <= 1) {
                const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
                h16 *orow = O + (sample_row(row0, b, L) + qidx[qq]) * ldo + (int64_t)head[qq] * DH;
#pragma unroll
                for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                    for (int ig = 0; ig < 4; ++ig) {
                        uint2 o;
                        o.x = pack2_h16(oacc[qq][db][ig * 4] * inv, oacc[qq][db][ig * 4 + 1] * inv);
                        o.y = pack2_h16(oacc[qq][db][ig * 4 + 2] * inv, oacc[qq][db][ig * 4 + 3] * inv);
                        *reinterpret_cast<uint2 *>(orow + db * 32 + ig * 8 + lhi * 4) = o;
                    }
            } else {
                const int64_t base = (((int64_t)b * nH + head[qq]) * splits + sp) * Upad + slot[qq];   // [b, head, split, slot]
                float *po = part_o + base * DH;
#pragma unroll
                for (int db = 0; db < DH / 32; ++db)
#pragma unroll
                    for (int ig = 0; ig < 4; ++ig) {
                        f32x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = oacc[qq][db][ig * 4 + e];
                        *reinterpret_cast<f32x4 *>(po + db * 32 + ig * 8 + lhi * 4) = o;
                    }
                if (lhi == 0) {
                    part_ml[base * 2] = m_run[qq];
                    part_ml[base * 2 + 1] = l_tot;
                }
            }
        }
        __syncthreads();            // the next pass restages the tile buffers
    }
}

// ---------------------------------------------------------------- host side
template <int DH, int QBS>
static int32_t launch_score(const AttnArgs &a, const void *Kx, sf_strides skx, int Lk, const uint8_t *key_mask,
                            const float *stats, float *score, int scoreH, hipStream_t st)
{
    const size_t lds = (size_t)2 * BKEY * (DH + PAD) * 2 + DH * 4 + (size_t)ceil_div(Lk, 32) * 4 +
                       (size_t)ceil_div(Lk, BKEY) * 2 + 16;
    const int qblocks = ceil_div(a.L, NWAVE * QBS * 32);
    const int64_t items = (int64_t)qblocks * a.B * a.nH;
    if (items > (1 << 30)) return fail(SF_ERR_SHAPE, "sparse_gqa(bf16): too many work items");
    dim3 grid((unsigned)align_up(items, 8));
    ProfScope prof(SF_KERNEL_SCORE, st);
    hipLaunchKernelGGL((score_bf16_kernel<DH, QBS>), grid, dim3(NWAVE * 64), lds, st, (const h16 *)a.Q,
                       a.sq, (const h16 *)Kx, skx, a.head_group, a.hg_stride, a.pattern_id, a.key_valid,
                       key_mask, stats, a.nH, a.nG, a.L, Lk, score, scoreH, qblocks, (int)items, a.row0,
                       Kx == a.K ? a.row0 : nullptr);
    return SF_OK;
}

int32_t score_bf16(const AttnArgs &a, const void *Kx, sf_strides skx, int Lk, const uint8_t *key_mask,
                   const float *stats, float *score, int scoreH, hipStream_t st)
{
    const bool wide = a.L >= 1024;
#define SF_SCORE_ARGS a, Kx, skx, Lk, key_mask, stats, score, scoreH, st
    switch (a.dh) {
    case 32:  return wide ? launch_score<32, 4>(SF_SCORE_ARGS) : launch_score<32, 2>(SF_SCORE_ARGS);
    case 64:  return wide ? launch_score<64, 4>(SF_SCORE_ARGS) : launch_score<64, 2>(SF_SCORE_ARGS);
    case 128: return wide ? launch_score<128, 2>(SF_SCORE_ARGS) : launch_score<128, 1>(SF_SCORE_ARGS);
    }
#undef SF_SCORE_ARGS
    return fail(SF_ERR_SHAPE, "sparse_gqa(bf16): dh must be 32, 64 or 128");
}

template <int DH, int QB>
static int32_t launch_attend(const AttnArgs &a, const AttnPlan &pl, const void *vt, sf_strides svt,
                             const int32_t *sel, int selH, hipStream_t st)
{
    const size_t lds = (size_t)2 * BKEY * (DH + PAD) * 2 + (size_t)2 * DH * (BKEY + PAD) * 2 +
                       (size_t)ceil_div(a.L, 32) * 4 + (size_t)ceil_div(a.L, BKEY) * 2 + 16;
    const int nqb = pl.Upad / 32, BG = a.B * a.nG;
    // pair chunks per (sample, group) for evenly spread heads; a group with more heads takes several passes
    const int pairs = ceil_div(a.nH, a.nG) * nqb;
    // four waves where the launch has a (sample, group) problem per compute unit or more (no key splits) and at most
    // four pairs per problem (measured: C3 active pass 66 -> 49 us); with split keys the launch is short of work per
    // compute unit and eight waves with key groups are faster (C5: 40 against 45 us); dh 128 needs 232 registers
    // with four waves, i.e. one wave per SIMD
    const int nw = (QB == 1 && DH <= 64 && pairs <= 4 && pl.splits == 1) ? 4 : AWAVE;
    const int chunks = ceil_div(pairs, nw * QB);
    const int64_t items = (int64_t)chunks * BG * pl.splits;
    if (items > (1 << 30)) return fail(SF_ERR_SHAPE, "sparse_gqa(bf16): too many work items");
    dim3 grid((unsigned)align_up(items, 8));
    ProfScope prof(SF_KERNEL_ATTEND, st);
    if constexpr (QB == 2) {
        hipLaunchKernelGGL((attend_pp_bf16_kernel<DH>), grid, dim3(AWAVE * 64), lds, st, (const h16 *)a.Q,
                           a.sq, (const h16 *)a.K, a.sk, (const h16 *)vt, svt, a.head_group, a.hg_stride,
                           a.pattern_id, a.key_valid, sel, selH, a.nH, a.nG, BG, chunks, a.L, pl.Lp, a.U, pl.Upad,
                           pl.splits, pl.keys_per_split, (h16 *)a.O, a.ldo, pl.part_o, pl.part_ml, a.row0);
    } else {
#define SF_ATTEND_ARGS grid, dim3(nw * 64), lds, st, (const h16 *)a.Q, a.sq, (const h16 *)a.K, a.sk, (const h16 *)vt, \
                       svt, a.head_group, a.hg_stride, a.pattern_id, a.key_valid, sel, selH, a.nH, a.nG, BG, chunks, a.L, \
                       pl.Lp, a.U, pl.Upad, pl.splits, pl.keys_per_split, (h16 *)a.O, a.ldo, pl.part_o, pl.part_ml, a.row0
        if (nw == 4) hipLaunchKernelGGL((attend_bf16_kernel<DH, QB, DH <= 64 ? 4 : AWAVE>), SF_ATTEND_ARGS);
        else hipLaunchKernelGGL((attend_bf16_kernel<DH, QB, AWAVE>), SF_ATTEND_ARGS);
#undef SF_ATTEND_ARGS
    }
    return SF_OK;
}

int32_t attend_bf16(const AttnArgs &a, const AttnPlan &pl, const void *vt, sf_strides svt,
                    const int32_t *sel, int selH, hipStream_t st)
{
    if (a.nH > 64) return fail(SF_ERR_SHAPE, "sparse_gqa(bf16): at most 64 heads");
    const bool many = a.U >= 256;       // dense-like: two query blocks per wave
    switch (a.dh) {
    case 32:  return many ? launch_attend<32, 2>(a, pl, vt, svt, sel, selH, st) : launch_attend<32, 1>(a, pl, vt, svt, sel, selH, st);
    case 64:  return many ? launch_attend<64, 2>(a, pl, vt, svt, sel, selH, st) : launch_attend<64, 1>(a, pl, vt, svt, sel, selH, st);
    case 128: return launch_attend<128, 1>(a, pl, vt, svt, sel, selH, st);
    }
    return fail(SF_ERR_SHAPE, "sparse_gqa(bf16): dh must be 32, 64 or 128");
}

}  // namespace sf
