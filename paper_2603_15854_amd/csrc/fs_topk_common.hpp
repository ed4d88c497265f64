// Order and in-wave sort shared by the kernels for truncated supports (Section "Top-k, Nucleus
// Sampling, and Masking"): larger key first; equal keys: lower id first; padding is (-inf, -1) and
// sorts last; NaN keys are turned into -inf when a key is formed.
//
// A candidate travels as one 64-bit word whose unsigned order IS that order: the high half is the
// key's bit pattern mapped monotonically to an unsigned integer (-0 folded into +0 first, so the two
// zeros tie like they do as floats), the low half is the complement of the id (lower id = larger
// word; the padding id -1 gives 0, the smallest).
#pragma once

#include "fs_common.hpp"

namespace fs {

constexpr int kTopkMax = 64;          // FS_TOPK_MAX_K
// Candidates a 128-id tile emits in the fused form: 8 where the stage-1 epilogue is hidden behind the
// W stream (B <= 32), 4 above (every round of the per-tile selection is exposed there; tiles that hold
// more winners than they emit are recomputed by the last selection level either way).
constexpr int kTopkTileM = 8, kTopkTileMLargeB = 4;
constexpr int kTopkCrowdMax = kTopkMax / kTopkTileMLargeB;   // tiles of one row that can need all their keys
constexpr int kTopkTruncate = 0, kTopkGumbel = 1;

// What the last selection level does with the k sorted candidates of a row.
struct TopkFinish {
    float top_p;
    int mode;
    uint64_t seed;
    const uint64_t* row_seeds;
    int64_t row_offset;
    uint32_t epi_flags;
    int32_t* out_idx;
    float* out_val;
    float* topk_val;      // [B, k] or null
    int32_t* topk_idx;    // [B, k] or null
    int32_t* n_kept;      // [B] or null
};

// How a key row is formed from stored logits (KEYS input): key = y / tau, plus the per-id Gumbel
// noise of the main path in Gumbel-top-k mode.
struct TopkKeys {
    const float* tau;
    uint64_t seed;
    const uint64_t* row_seeds;
    int64_t row_offset;
    int mode;
    uint32_t epi_flags;
};

// Fused path with more than kTopkTileM candidates wanted: stage 1 kept only the m best of every
// tile.  A tile whose m-th candidate is among the k winners of a row may hold more of the true top
// k; every other tile cannot (what it did not emit comes after its m-th, which already lost).  The
// last selection level finds those tiles (at most k / m per row, none for typical logits),
// recomputes their 128 keys from the row's hidden state and W (plain fp32 dot products), and
// selects again among the winners of the other tiles and those keys.
struct TopkCrowd {
    const uint64_t* cand;     // [B, T, m] stage-1 candidates; null: nothing to check
    int T, m;
    int32_t vocab_offset;
    const uint16_t* H;        // [B, D] bf16
    const uint16_t* W;        // [V, D] bf16
    int D, V;
    const float* tau;         // [B]
};

__device__ __forceinline__ float key_sanitize(float k) { return k == k ? k : -__builtin_inff(); }

// key -> unsigned integer with the same order (NaN -> -inf, -0 -> +0 first); never 0
__device__ __forceinline__ uint32_t topk_ordered(float key)
{
    key = key_sanitize(key);
    key = key == 0.0f ? 0.0f : key;
    const uint32_t b = __float_as_uint(key);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}

__device__ __forceinline__ uint64_t topk_pack(float key, int32_t id)
{
    return ((uint64_t)topk_ordered(key) << 32) | (uint64_t)(~(uint32_t)id);
}

constexpr uint64_t kTopkPad = 0x007FFFFF00000000ull;      // topk_pack(-inf, -1)

__device__ __forceinline__ float topk_key(uint64_t w)
{
    uint32_t b = (uint32_t)(w >> 32);
    b = (b & 0x80000000u) ? b ^ 0x80000000u : ~b;
    return __uint_as_float(b);
}

__device__ __forceinline__ int32_t topk_id(uint64_t w) { return (int32_t)~(uint32_t)w; }

// Sort 128 words in descending order.  Element e = 64 r + lane lives in a_r of the lane; after the
// call element e is the e-th largest, so a0 of lanes 0..k-1 is the top k (k <= 64).
__device__ __forceinline__ void wave_sort128_desc(uint64_t& a0, uint64_t& a1, int lane)
{
#pragma unroll
    for (int size = 2; size <= 128; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            if (stride == 64) {   // partner is the other word of the same lane (size = 128: descending)
                const uint64_t hi = a0 > a1 ? a0 : a1, lo = a0 > a1 ? a1 : a0;
                a0 = hi; a1 = lo;
            } else {
                // blocks of `size` elements alternate direction; bit 6 of e is r
                const bool low = (lane & stride) == 0;             // this element is the lower index of its pair
                const bool up0 = size >= 64 ? true : (lane & size) == 0;                         // r = 0
                const bool up1 = size == 128 ? true : size == 64 ? false : (lane & size) == 0;   // r = 1
                const uint64_t o0 = __shfl_xor((unsigned long long)a0, stride, kWave);
                const uint64_t o1 = __shfl_xor((unsigned long long)a1, stride, kWave);
                a0 = ((a0 > o0) == (low == up0)) ? a0 : o0;      // all words differ unless both are padding
                a1 = ((a1 > o1) == (low == up1)) ? a1 : o1;
            }
        }
    }
}

// Sort 64 words (one per lane) in descending order: lane j ends with the j-th largest.
__device__ __forceinline__ void wave_sort64_desc(uint64_t& a, int lane)
{
#pragma unroll
    for (int size = 2; size <= 64; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            const bool low = (lane & stride) == 0;
            const bool up = size == 64 ? true : (lane & size) == 0;
            const uint64_t o = __shfl_xor((unsigned long long)a, stride, kWave);
            a = ((a > o) == (low == up)) ? a : o;
        }
    }
}

// Maximum of an unsigned word over the wave, for four independent words at once.  Six steps through
// the data-parallel lane permutes of the vector ALU (no LDS traffic): quads, half rows, rows of 16,
// then the row 0 -> 1 and 2 -> 3 and the rows 0..1 -> 2..3 broadcasts, after which lane 63 holds the
// maximum.  Written as one assembly block because the compiler does not fold the permute into the
// max (three instructions per step instead of one).  A permuting instruction must not read a
// register in the two issue slots after a vector instruction wrote it: the four chains are
// interleaved, so the three instructions of the other chains fill those slots, and a two-slot nop
// separates the block from whatever wrote the inputs.
__device__ __forceinline__ void wave_max4(uint32_t& a, uint32_t& b, uint32_t& c, uint32_t& d)
{
#define FS_DPP_MAX4(ctrl)                                   \
    "v_max_u32_dpp %0, %0, %0 " ctrl "\n\t"                 \
    "v_max_u32_dpp %1, %1, %1 " ctrl "\n\t"                 \
    "v_max_u32_dpp %2, %2, %2 " ctrl "\n\t"                 \
    "v_max_u32_dpp %3, %3, %3 " ctrl "\n\t"
    asm volatile("s_nop 1\n\t"
                 FS_DPP_MAX4("quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")
                 FS_DPP_MAX4("quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf")
                 FS_DPP_MAX4("row_half_mirror row_mask:0xf bank_mask:0xf")
                 FS_DPP_MAX4("row_mirror row_mask:0xf bank_mask:0xf")
                 FS_DPP_MAX4("row_bcast:15 row_mask:0xa bank_mask:0xf")
                 FS_DPP_MAX4("row_bcast:31 row_mask:0xc bank_mask:0xf")
                 "s_nop 1"
                 : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
#undef FS_DPP_MAX4
    a = (uint32_t)__builtin_amdgcn_readlane((int)a, 63);
    b = (uint32_t)__builtin_amdgcn_readlane((int)b, 63);
    c = (uint32_t)__builtin_amdgcn_readlane((int)c, 63);
    d = (uint32_t)__builtin_amdgcn_readlane((int)d, 63);
}

// The m best of the 128 keys of each of U tiles at once (m <= 64 and small).  Unit u: k0[u] is the
// ordered key (topk_ordered) of id id0[u] + lane, k1[u] of id0[u] + 64 + lane, 0 where the id does not
// exist.  m rounds of (wave maximum, lowest id that attains it, strike it); the U chains are
// independent, which is what hides the latency of a round.  Lane j < m gets the j-th best of unit u
// in res[u], packed; padding where the tile has fewer.
template <int U>
__device__ __forceinline__ void wave_top_m(uint32_t (&k0)[U], uint32_t (&k1)[U], const int32_t (&id0)[U], int m, int lane,
                                           uint64_t (&res)[U])
{
    static_assert(U == 4, "four chains fill each other's permute wait slots");
#pragma unroll
    for (int u = 0; u < U; ++u) res[u] = kTopkPad;
    for (int j = 0; j < m; ++j) {
        uint32_t mxs[U];
#pragma unroll
        for (int u = 0; u < U; ++u) mxs[u] = k0[u] > k1[u] ? k0[u] : k1[u];
        wave_max4(mxs[0], mxs[1], mxs[2], mxs[3]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t mx = mxs[u];
            const uint64_t b0 = __ballot(k0[u] == mx), b1 = __ballot(k1[u] == mx);
            const bool any = mx != 0u;                       // wave-uniform: something is left
            const bool first = b0 != 0ull;
            const int win = __builtin_ctzll(first ? b0 : b1);
            if (any && lane == j) res[u] = ((uint64_t)mx << 32) | (uint64_t)(~(uint32_t)(id0[u] + win + (first ? 0 : 64)));
            if (any && lane == win) {
                if (first) k0[u] = 0u; else k1[u] = 0u;
            }
        }
    }
}

// A lane's sorted list of its M best (ordered key, payload) pairs, best first; ka = 0 marks an empty
// place.  Inserts (x, e) behind every entry with a key >= x: among equal keys the pair inserted first
// stays ahead, so a caller that inserts in ascending id order keeps the lowest ids.
template <int M>
__device__ __forceinline__ void top_insert(uint32_t (&ka)[M], int32_t (&ke)[M], uint32_t x, int32_t e)
{
    bool c[M];
#pragma unroll
    for (int s = 0; s < M; ++s) c[s] = x > ka[s];
#pragma unroll
    for (int s = M - 1; s > 0; --s) {
        ka[s] = c[s - 1] ? ka[s - 1] : c[s] ? x : ka[s];
        ke[s] = c[s - 1] ? ke[s - 1] : c[s] ? e : ke[s];
    }
    ka[0] = c[0] ? x : ka[0];
    ke[0] = c[0] ? e : ke[0];
}

// w and o: two lists of M packed words, w in descending and o in ASCENDING order.  Afterwards w holds
// the M largest of the 2 M words in descending order: the elementwise maximum is the upper half of the
// union as a bitonic sequence, which log2(M) rounds of compare-exchange sort.
template <int M>
__device__ __forceinline__ void top_merge_lists(uint64_t (&w)[M], const uint64_t (&o)[M])
{
#pragma unroll
    for (int s = 0; s < M; ++s) w[s] = w[s] > o[s] ? w[s] : o[s];
#pragma unroll
    for (int d = M / 2; d > 0; d >>= 1)
#pragma unroll
        for (int s = 0; s < M; ++s)
            if ((s & d) == 0) {
                const uint64_t hi = w[s] > w[s + d] ? w[s] : w[s + d], lo = w[s] > w[s + d] ? w[s + d] : w[s];
                w[s] = hi;
                w[s + d] = lo;
            }
}

// w: this lane's M packed words in descending order.  Afterwards both this lane and the lane `step`
// away (lane ^ step) hold the M largest of their 2 M words, in descending order.  Packed words of
// different ids differ, so both lanes agree.
template <int M>
__device__ __forceinline__ void top_merge(uint64_t (&w)[M], int step)
{
    uint64_t o[M];
#pragma unroll
    for (int s = 0; s < M; ++s) o[s] = __shfl_xor((unsigned long long)w[M - 1 - s], step, kWave);
    top_merge_lists<M>(w, o);
}

}  // namespace fs
