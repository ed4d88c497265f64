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
constexpr int kTopkTileM = 8;         // candidates a 128-id tile emits in the fused first pass
constexpr int kTopkFixMax = kTopkMax / kTopkTileM;   // tiles of one row that can need all their candidates
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

// Fused path with more than kTopkTileM candidates wanted: the first pass kept only the m best of
// every tile.  A tile whose m-th candidate is among the k winners of a row may hold more of the true
// top k; every other tile cannot (what it did not emit comes after its m-th, which already lost).
// The last selection level finds those tiles (at most k / m per row), lists them for the second
// stage-1 pass, and prepares the row's second selection: rowbuf[b] = k winners (those of listed
// tiles blanked) followed by kTopkFixMax runs of k words, blank until the second pass fills them.
struct TopkFix {
    const uint64_t* cand;     // [B, T, m] first-pass candidates; null: nothing to check
    int T, m;
    int32_t vocab_offset;
    int32_t* tile_flag;       // [T]
    int32_t* n_fix;           // [B]
    int32_t* fix_tiles;       // [B, kTopkFixMax]
    uint64_t* rowbuf;         // [B, rowbuf_stride]
    int rowbuf_stride;
    const int32_t* row_gate;  // second selection: rows with row_gate[b] == 0 leave at once; null: all rows run
};

__device__ __forceinline__ float key_sanitize(float k) { return k == k ? k : -__builtin_inff(); }

__device__ __forceinline__ uint64_t topk_pack(float key, int32_t id)
{
    key = key_sanitize(key);
    key = key == 0.0f ? 0.0f : key;
    uint32_t b = __float_as_uint(key);
    b ^= (uint32_t)((int32_t)b >> 31) | 0x80000000u;
    return ((uint64_t)b << 32) | (uint64_t)(~(uint32_t)id);
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

// Maximum of a float over the wave, in every lane.  Six steps through the data-parallel lane
// permutes of the vector ALU (no LDS traffic): quads, half rows, rows of 16, then row 0 -> 1 and
// 2 -> 3 and rows 0..1 -> 2..3 broadcasts, after which lane 63 holds the maximum.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_max_step(float x)
{
    const int y = __builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, ROW_MASK, 0xF, false);
    return fmaxf(x, __int_as_float(y));
}

__device__ __forceinline__ float wave_max(float x)
{
    x = dpp_max_step<0xB1, 0xF>(x);      // quad_perm [1,0,3,2]
    x = dpp_max_step<0x4E, 0xF>(x);      // quad_perm [2,3,0,1]
    x = dpp_max_step<0x141, 0xF>(x);     // row_half_mirror
    x = dpp_max_step<0x140, 0xF>(x);     // row_mirror
    x = dpp_max_step<0x142, 0xA>(x);     // row_bcast15 into rows 1 and 3
    x = dpp_max_step<0x143, 0xC>(x);     // row_bcast31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// The m best of the 128 keys of a tile, m <= 64 and small: key v0 belongs to id id0 + lane, v1 to
// id0 + 64 + lane; live0 / live1 say which of them exist.  m rounds of (wave maximum, lowest id that
// attains it, strike it).  Lane j < m returns the j-th best, packed; padding where the tile has fewer.
__device__ __forceinline__ uint64_t wave_top_m(float v0, float v1, bool live0, bool live1, int32_t id0, int m, int lane)
{
    const float ninf = -__builtin_inff();
    v0 = live0 ? key_sanitize(v0) : ninf;
    v1 = live1 ? key_sanitize(v1) : ninf;
    uint64_t res = kTopkPad;
    for (int j = 0; j < m; ++j) {
        const float mx = wave_max(fmaxf(v0, v1));
        const uint64_t b0 = __ballot(live0 && v0 == mx), b1 = __ballot(live1 && v1 == mx);
        if ((b0 | b1) == 0ull) break;                    // nothing left (wave-uniform)
        const bool first = b0 != 0ull;
        const int win = __builtin_ctzll(first ? b0 : b1);
        if (lane == j) res = topk_pack(mx, id0 + win + (first ? 0 : 64));
        if (lane == win) {
            if (first) { live0 = false; v0 = ninf; } else { live1 = false; v1 = ninf; }
        }
    }
    return res;
}

}  // namespace fs
