// Order and in-wave sort shared by the kernels for truncated supports (Section "Top-k, Nucleus
// Sampling, and Masking"): larger key first; equal keys: lower id first; padding is (-inf, -1) and
// sorts last (ids compare as unsigned, so -1 is the largest); NaN keys are turned into -inf when a
// key is formed.
#pragma once

#include "fs_common.hpp"

namespace fs {

constexpr int kTopkMax = 64;          // FS_TOPK_MAX_K
constexpr int kTopkTruncate = 0, kTopkGumbel = 1;

// (av, ai) comes before (bv, bi) in the order above
__device__ __forceinline__ bool pair_before(float av, int ai, float bv, int bi)
{
    return av > bv || (av == bv && (uint32_t)ai < (uint32_t)bi);
}

__device__ __forceinline__ float key_sanitize(float k) { return k == k ? k : -__builtin_inff(); }

// Sort 128 pairs in descending order.  Element e = 64 r + lane lives in register pair r of the lane;
// after the call element e is the e-th best, so register pair 0 of lanes 0..k-1 is the top k (k <= 64).
__device__ __forceinline__ void wave_sort128_desc(float& v0, int& i0, float& v1, int& i1, int lane)
{
#pragma unroll
    for (int size = 2; size <= 128; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            if (stride == 64) {   // partner is the other register pair of the same lane (size = 128: descending)
                const bool swap = pair_before(v1, i1, v0, i0);
                const float tv = v0; const int ti = i0;
                v0 = swap ? v1 : v0; i0 = swap ? i1 : i0;
                v1 = swap ? tv : v1; i1 = swap ? ti : i1;
            } else {
                // blocks of `size` elements alternate direction; bit 6 of e is r
                const bool low = (lane & stride) == 0;             // this element is the lower index of its pair
                const bool up0 = size == 128 ? true : size == 64 ? true : (lane & size) == 0;    // r = 0
                const bool up1 = size == 128 ? true : size == 64 ? false : (lane & size) == 0;   // r = 1
                {
                    const float ov = __shfl_xor(v0, stride, kWave);
                    const int oi = __shfl_xor(i0, stride, kWave);
                    const bool mine_first = pair_before(v0, i0, ov, oi);
                    const bool keep_better = low == up0;
                    const bool keep_mine = mine_first == keep_better;
                    v0 = keep_mine ? v0 : ov; i0 = keep_mine ? i0 : oi;
                }
                {
                    const float ov = __shfl_xor(v1, stride, kWave);
                    const int oi = __shfl_xor(i1, stride, kWave);
                    const bool mine_first = pair_before(v1, i1, ov, oi);
                    const bool keep_better = low == up1;
                    const bool keep_mine = mine_first == keep_better;
                    v1 = keep_mine ? v1 : ov; i1 = keep_mine ? i1 : oi;
                }
            }
        }
    }
}

}  // namespace fs
