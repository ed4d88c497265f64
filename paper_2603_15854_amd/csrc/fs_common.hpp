// Device-side building blocks shared by the stage-1 kernels of the fused LM-head sampler:
// the noise generator, the Gumbel transform, the (value, id) candidate merge and the
// parameter block.  gfx950 (CDNA4) only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fs {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kVocabTile = 128;  // vocabulary ids per candidate (FS_VOCAB_TILE)
constexpr int kWave = 64;

// Arguments of one stage-1 launch (Alg. 1, stage 1).
struct Stage1Params {
    const uint16_t* H;        // [B, D] bf16
    const uint16_t* W;        // [V, D] bf16
    int B, D, V, T;           // T = ceil(V / kVocabTile)
    const float* tau;         // [B]
    uint64_t seed;
    const uint64_t* row_seeds;  // [B] or nullptr
    int64_t row_offset;
    int32_t vocab_offset;
    float* cand_val;          // [B, T]  (nullptr: no sampling epilogue)
    int32_t* cand_idx;        // [B, T]
    float* logits;            // [B, V] fp32 or nullptr (logits-store flag)
};

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two 32x32->64 multiplies
// whose halves are crossed with the neighbouring counter words and the round key; the key is
// bumped by the Weyl constants between rounds.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4])
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        // one 32x32->64 multiply per product (v_mad_u64_u32) instead of separate high and low halves
        const uint64_t p0 = (uint64_t)M0 * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)M1 * (uint64_t)c2;
        const uint32_t t0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t t2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c0 = t0; c1 = (uint32_t)p1; c2 = t2; c3 = (uint32_t)p0;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// 32-bit word -> Gumbel(0,1) variate in fp32 (Alg. 1: u in (0,1), g = -log(-log u)).
//   x = min(fma(float(r), 2^-32, 2^-33), 1 - 2^-24) is 1 - u; it is strictly inside (0,1) and
//   is fine-grained near 0, i.e. near u -> 1, the upper Gumbel tail that decides winners.
//   e = -log(1 - x): five-term Maclaurin series below 2^-5 (relative truncation error < 1e-8),
//   hardware log2 otherwise (1 - x is then exact or within half an ulp of 1/2..1).
//   g = -log(e) by hardware log2.
__device__ __forceinline__ float gumbel_from_word(uint32_t r)
{
    constexpr float kLn2 = 0.6931471805599453f;
    const float x = fminf(fmaf((float)r, 0x1p-32f, 0x1p-33f), 1.0f - 0x1p-24f);
    const float series =
        x * fmaf(x, fmaf(x, fmaf(x, fmaf(x, 0.2f, 0.25f), 1.0f / 3.0f), 0.5f), 1.0f);
    const float vialog = -kLn2 * __builtin_amdgcn_logf(1.0f - x);
    const float e = x < 0x1p-5f ? series : vialog;
    return -kLn2 * __builtin_amdgcn_logf(e);
}

// Gumbel noise for four consecutive vocabulary ids vid0 .. vid0+3 of one row.  One Philox block
// serves the four ids of an aligned group (counter word 0 is id >> 2, output word is id & 3);
// a misaligned start (vocabulary shard offset not a multiple of 4) straddles two blocks.
__device__ __forceinline__ void gumbel4(uint64_t seed, uint32_t row, uint32_t vid0, float g[4])
{
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t w[4];
    philox4x32_10(vid0 >> 2, row, 0u, 0u, k0, k1, w);
    const uint32_t sh = vid0 & 3u;
    if (sh == 0u) {
#pragma unroll
        for (int j = 0; j < 4; ++j) g[j] = gumbel_from_word(w[j]);
    } else {
        uint32_t w2[4];
        philox4x32_10((vid0 >> 2) + 1u, row, 0u, 0u, k0, k1, w2);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t q = sh + (uint32_t)j;  // 1..6
            const uint32_t lo = q == 1u ? w[1] : q == 2u ? w[2] : w[3];
            const uint32_t hi = q == 4u ? w2[0] : q == 5u ? w2[1] : w2[2];
            g[j] = gumbel_from_word(q < 4u ? lo : hi);
        }
    }
}

// Single id (used by the stand-alone kernels' ragged tails).
__device__ __forceinline__ float gumbel1(uint64_t seed, uint32_t row, uint32_t vid)
{
    uint32_t w[4];
    philox4x32_10(vid >> 2, row, 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), w);
    const uint32_t q = vid & 3u;
    return gumbel_from_word(q == 0u ? w[0] : q == 1u ? w[1] : q == 2u ? w[2] : w[3]);
}

// ---------------------------------------------------------------------------------------------
// Candidate = (perturbed score, vocabulary id).  "No candidate yet" is (-inf, -1).  A candidate
// replaces the current one when its score is larger, or equal with a lower id (the strict >
// of the streaming algorithm taken in ascending id order).  NaN never replaces anything.
__device__ __forceinline__ void cand_merge(float& v, int& i, float ov, int oi)
{
    const bool take = (ov > v) || (ov == v && oi < i);
    v = take ? ov : v;
    i = take ? oi : i;
}

// Reduce candidates over the four 16-lane groups of a wave (lanes l, l^16, l^32, l^48).
__device__ __forceinline__ void cand_reduce_lane_groups(float& v, int& i)
{
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const float ov = __shfl_xor(v, off, kWave);
        const int oi = __shfl_xor(i, off, kWave);
        cand_merge(v, i, ov, oi);
    }
}

__device__ __forceinline__ uint4 ld_global_16B(const uint16_t* p)
{
    return *reinterpret_cast<const uint4*>(p);
}

// 128-bit streaming load for data that is read exactly once (W): the non-temporal hint keeps
// the stream from displacing cache lines and measurably raises the sustained HBM read rate on
// MI355X (about 7.0 TB/s against 6.1 TB/s for plain loads in a pure read kernel).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_global_16B_stream(const uint16_t* p)
{
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

}  // namespace fs
