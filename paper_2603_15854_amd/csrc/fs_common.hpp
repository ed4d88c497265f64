// Device-side building blocks shared by the stage-1 kernels of the fused LM-head sampler:
// the noise generator, the Gumbel transform, the (value, id) candidate merge and the
// parameter block.  gfx950 (CDNA4) only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace fs {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kVocabTile = 128;  // vocabulary ids per candidate (FS_VOCAB_TILE)
constexpr int kWave = 64;

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}): a loop whose
// index is a constant expression in the body (immediate operands of inline assembly need one)
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

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
    // full transform and log-normaliser (kernels instantiated with FULL = true only)
    const float* bias;        // [V] fp32 or nullptr: z = (y + bias) / tau
    const uint32_t* allowed;  // bit rows (bit i%32 of word i/32 set = id i allowed) or nullptr
    int64_t mask_stride;      // 32-bit words per batch row of `allowed`; 0 = one row for all
    float* lse_max;           // [B, T] running maximum of z per (row, tile), or nullptr
    float* lse_sum;           // [B, T] sum of exp(z - max) per (row, tile)
    // FP8 weights (kernels instantiated for one-byte W elements only): W points at E4M3 codes
    const float* w_scale = nullptr;   // [V] fp32 per-row scale of the logits, or nullptr (= 1)
    const uint8_t* w4_scales = nullptr;   // MXFP4 (tiled kernel, W4): E8M0 block scales [V, D / 32]
    // epilogue mode bits (FS_FLAG_GREEDY, FS_FLAG_EXACT_LOG of the C ABI)
    uint32_t epi_flags = 0;
    // Truncated supports (kernels instantiated with TOPK only): the topk_k best candidates of every
    // (row, 128-id tile), sorted, packed (fs_topk_common.hpp), at topk_out[(b T + t) topk_k + j]
    uint64_t* topk_out = nullptr;
    int topk_k = 0;
    int topk_mode = 0;                // 0: key = y / tau; 1: key = y / tau + Gumbel noise
};

constexpr uint32_t kEpiGreedy = 0x1u;     // no noise: the candidate is the arg max of the transformed logits
constexpr uint32_t kEpiExactLog = 0x2u;   // Gumbel transform with the library logarithms instead of v_log_f32

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
        // a ^ b ^ c as one three-input bit operation (truth table 0x96); the compiler emits two xors
        const uint32_t t0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
        const uint32_t t2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
        c0 = t0; c1 = (uint32_t)p1; c2 = t2; c3 = (uint32_t)p0;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// 32-bit word -> Gumbel(0,1) variate in fp32 (Alg. 1: u in (0,1), g = -log(-log u)).
//   x = min(fma(float(r), 2^-32, 2^-33), 1 - 2^-24) is 1 - u; it is strictly inside (0,1) and
//   is fine-grained near 0, i.e. near u -> 1, the upper Gumbel tail that decides winners.
// Two evaluations of the logarithms (appendix "Numerically Stable and Fast Gumbel Generation":
// an exact-math and a fast-math mode):
//   fast (default)  e = -log(1 - x): five-term Maclaurin series below 2^-5 (relative truncation
//                   error < 1e-8), hardware log2 otherwise (1 - x is then exact or within half an
//                   ulp of 1/2..1); g = -log(e) by hardware log2 (v_log_f32, about 1 ulp)
//   exact           e = -log1p(-x), g = -log(e) with the device library's log1pf / logf
__device__ __forceinline__ float uniform_x_from_word(uint32_t r)
{
    return fminf(fmaf((float)r, 0x1p-32f, 0x1p-33f), 1.0f - 0x1p-24f);
}
__device__ __forceinline__ float gumbel_from_word(uint32_t r)
{
    constexpr float kLn2 = 0.6931471805599453f;
    const float x = uniform_x_from_word(r);
    const float series =
        x * fmaf(x, fmaf(x, fmaf(x, fmaf(x, 0.2f, 0.25f), 1.0f / 3.0f), 0.5f), 1.0f);
    const float vialog = -kLn2 * __builtin_amdgcn_logf(1.0f - x);
    const float e = x < 0x1p-5f ? series : vialog;
    return -kLn2 * __builtin_amdgcn_logf(e);
}
__device__ __forceinline__ float gumbel_from_word_exact(uint32_t r)
{
    return -logf(-log1pf(-uniform_x_from_word(r)));
}

// Gumbel noise for four consecutive vocabulary ids vid0 .. vid0+3 of one row.  One Philox block
// serves the four ids of an aligned group (counter word 0 is id >> 2, output word is id & 3);
// a misaligned start (vocabulary shard offset not a multiple of 4) straddles two blocks.
__device__ __forceinline__ void gumbel4(uint64_t seed, uint32_t row, uint32_t vid0, float g[4], bool exact_log = false)
{
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t w[4];
    philox4x32_10(vid0 >> 2, row, 0u, 0u, k0, k1, w);
    const uint32_t sh = vid0 & 3u;
    if (sh != 0u) {   // the four ids straddle two blocks: words sh..3 of this one, 0..sh-1 of the next
        uint32_t w2[4];
        philox4x32_10((vid0 >> 2) + 1u, row, 0u, 0u, k0, k1, w2);
        uint32_t m[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t q = sh + (uint32_t)j;  // 1..6
            const uint32_t lo = q == 1u ? w[1] : q == 2u ? w[2] : w[3];
            const uint32_t hi = q == 4u ? w2[0] : q == 5u ? w2[1] : w2[2];
            m[j] = q < 4u ? lo : hi;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = m[j];
    }
    if (exact_log) {    // uniform over the launch
#pragma unroll
        for (int j = 0; j < 4; ++j) g[j] = gumbel_from_word_exact(w[j]);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) g[j] = gumbel_from_word(w[j]);
    }
}

// gumbel4 for U quads of one row at once, all with the same vid0 % 4: the U generator chains are
// independent and the two uniform branches (straddling quads, log mode) are taken once, so a wave that
// is alone on its SIMD overlaps the chains.
template <int U>
__device__ __forceinline__ void gumbel4_multi(uint64_t seed, uint32_t row, const uint32_t (&vid0)[U], float (&g)[U][4],
                                              bool exact_log)
{
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t w[U][4];
#pragma unroll
    for (int u = 0; u < U; ++u) philox4x32_10(vid0[u] >> 2, row, 0u, 0u, k0, k1, w[u]);
    const uint32_t sh = vid0[0] & 3u;
    if (sh != 0u) {
        uint32_t w2[U][4];
#pragma unroll
        for (int u = 0; u < U; ++u) philox4x32_10((vid0[u] >> 2) + 1u, row, 0u, 0u, k0, k1, w2[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t m[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t q = sh + (uint32_t)j;  // 1..6
                const uint32_t lo = q == 1u ? w[u][1] : q == 2u ? w[u][2] : w[u][3];
                const uint32_t hi = q == 4u ? w2[u][0] : q == 5u ? w2[u][1] : w2[u][2];
                m[j] = q < 4u ? lo : hi;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) w[u][j] = m[j];
        }
    }
    if (exact_log) {    // uniform over the launch
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) g[u][j] = gumbel_from_word_exact(w[u][j]);
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) g[u][j] = gumbel_from_word(w[u][j]);
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

// ---------------------------------------------------------------------------------------------
// Online log-sum-exp state (m, s): log sum exp = m + log s.  Empty state is (-inf, 0).
__device__ __forceinline__ float exp_diff(float a, float m)   // exp(a - m), 0 when a = -inf
{
    constexpr float kLog2e = 1.4426950408889634f;
    return a == -__builtin_inff() ? 0.0f : __builtin_amdgcn_exp2f((a - m) * kLog2e);
}
__device__ __forceinline__ void lse_merge(float& m, float& s, float om, float os)
{
    const float nm = fmaxf(m, om);
    s = s * exp_diff(m, nm) + os * exp_diff(om, nm);
    m = nm;
}
__device__ __forceinline__ void lse_reduce_lane_groups(float& m, float& s)
{
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const float om = __shfl_xor(m, off, kWave);
        const float os = __shfl_xor(s, off, kWave);
        lse_merge(m, s, om, os);
    }
}

// Per-row constants of the sampling epilogue.
struct RowEpi {
    float inv_tau;
    uint64_t seed;
    uint32_t row_word;
    const uint32_t* allowed_row;   // FULL only
};

template <bool FULL>
__device__ __forceinline__ RowEpi make_row_epi(const Stage1Params& p, int b)
{
    RowEpi r;
    r.inv_tau = 1.0f / p.tau[b];
    r.seed = p.row_seeds ? p.row_seeds[b] : p.seed;
    r.row_word = (uint32_t)(uint64_t)(p.row_offset + b);
    r.allowed_row = nullptr;
    if constexpr (FULL) {
        if (p.allowed) r.allowed_row = p.allowed + (size_t)b * (size_t)p.mask_stride;
    }
    return r;
}

// Epilogue of Alg. 1 for the four consecutive vocabulary rows v0 .. v0+3 (local ids, v0 % 4 == 0)
// a lane holds for one batch row: transform, noise, perturbed score, running argmax; with FULL
// also additive bias, the allowed-id mask (-inf before perturbation) and the online
// log-sum-exp of the transformed logits.
template <bool FULL>
__device__ __forceinline__ void epilogue_quad(const Stage1Params& p, const RowEpi& r, const f32x4 y,
                                              int v0, int V, float& best, int& best_id,
                                              float& lmax, float& lsum)
{
    float gn[4] = {0.f, 0.f, 0.f, 0.f};
    if (!(p.epi_flags & kEpiGreedy))   // uniform over the launch
        gumbel4(r.seed, r.row_word, (uint32_t)(p.vocab_offset + v0), gn, (p.epi_flags & kEpiExactLog) != 0u);
    if constexpr (!FULL) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float s = fmaf(y[j], r.inv_tau, gn[j]);
            if (v0 + j < V && s > best) { best = s; best_id = p.vocab_offset + v0 + j; }
        }
    } else {
        float bq[4] = {0.f, 0.f, 0.f, 0.f};
        if (p.bias) {
            if (v0 + 3 < V) {
                const f32x4 q = *reinterpret_cast<const f32x4*>(p.bias + v0);
                bq[0] = q[0]; bq[1] = q[1]; bq[2] = q[2]; bq[3] = q[3];
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (v0 + j < V) bq[j] = p.bias[v0 + j];
            }
        }
        uint32_t bits = 0xFu;
        if (r.allowed_row) bits = r.allowed_row[v0 >> 5] >> (v0 & 31);
        float z[4];
        float zmax = -__builtin_inff();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            z[j] = (y[j] + bq[j]) * r.inv_tau;
            if (!((bits >> j) & 1u) || v0 + j >= V) z[j] = -__builtin_inff();
            zmax = fmaxf(zmax, z[j]);          // fmaxf ignores NaN
            const float s = z[j] + gn[j];
            if (s > best) { best = s; best_id = p.vocab_offset + v0 + j; }
        }
        if (p.lse_max && zmax > -__builtin_inff()) {
            float m4 = zmax, s4 = 0.0f;
#pragma unroll
            for (int j = 0; j < 4; ++j) s4 += exp_diff(z[j], m4);
            lse_merge(lmax, lsum, m4, s4);
        }
    }
}

// The plain epilogue (1/tau scaling, default log mode) for a quad that needs no checks: vid0 % 4 == 0
// and all four ids valid.  Same arithmetic as epilogue_quad<false>, without a branch, so that a
// caller can run several independent quads side by side (the ten Philox rounds are one long
// dependent chain, and a wave that is alone on its SIMD has nothing else to overlap it with).
__device__ __forceinline__ void epilogue_quad_fast(uint64_t seed, uint32_t row_word, float inv_tau, const f32x4 y,
                                                   int vid0, float& best, int& best_id)
{
    uint32_t w[4];
    philox4x32_10((uint32_t)vid0 >> 2, row_word, 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), w);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float s = fmaf(y[j], inv_tau, gumbel_from_word(w[j]));
        const bool take = s > best;
        best = take ? s : best;
        best_id = take ? vid0 + j : best_id;
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

// Eight OCP FP8 E4M3 codes (two dwords, element k in byte k) -> eight bf16 values, exactly: every
// E4M3 value is representable in bf16.  The hardware convert takes two codes per instruction.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x8 e4m3x8_to_bf16x8(uint32_t lo, uint32_t hi)
{
    const bf16x2_t a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false);
    const bf16x2_t b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true);
    const bf16x2_t c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false);
    const bf16x2_t d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true);
    uint4 v;
    v.x = __builtin_bit_cast(uint32_t, a);
    v.y = __builtin_bit_cast(uint32_t, b);
    v.z = __builtin_bit_cast(uint32_t, c);
    v.w = __builtin_bit_cast(uint32_t, d);
    return __builtin_bit_cast(bf16x8, v);
}

// Eight E2M1 codes (one dword, element k in nibble k) times 2^(e - 127) -> eight bf16 values.
__device__ __forceinline__ bf16x8 mxfp4x8_to_bf16x8(uint32_t codes, uint32_t e8m0)
{
    // 2^(e - 127) as an fp32: exponent field e (e = 0 is the denormal 2^-127)
    const uint32_t bits = e8m0 << 23;          // 0 only for e = 0; every other exponent field is above 0x00400000
    const float scale = __uint_as_float(bits > 0x00400000u ? bits : 0x00400000u);
    uint4 v;
    v.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 0));
    v.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 1));
    v.z = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 2));
    v.w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 3));
    return __builtin_bit_cast(bf16x8, v);
}


}  // namespace fs
