// The small kernels around stage 1: the stage-2 tile argmax, the stand-alone Gumbel-max over
// stored logits (second half of the unfused comparison path), the noise tap and the streaming
// probe.
#pragma once

#include "fs_common.hpp"

namespace fs {

// ---------------------------------------------------------------------------------------------
// Stage 2 of Alg. 1: t* = argmax_t m[b, t], i*_b = idx[b, t*].  One 256-thread workgroup per row.
__global__ void __launch_bounds__(256)
stage2_kernel(const float* __restrict__ cand_val, const int32_t* __restrict__ cand_idx, int T,
              int32_t* __restrict__ out_idx, float* __restrict__ out_val)
{
    __shared__ float sv[4];
    __shared__ int si[4];
    const int b = blockIdx.x;
    const float* cv = cand_val + (size_t)b * T;
    const int32_t* ci = cand_idx + (size_t)b * T;
    float best = -__builtin_inff();
    int best_id = -1;
    for (int t0 = 0; t0 < T; t0 += 4 * 256) {   // four independent loads per thread in flight
        float v[4];
        int id[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = t0 + u * 256 + (int)threadIdx.x;
            v[u] = t < T ? cv[t] : -__builtin_inff();
            id[u] = t < T ? ci[t] : -1;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) cand_merge(best, best_id, v[u], id[u]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(best, off, kWave);
        const int oi = __shfl_xor(best_id, off, kWave);
        cand_merge(best, best_id, ov, oi);
    }
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = best_id; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < 4; ++w) cand_merge(best, best_id, sv[w], si[w]);
        out_idx[b] = best_id;
        out_val[b] = best;
    }
}

// Log-normaliser finish: merges the per-tile online log-sum-exp states (max, sum) of a row into
// out_lse[b] = log sum_i exp(z_i) (appendix "Returning Log-Normalizers or Max Values").
__global__ void __launch_bounds__(256)
lse_reduce_kernel(const float* __restrict__ lse_max, const float* __restrict__ lse_sum, int T,
                  float* __restrict__ out_lse)
{
    __shared__ float sm[4];
    __shared__ float ss[4];
    const int b = blockIdx.x;
    const float* pm = lse_max + (size_t)b * T;
    const float* ps = lse_sum + (size_t)b * T;
    float m = -__builtin_inff(), s = 0.0f;
    for (int t = threadIdx.x; t < T; t += 256) lse_merge(m, s, pm[t], ps[t]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float om = __shfl_xor(m, off, kWave);
        const float os = __shfl_xor(s, off, kWave);
        lse_merge(m, s, om, os);
    }
    if ((threadIdx.x & 63) == 0) { sm[threadIdx.x >> 6] = m; ss[threadIdx.x >> 6] = s; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < 4; ++w) lse_merge(m, s, sm[w], ss[w]);
        constexpr float kLn2 = 0.6931471805599453f;
        out_lse[b] = s > 0.0f ? m + kLn2 * __builtin_amdgcn_logf(s) : -__builtin_inff();
    }
}

// ---------------------------------------------------------------------------------------------
// Streaming Gumbel-max over materialised fp32 logits (appendix Alg. "Gumbel-Max sampling
// (standalone logits)").  Workgroup (t, b) scans vocabulary ids [1024 t, 1024 t + 1024) of row b,
// four ids per thread (one Philox block), and writes one candidate.
constexpr int kLogitsChunk = 1024;

__global__ void __launch_bounds__(256)
gumbel_argmax_logits_kernel(const float* __restrict__ logits, int V, int TC,
                            const float* __restrict__ tau, uint64_t seed,
                            const uint64_t* __restrict__ row_seeds, int64_t row_offset,
                            int32_t vocab_offset, float* __restrict__ cand_val,
                            int32_t* __restrict__ cand_idx)
{
    __shared__ float sv[4];
    __shared__ int si[4];
    const int b = blockIdx.y;
    const int t = blockIdx.x;
    const float inv_tau = 1.0f / tau[b];
    const uint64_t seed_b = row_seeds ? row_seeds[b] : seed;
    const uint32_t row_word = (uint32_t)(uint64_t)(row_offset + b);
    const float* row = logits + (size_t)b * V;
    const int v0 = t * kLogitsChunk + threadIdx.x * 4;
    float best = -__builtin_inff();
    int best_id = -1;
    if (v0 < V) {
        float y[4];
        if (v0 + 3 < V && (V & 3) == 0) {
            const f32x4 q = *reinterpret_cast<const f32x4*>(row + v0);
            y[0] = q[0]; y[1] = q[1]; y[2] = q[2]; y[3] = q[3];
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) y[j] = v0 + j < V ? row[v0 + j] : 0.0f;
        }
        float gn[4];
        gumbel4(seed_b, row_word, (uint32_t)(vocab_offset + v0), gn);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float s = fmaf(y[j], inv_tau, gn[j]);
            if (v0 + j < V && s > best) { best = s; best_id = vocab_offset + v0 + j; }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(best, off, kWave);
        const int oi = __shfl_xor(best_id, off, kWave);
        cand_merge(best, best_id, ov, oi);
    }
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = best_id; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < 4; ++w) cand_merge(best, best_id, sv[w], si[w]);
        cand_val[(size_t)b * TC + t] = best;
        cand_idx[(size_t)b * TC + t] = best_id;
    }
}

// ---------------------------------------------------------------------------------------------
// Noise tap: the Gumbel variates of the stage-1 epilogue for one row, ids v0 .. v0+n-1.
__global__ void __launch_bounds__(256)
noise_kernel(uint64_t seed, uint32_t row_word, int32_t v0, int n, float* __restrict__ g_out)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k < n) g_out[k] = gumbel1(seed, row_word, (uint32_t)(v0 + k));
}

__global__ void __launch_bounds__(256)
gumbel_transform_kernel(const uint32_t* __restrict__ words, int n, float* __restrict__ g_out, uint32_t flags)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k < n) g_out[k] = (flags & kEpiExactLog) ? gumbel_from_word_exact(words[k]) : gumbel_from_word(words[k]);
}

// Decode tap: the FP8 E4M3 -> bf16 conversion of the FP8-weight kernels on caller-given codes
// (eight per thread, as in the kernels), widened to fp32.
__global__ void __launch_bounds__(256)
e4m3_decode_kernel(const uint32_t* __restrict__ codes, int n8, float* __restrict__ out)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= n8) return;
    const bf16x8 v = e4m3x8_to_bf16x8(codes[2 * k], codes[2 * k + 1]);
    const uint4 bits = __builtin_bit_cast(uint4, v);
    const uint32_t w[4] = {bits.x, bits.y, bits.z, bits.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        out[8 * k + 2 * j] = __uint_as_float(w[j] << 16);
        out[8 * k + 2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
    }
}

// ---------------------------------------------------------------------------------------------
// Streaming probe: grid-stride 128-bit reads (xor-folded so they cannot be dropped) or a copy.
__global__ void __launch_bounds__(256)
stream_probe_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16,
                    uint32_t* __restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (dst) {
        for (; i < n16; i += stride) dst[i] = src[i];
    } else {
        uint4 acc = make_uint4(0u, 0u, 0u, 0u);
        for (; i + 3 * stride < n16; i += 4 * stride) {
            const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
            acc.x ^= a.x ^ b.x ^ c.x ^ d.x; acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
            acc.z ^= a.z ^ b.z ^ c.z ^ d.z; acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
        }
        for (; i < n16; i += stride) {
            const uint4 a = src[i];
            acc.x ^= a.x; acc.y ^= a.y; acc.z ^= a.z; acc.w ^= a.w;
        }
        const uint32_t f = acc.x ^ acc.y ^ acc.z ^ acc.w;
        if (f == 0x9E3779B1u && sink) *sink = f;   // practically never true: keeps the loads alive
    }
}

}  // namespace fs
