// Group choice of the grouped variants (Section "Group-Gumbel-Max: Hierarchical Exact Sampling";
// appendix algorithms "FlashSampling (parallel)" and "FlashSampling (sequential/online)").
//
// Stage 1 (full-transform epilogue) leaves, per row and 128-id vocabulary tile, the tile's best
// perturbed candidate and its online log-sum-exp state.  A group is `gt` consecutive tiles.  Its
// local sample z_k is the best candidate of its tiles (a Gumbel-max sample restricted to the
// group) and its log-mass L_k is the merge of the tiles' log-sum-exp states.  The kernels here
// pick the group with noise that is independent of the per-id noise:
//   parallel : k* = argmax_k (L_k + Gumbel(ubar_k))
//   online   : running (ell, z) over ascending k; group k replaces z when u_k < exp(L_k - ell_new)
// and return z_{k*} and ell_Z = lse(L).  Both are exact in distribution (Lemma "Exact group
// factorization", Lemma "binary merge"); neither is pathwise equal to the default path.
//
// Noise: word (k & 3) of Philox4x32-10(counter = (k >> 2, row, stream, 0)), k the global group id,
// stream 1 for the outer Gumbels, stream 2 for the online uniforms (stream 0 is the per-id noise).
#pragma once

#include "fs_common.hpp"

namespace fs {

constexpr uint32_t kStreamOuterGumbel = 1u;
constexpr uint32_t kStreamOnlineUniform = 2u;

__device__ __forceinline__ uint32_t group_word(uint64_t seed, uint32_t row, uint32_t gid, uint32_t stream)
{
    uint32_t w[4];
    philox4x32_10(gid >> 2, row, stream, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), w);
    const uint32_t q = gid & 3u;
    return q == 0u ? w[0] : q == 1u ? w[1] : q == 2u ? w[2] : w[3];
}

// The open-interval uniform of the Gumbel transform, used directly by the online accept test.
__device__ __forceinline__ float uniform_from_word(uint32_t r)
{
    return fminf(fmaf((float)r, 0x1p-32f, 0x1p-33f), 1.0f - 0x1p-24f);
}

// Per-tile inputs of one row.  cand_val / lse_sum may be null when every "tile" already is a
// whole group given as (sample id, log-mass): then the id alone says whether the group has mass.
struct GroupInputs {
    const float* cand_val;
    const int32_t* cand_idx;
    const float* lse_max;
    const float* lse_sum;
    int T;    // tiles per row
    int gt;   // tiles per group
};

// Group k of a row: local sample (cv, ci) and log-sum-exp state (lm, ls).
__device__ __forceinline__ void load_group(const GroupInputs& in, size_t row_base, int k, float& cv,
                                           int& ci, float& lm, float& ls)
{
    cv = -__builtin_inff(); ci = -1; lm = -__builtin_inff(); ls = 0.0f;
    const int t0 = k * in.gt;
    const int t1 = t0 + in.gt < in.T ? t0 + in.gt : in.T;
    for (int t = t0; t < t1; ++t) {
        const int id = in.cand_idx[row_base + t];
        const float v = in.cand_val ? in.cand_val[row_base + t] : (id >= 0 ? 0.0f : -__builtin_inff());
        cand_merge(cv, ci, v, id);
        const float m = in.lse_max[row_base + t];
        const float s = in.lse_sum ? in.lse_sum[row_base + t] : (m > -__builtin_inff() ? 1.0f : 0.0f);
        lse_merge(lm, ls, m, s);
    }
}

__device__ __forceinline__ float log_mass(float lm, float ls)
{
    constexpr float kLn2 = 0.6931471805599453f;
    return ls > 0.0f ? lm + kLn2 * __builtin_amdgcn_logf(ls) : -__builtin_inff();
}

// One 256-thread workgroup per row.  MODE 0 = parallel, 1 = online.  m groups per row;
// group_log_mass / group_sample ([B, m], optional) receive L_k and z_k.
template <int MODE>
__global__ void __launch_bounds__(256)
group_choose_kernel(GroupInputs in, int m, uint64_t seed, const uint64_t* __restrict__ row_seeds,
                    int64_t row_offset, uint32_t group_offset, int32_t* __restrict__ out_idx,
                    float* __restrict__ out_lse, float* __restrict__ group_log_mass,
                    int32_t* __restrict__ group_sample)
{
    __shared__ float sh_a[256];
    __shared__ float sh_b[256];
    __shared__ int sh_i[4];
    __shared__ int sh_j[4];
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const size_t row_base = (size_t)b * in.T;
    const size_t out_base = (size_t)b * m;
    const uint64_t seed_b = row_seeds ? row_seeds[b] : seed;
    const uint32_t row_word = (uint32_t)(uint64_t)(row_offset + b);

    if constexpr (MODE == 0) {
        float best = -__builtin_inff();
        int best_id = -1;
        float tm = -__builtin_inff(), ts = 0.0f;
        for (int k = tid; k < m; k += 256) {
            float cv, lm, ls;
            int ci;
            load_group(in, row_base, k, cv, ci, lm, ls);
            const float L = log_mass(lm, ls);
            if (group_log_mass) group_log_mass[out_base + k] = L;
            if (group_sample) group_sample[out_base + k] = ci;
            // zero-mass groups are skipped; ties go to the lower group (= the lower vocabulary id)
            const float s = ls > 0.0f
                ? L + gumbel_from_word(group_word(seed_b, row_word, group_offset + (uint32_t)k, kStreamOuterGumbel))
                : -__builtin_inff();
            cand_merge(best, best_id, s, ls > 0.0f ? ci : -1);
            lse_merge(tm, ts, lm, ls);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(best, off, kWave);
            const int oi = __shfl_xor(best_id, off, kWave);
            cand_merge(best, best_id, ov, oi);
            const float om = __shfl_xor(tm, off, kWave);
            const float os = __shfl_xor(ts, off, kWave);
            lse_merge(tm, ts, om, os);
        }
        if ((tid & 63) == 0) {
            sh_a[tid >> 6] = best; sh_i[tid >> 6] = best_id;
            sh_a[4 + (tid >> 6)] = tm; sh_b[tid >> 6] = ts;
        }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int w = 1; w < 4; ++w) {
                cand_merge(best, best_id, sh_a[w], sh_i[w]);
                lse_merge(tm, ts, sh_a[4 + w], sh_b[w]);
            }
            out_idx[b] = best_id;
            if (out_lse) out_lse[b] = log_mass(tm, ts);
        }
    } else {
        // Each thread owns a contiguous run of groups, so that "ascending k" is thread order.
        const int per = (m + 255) / 256;
        const int k0 = tid * per < m ? tid * per : m;
        const int k1 = k0 + per < m ? k0 + per : m;
        float am = -__builtin_inff(), as = 0.0f;
        for (int k = k0; k < k1; ++k) {
            float cv, lm, ls;
            int ci;
            load_group(in, row_base, k, cv, ci, lm, ls);
            if (group_log_mass) group_log_mass[out_base + k] = log_mass(lm, ls);
            if (group_sample) group_sample[out_base + k] = ci;
            lse_merge(am, as, lm, ls);
        }
        sh_a[tid] = am;
        sh_b[tid] = as;
        __syncthreads();
        // running log-mass of everything before this thread's first group, in ascending order
        float rm = -__builtin_inff(), rs = 0.0f;
        for (int t = 0; t < tid; ++t) lse_merge(rm, rs, sh_a[t], sh_b[t]);
        int acc_k = -1, acc_id = -1;
        for (int k = k0; k < k1; ++k) {
            float cv, lm, ls;
            int ci;
            load_group(in, row_base, k, cv, ci, lm, ls);
            if (ls > 0.0f) {
                float nm = rm, ns = rs;
                lse_merge(nm, ns, lm, ls);
                // exp(L_k - ell_new) without a logarithm; exactly 1 for the first group with mass
                const float p_replace = ls * exp_diff(lm, nm) / ns;
                const float u = uniform_from_word(
                    group_word(seed_b, row_word, group_offset + (uint32_t)k, kStreamOnlineUniform));
                if (u < p_replace) { acc_k = k; acc_id = ci; }
                rm = nm; rs = ns;
            }
        }
        // the last accepted group wins
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const int ok = __shfl_xor(acc_k, off, kWave);
            const int oi = __shfl_xor(acc_id, off, kWave);
            if (ok > acc_k) { acc_k = ok; acc_id = oi; }
        }
        __syncthreads();   // everyone is done reading the per-thread totals
        if ((tid & 63) == 0) { sh_i[tid >> 6] = acc_k; sh_j[tid >> 6] = acc_id; }
        if (tid == 255) { sh_a[0] = rm; sh_b[0] = rs; }   // the last thread holds the total
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int w = 1; w < 4; ++w)
                if (sh_i[w] > acc_k) { acc_k = sh_i[w]; acc_id = sh_j[w]; }
            out_idx[b] = acc_id;
            if (out_lse) out_lse[b] = log_mass(sh_a[0], sh_b[0]);
        }
    }
}

}  // namespace fs
