// Truncated supports (Section "Top-k, Nucleus Sampling, and Masking"): per-tile top-k candidates,
// the reduction of candidates to a global top-k, the nucleus rule on the k candidates and the draw.
//
// Order used everywhere: larger key first; equal keys: lower id first; padding is (-inf, -1) and
// sorts last (ids compare as unsigned, so -1 is the largest); NaN keys are turned into -inf when
// a key is formed.  Two kinds of key, chosen by the caller:
//   truncation    key = z = y / tau: the k candidates are the support the draw is cut to;
//   Gumbel-top-k  key = s = z + g:   the k candidates, in order, ARE the draw (k ids without
//                 replacement); the first one is the plain Gumbel-max sample.
//
// Pieces:
//   wave_sort128_desc    a wave sorts 128 (key, id) pairs held two per lane (bitonic network over
//                        lanes by shuffles): the per-tile top-k of the fused stage-1 epilogue
//   keys_from_logits     the unfused path: stored logits -> keys, in place
//   topk_select_kernel   the k best of a chunk of a row, from pairs or from a key row; run once
//                        over chunks (many workgroups per row) and once over the chunks' results
//   topk_finish_kernel   nucleus rule on the k sorted candidates + Gumbel-max over the kept ones
#pragma once

#include "fs_common.hpp"
#include "fs_topk_common.hpp"

namespace fs {

// ---------------------------------------------------------------------------------------------
// Unfused path: stored fp32 logits [B, V] -> keys, in place (z = y / tau, plus the per-id Gumbel noise
// of the main path in Gumbel-top-k mode).  Four ids per thread, one Philox block.
__global__ void __launch_bounds__(256)
keys_from_logits_kernel(float* __restrict__ logits, int V, const float* __restrict__ tau, uint64_t seed,
                        const uint64_t* __restrict__ row_seeds, int64_t row_offset, int32_t vocab_offset,
                        int mode, uint32_t epi_flags)
{
    const int b = blockIdx.y;
    const int v0 = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (v0 >= V) return;
    float* row = logits + (size_t)b * V;
    const float inv_tau = 1.0f / tau[b];
    float gn[4] = {0.f, 0.f, 0.f, 0.f};
    if (mode == kTopkGumbel)
        gumbel4(row_seeds ? row_seeds[b] : seed, (uint32_t)(uint64_t)(row_offset + b), (uint32_t)(vocab_offset + v0), gn,
                (epi_flags & kEpiExactLog) != 0u);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (v0 + j < V) row[v0 + j] = key_sanitize(fmaf(row[v0 + j], inv_tau, gn[j]));
}

// ---------------------------------------------------------------------------------------------
// The k best pairs of one chunk of one row.  grid = (chunks, B).  Input: PAIRS ? (vals, ids)[b, 0..N)
// : keys[b, 0..N) with id = id_base + position.  Output: out[(b * chunks + c) * k + j], j < k, sorted,
// padded with (-inf, -1).
//
// The workgroup keeps the best k seen so far, sorted, at the head of an LDS buffer of 2048 pairs, and
// the k-th of them as a threshold.  Elements are read 1024 at a time; those that come before the
// threshold are appended behind the head; when the buffer could overflow (or at the end) the whole
// buffer is sorted (bitonic, in LDS), the head is the new top k, and the threshold moves up.  After
// the first few blocks hardly anything passes the threshold, so a row costs little more than reading
// it; an adversarial (ascending) row sorts once per 1024 elements.  The result does not depend on
// the order in which the appends land: the sort is a total order on (key, id).
constexpr int kSelBuf = 2048;
constexpr int kSelStep = 1024;

__device__ __forceinline__ void lds_sort_desc(float* sv, int* si, int n, int tid)   // n: power of two <= kSelBuf
{
    for (int size = 2; size <= n; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = tid; t < (n >> 1); t += 256) {
                const int lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                const int hi = lo | stride;
                const bool up = (lo & size) == 0 || size == n;      // the last merge sorts the whole array descending
                const float av = sv[lo], bv = sv[hi];
                const int ai = si[lo], bi = si[hi];
                const bool a_first = pair_before(av, ai, bv, bi);
                if (a_first != up) { sv[lo] = bv; si[lo] = bi; sv[hi] = av; si[hi] = ai; }
            }
            __syncthreads();
        }
    }
}

template <bool PAIRS>
__global__ void __launch_bounds__(256)
topk_select_kernel(const float* __restrict__ vals, const int32_t* __restrict__ ids, int64_t row_stride, int N,
                   int32_t id_base, int chunk_len, int k, float* __restrict__ out_val, int32_t* __restrict__ out_idx)
{
    __shared__ float sv[kSelBuf];
    __shared__ int si[kSelBuf];
    __shared__ int s_count;
    const int tid = threadIdx.x;
    const int b = blockIdx.y, c = blockIdx.x;
    const float* rv = vals + (size_t)b * row_stride;
    const int32_t* ri = PAIRS ? ids + (size_t)b * row_stride : nullptr;
    const int begin = c * chunk_len;
    int end = begin + chunk_len;
    end = end < N ? end : N;

    for (int t = tid; t < kSelBuf; t += 256) { sv[t] = -__builtin_inff(); si[t] = -1; }
    if (tid == 0) s_count = 0;
    __syncthreads();

    auto flush = [&]() {      // sort head + pending, pad the rest again; all threads call it
        const int used = k + s_count;
        int n = 64;
        while (n < used) n <<= 1;
        lds_sort_desc(sv, si, n, tid);
        for (int t = k + tid; t < n; t += 256) { sv[t] = -__builtin_inff(); si[t] = -1; }
        if (tid == 0) s_count = 0;
        __syncthreads();
    };

    for (int base = begin; base < end; base += kSelStep) {
        if (k + s_count + kSelStep > kSelBuf) flush();      // s_count is uniform here (read after a barrier)
        const float thr_v = sv[k - 1];
        const int thr_i = si[k - 1];
#pragma unroll
        for (int u = 0; u < kSelStep / 256; ++u) {
            const int pos = base + u * 256 + tid;
            if (pos < end) {
                const float v = key_sanitize(rv[pos]);
                const int id = PAIRS ? ri[pos] : id_base + pos;
                if (pair_before(v, id, thr_v, thr_i)) {
                    const int slot = atomicAdd(&s_count, 1);
                    sv[k + slot] = v;
                    si[k + slot] = id;
                }
            }
        }
        __syncthreads();
    }
    flush();
    const size_t o = ((size_t)b * gridDim.x + c) * (size_t)k;
    for (int t = tid; t < k; t += 256) { out_val[o + t] = sv[t]; out_idx[o + t] = si[t]; }
}

// ---------------------------------------------------------------------------------------------
// Last step, one wave per row: the k sorted candidates (key, id) of the row ->
//   truncation    nucleus rule on the softmax over the candidates (keep the shortest prefix whose
//                 mass reaches top_p, at least one), then Gumbel-max over the kept ids with the
//                 per-id noise of the main path (lowest id on exact ties);
//   Gumbel-top-k  the first candidate.
// Also copies the candidates to the caller's arrays (if given) and reports how many were kept.
__global__ void __launch_bounds__(64)
topk_finish_kernel(const float* __restrict__ cand_val, const int32_t* __restrict__ cand_idx, int k, float top_p, int mode,
                   uint64_t seed, const uint64_t* __restrict__ row_seeds, int64_t row_offset, uint32_t epi_flags,
                   int32_t* __restrict__ out_idx, float* __restrict__ out_val, float* __restrict__ topk_val,
                   int32_t* __restrict__ topk_idx, int32_t* __restrict__ n_kept)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    float key = -__builtin_inff();
    int id = -1;
    if (lane < k) { key = cand_val[(size_t)b * k + lane]; id = cand_idx[(size_t)b * k + lane]; }
    if (lane < k) {
        if (topk_val) topk_val[(size_t)b * k + lane] = key;
        if (topk_idx) topk_idx[(size_t)b * k + lane] = id;
    }
    const bool live = id >= 0 && key > -__builtin_inff();
    float best = -__builtin_inff();
    int best_id = -1;
    int kept_count;
    if (mode == kTopkGumbel) {
        kept_count = (int)__builtin_popcountll(__ballot(live));
        if (lane == 0 && live) { best = key; best_id = id; }
    } else {
        const float zmax = __shfl(key, 0, kWave);
        const float e = live ? exp_diff(key, zmax) : 0.0f;
        float cum = e;                                      // inclusive prefix sum over lanes
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const float o = __shfl_up(cum, off, kWave);
            if (lane >= off) cum += o;
        }
        const float total = __shfl(cum, kWave - 1, kWave);
        // kept: everything before it has not reached top_p yet (the first live candidate always is)
        const bool kept = live && (top_p >= 1.0f || lane == 0 || (cum - e) < top_p * total);
        kept_count = (int)__builtin_popcountll(__ballot(kept));
        if (kept) {
            const uint64_t sd = row_seeds ? row_seeds[b] : seed;
            const uint32_t w = [&]() {
                uint32_t ww[4];
                philox4x32_10((uint32_t)id >> 2, (uint32_t)(uint64_t)(row_offset + b), 0u, 0u, (uint32_t)sd, (uint32_t)(sd >> 32), ww);
                const uint32_t q = (uint32_t)id & 3u;
                return q == 0u ? ww[0] : q == 1u ? ww[1] : q == 2u ? ww[2] : ww[3];
            }();
            best = key + ((epi_flags & kEpiExactLog) ? gumbel_from_word_exact(w) : gumbel_from_word(w));
            best_id = id;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(best, off, kWave);
        const int oi = __shfl_xor(best_id, off, kWave);
        const bool take = (ov > best) || (ov == best && oi >= 0 && (best_id < 0 || oi < best_id));
        best = take ? ov : best;
        best_id = take ? oi : best_id;
    }
    if (lane == 0) {
        out_idx[b] = best_id;
        out_val[b] = best;
        if (n_kept) n_kept[b] = kept_count;
    }
}

}  // namespace fs
