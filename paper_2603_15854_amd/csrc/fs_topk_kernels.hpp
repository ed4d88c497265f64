// Truncated supports (Section "Top-k, Nucleus Sampling, and Masking"): the reduction of candidates to
// a global top-k, the nucleus rule on the k candidates and the draw.
//
// Two kinds of key, chosen by the caller:
//   truncation    key = z = y / tau: the k candidates are the support the draw is cut to;
//   Gumbel-top-k  key = s = z + g:   the k candidates, in order, ARE the draw (k ids without
//                 replacement); the first one is the plain Gumbel-max sample.
//
// Pieces:
//   topk_select_kernel   the k best of a chunk of a row, from a key row or from packed candidates;
//                        run over chunks (many workgroups per row), then over the chunks' results;
//                        the last level also applies the nucleus rule and draws (topk_finish)
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
// One wave, lane j holds the j-th candidate of row b (padding beyond k):
//   truncation    nucleus rule on the softmax over the candidates (keep the shortest prefix whose
//                 mass reaches top_p, at least one), then Gumbel-max over the kept ids with the
//                 per-id noise of the main path (lowest id on exact ties);
//   Gumbel-top-k  the first candidate.
// Also copies the candidates to the caller's arrays (if given) and reports how many were kept.
__device__ __forceinline__ void topk_finish(const TopkFinish& f, int b, int k, int lane, float key, int32_t id)
{
    if (lane < k) {
        if (f.topk_val) f.topk_val[(size_t)b * k + lane] = key;
        if (f.topk_idx) f.topk_idx[(size_t)b * k + lane] = id;
    }
    const bool live = id >= 0 && key > -__builtin_inff();
    float best = -__builtin_inff();
    int best_id = -1;
    int kept_count;
    if (f.mode == kTopkGumbel) {
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
        const bool kept = live && (f.top_p >= 1.0f || lane == 0 || (cum - e) < f.top_p * total);
        kept_count = (int)__builtin_popcountll(__ballot(kept));
        if (kept) {
            const uint64_t sd = f.row_seeds ? f.row_seeds[b] : f.seed;
            uint32_t ww[4];
            philox4x32_10((uint32_t)id >> 2, (uint32_t)(uint64_t)(f.row_offset + b), 0u, 0u, (uint32_t)sd, (uint32_t)(sd >> 32), ww);
            const uint32_t q = (uint32_t)id & 3u;
            const uint32_t w = q == 0u ? ww[0] : q == 1u ? ww[1] : q == 2u ? ww[2] : ww[3];
            best = key + ((f.epi_flags & kEpiExactLog) ? gumbel_from_word_exact(w) : gumbel_from_word(w));
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
        f.out_idx[b] = best_id;
        f.out_val[b] = best;
        if (f.n_kept) f.n_kept[b] = kept_count;
    }
}

// ---------------------------------------------------------------------------------------------
// ---------------------------------------------------------------------------------------------
// The k best candidates of one chunk of one row.  grid = (chunks, B), 256 threads.
//   KEYS   input is a row of stored fp32 logits, id = id_base + position, key formed on the fly;
//          otherwise packed candidates
//   FINAL  one chunk per row: nucleus rule and draw follow (topk_finish); otherwise the k words go
//          to out[(b * chunks + c) * k + j], sorted, padded
//   CROWD  (with FINAL, fused path, k > kTopkTileM) before the draw, look for tiles that hold more
//          winners than stage 1 emitted (TopkCrowd), recompute their keys and select again
//
// Every thread holds kSelE candidates of the chunk in registers.  The k-th largest of the 256
// per-thread maxima is a lower bound of the chunk's k-th largest candidate (k threads hold one at
// least as large), and only the threads that own those k maxima can hold anything at or above it:
// at most k * kSelE candidates pass, whatever the data (typically little more than k).  They go to a
// list in LDS, which one wave sorts in registers when it has at most 128 entries and the workgroup
// sorts in LDS otherwise.  The result does not depend on the order in which the list is filled: the
// order on words is total.  The k-th largest maximum: every wave sorts its 64 maxima, then each
// thread ranks its own among the other three runs by binary search.
constexpr int kSelE = 32;
constexpr int kSelChunk = 256 * kSelE;          // candidates one workgroup can take
constexpr int kSelList = kTopkMax * kSelE;      // bound of the list

__device__ __forceinline__ void lds_sort_desc(uint64_t* s, int n, int tid)   // n: power of two
{
    for (int size = 2; size <= n; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = tid; t < (n >> 1); t += 256) {
                const int lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                const int hi = lo | stride;
                const bool up = (lo & size) == 0 || size == n;      // the last merge sorts the whole array descending
                const uint64_t a = s[lo], c = s[hi];
                if ((a > c) != up) { s[lo] = c; s[hi] = a; }
            }
            __syncthreads();
        }
    }
}

template <bool KEYS, bool FINAL, bool CROWD = false>
__global__ void __launch_bounds__(256)
topk_select_kernel(const void* __restrict__ in, int64_t row_stride, int N, int32_t id_base, int chunk_len, int k,
                   uint64_t* __restrict__ out, TopkKeys kp, TopkFinish fin, TopkCrowd crowd)
{
    // CROWD: room for 64 winners + kTopkCrowdMax whole tiles, padded to a power of two for the sort
    __shared__ uint64_t s_list[CROWD ? 4096 : kSelList];
    __shared__ uint64_t s_max[256];
    __shared__ uint64_t s_thr;
    __shared__ int s_count;
    __shared__ int s_ncrowd;
    __shared__ int s_crowd_tile[kTopkCrowdMax];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.y, c = blockIdx.x;
    const int begin = c * chunk_len;
    int end = begin + chunk_len;
    end = end < N ? end : N;

    uint64_t it[kSelE];
    uint64_t m = kTopkPad;
    if constexpr (KEYS) {
        // four consecutive ids per thread and load: one Philox block serves them
        const float* row = static_cast<const float*>(in) + (size_t)b * row_stride;
        const float inv_tau = 1.0f / kp.tau[b];
        const uint64_t sd = kp.row_seeds ? kp.row_seeds[b] : kp.seed;
        const bool vec = (((uint64_t)row_stride | (uint64_t)begin) & 3u) == 0u && ((uintptr_t)in & 15u) == 0u;
#pragma unroll
        for (int j = 0; j < kSelE / 4; ++j) {
            const int p4 = begin + (j * 256 + tid) * 4;
            float y[4] = {0.f, 0.f, 0.f, 0.f};
            if (p4 + 3 < end && vec) {
                const f32x4 q = *reinterpret_cast<const f32x4*>(row + p4);
                y[0] = q[0]; y[1] = q[1]; y[2] = q[2]; y[3] = q[3];
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (p4 + q < end) y[q] = row[p4 + q];
            }
            float gn[4] = {0.f, 0.f, 0.f, 0.f};
            if (kp.mode == kTopkGumbel && p4 < end)
                gumbel4(sd, (uint32_t)(uint64_t)(kp.row_offset + b), (uint32_t)(id_base + p4), gn,
                        (kp.epi_flags & kEpiExactLog) != 0u);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint64_t w = p4 + q < end ? topk_pack(fmaf(y[q], inv_tau, gn[q]), id_base + p4 + q) : kTopkPad;
                it[4 * j + q] = w;
                m = w > m ? w : m;
            }
        }
    } else {
        // candidate j of the thread: position 256 j + ((tid + 37 j) mod 256) of the chunk -- coalesced, and
        // the rotation keeps a thread from collecting the same rank of many sorted runs
        const uint64_t* words = static_cast<const uint64_t*>(in) + (size_t)b * row_stride;
#pragma unroll
        for (int j = 0; j < kSelE; ++j) {
            const int pos = begin + j * 256 + ((tid + 37 * j) & 255);
            it[j] = pos < end ? words[pos] : kTopkPad;
            m = it[j] > m ? it[j] : m;
        }
    }
    wave_sort64_desc(m, lane);
    s_max[tid] = m;                              // four descending runs of 64
    if (tid == 0) s_count = 0;
    __syncthreads();
    int rank = lane;                             // position of m among the 256 maxima (ties: lower wave first)
    {
        // the three other runs are searched side by side: their LDS reads are independent chains
        int cnt[3] = {0, 0, 0};
        auto before = [&](int r, uint64_t o) {
            const int w2 = r + (r >= wave ? 1 : 0);
            return o > m || (o == m && w2 < wave);
        };
        auto run = [&](int r) { return s_max + (r + (r >= wave ? 1 : 0)) * 64; };
#pragma unroll
        for (int step = 32; step >= 1; step >>= 1) {
            uint64_t o[3];
#pragma unroll
            for (int r = 0; r < 3; ++r) o[r] = run(r)[cnt[r] + step - 1];
#pragma unroll
            for (int r = 0; r < 3; ++r)
                if (before(r, o[r])) cnt[r] += step;
        }
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            if (cnt[r] == 63 && before(r, run(r)[63])) cnt[r] = 64;
            rank += cnt[r];
        }
    }
    if (rank == k - 1) s_thr = m;
    __syncthreads();
    const uint64_t thr = s_thr;
#pragma unroll
    for (int j = 0; j < kSelE; ++j) {
        if (it[j] >= thr && (uint32_t)it[j] != 0u) {      // low half 0: padding
            const int slot = atomicAdd(&s_count, 1);
            s_list[slot] = it[j];
        }
    }
    __syncthreads();
    const int n = s_count;
    if (n <= 64) {                               // the usual case: little more than k passers
        if (tid < kWave) {
            uint64_t a0 = tid < n ? s_list[tid] : kTopkPad;
            wave_sort64_desc(a0, tid);
            s_list[tid] = a0;
        }
    } else if (n <= 128) {
        if (tid < kWave) {
            uint64_t a0 = tid < n ? s_list[tid] : kTopkPad;
            uint64_t a1 = tid + 64 < n ? s_list[tid + 64] : kTopkPad;
            wave_sort128_desc(a0, a1, tid);
            s_list[tid] = a0;
        }
    } else {
        int n2 = 256;
        while (n2 < n) n2 <<= 1;
        for (int t = n + tid; t < n2; t += 256) s_list[t] = kTopkPad;
        __syncthreads();
        lds_sort_desc(s_list, n2, tid);
    }
    __syncthreads();
    if constexpr (!FINAL) {
        if (tid < k) out[((size_t)b * gridDim.x + c) * (size_t)k + tid] = s_list[tid];
    } else if constexpr (!CROWD) {
        if (tid < kWave) {
            const uint64_t w = tid < k ? s_list[tid] : kTopkPad;
            topk_finish(fin, b, k, tid, topk_key(w), topk_id(w));
        }
    } else {
        // which winners are the m-th (last) candidate of their tile?
        if (tid < kWave) {
            const uint64_t w = tid < k ? s_list[tid] : kTopkPad;
            int t = -1;
            bool flagged = false;
            if ((uint32_t)w != 0u) {
                t = (topk_id(w) - crowd.vocab_offset) >> 7;
                flagged = crowd.cand[((size_t)b * crowd.T + t) * (size_t)crowd.m + (crowd.m - 1)] == w;
            }
            const uint64_t fb = __ballot(flagged);
            const int ncrowd = (int)__builtin_popcountll(fb);        // <= k / m: such a tile holds m winners
            if (tid == 0) s_ncrowd = ncrowd;
            if (ncrowd == 0) {
                topk_finish(fin, b, k, tid, topk_key(w), topk_id(w));
            } else {
                if (flagged) s_crowd_tile[(int)__builtin_popcountll(fb & ((1ull << tid) - 1ull))] = t;
                bool listed = false;
                for (uint64_t r = fb; r != 0ull; r &= r - 1ull) {
                    const int tf = __shfl(t, (int)__builtin_ctzll(r), kWave);
                    listed = listed || t == tf;
                }
                s_list[tid] = listed ? kTopkPad : w;        // the listed tiles come back whole below
            }
        }
        __syncthreads();
        const int ncrowd = s_ncrowd;
        if (ncrowd == 0) return;                                     // uniform over the workgroup
        // keys of the listed tiles: wave w takes rows 32 w .. 32 w + 31 of a tile, its lanes split K
        const int D = crowd.D;
        const uint16_t* h = crowd.H + (size_t)b * D;
        const float inv_tau = 1.0f / crowd.tau[b];
        const uint64_t sd = fin.row_seeds ? fin.row_seeds[b] : fin.seed;
        for (int f = 0; f < ncrowd; ++f) {
            const int v0 = s_crowd_tile[f] * kVocabTile + wave * 32;
            float acc[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) acc[i] = 0.0f;
            for (int kc = lane * 8; kc < D; kc += 512) {
                const uint4 hv = *reinterpret_cast<const uint4*>(h + kc);
                const uint32_t hw[4] = {hv.x, hv.y, hv.z, hv.w};
#pragma unroll
                for (int i = 0; i < 32; ++i) {
                    int row = v0 + i;
                    row = row < crowd.V - 1 ? row : crowd.V - 1;
                    const uint4 wv = *reinterpret_cast<const uint4*>(crowd.W + (size_t)row * D + kc);
                    const uint32_t ww[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        acc[i] = fmaf(__uint_as_float(hw[q] << 16), __uint_as_float(ww[q] << 16), acc[i]);
                        acc[i] = fmaf(__uint_as_float(hw[q] & 0xFFFF0000u), __uint_as_float(ww[q] & 0xFFFF0000u), acc[i]);
                    }
                }
            }
            float y = 0.0f;
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                float a = acc[i];
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) a += __shfl_xor(a, off, kWave);
                y = lane == i ? a : y;
            }
            if (lane < 32) {
                const int v = v0 + lane;
                const int32_t id = crowd.vocab_offset + v;
                float g = 0.0f;
                if (fin.mode == kTopkGumbel) {
                    uint32_t pw[4];
                    philox4x32_10((uint32_t)id >> 2, (uint32_t)(uint64_t)(fin.row_offset + b), 0u, 0u, (uint32_t)sd, (uint32_t)(sd >> 32), pw);
                    const uint32_t q = (uint32_t)id & 3u;
                    const uint32_t r = q == 0u ? pw[0] : q == 1u ? pw[1] : q == 2u ? pw[2] : pw[3];
                    g = (fin.epi_flags & kEpiExactLog) ? gumbel_from_word_exact(r) : gumbel_from_word(r);
                }
                s_list[64 + f * kVocabTile + wave * 32 + lane] = v < crowd.V ? topk_pack(fmaf(y, inv_tau, g), id) : kTopkPad;
            }
        }
        static_assert(64 + kTopkCrowdMax * kVocabTile <= 4096, "list of the second selection");
        const int n = 64 + ncrowd * kVocabTile;
        int n2 = 256;
        while (n2 < n) n2 <<= 1;
        for (int t2 = k + tid; t2 < 64; t2 += 256) s_list[t2] = kTopkPad;
        for (int t2 = n + tid; t2 < n2; t2 += 256) s_list[t2] = kTopkPad;
        __syncthreads();
        lds_sort_desc(s_list, n2, tid);                               // ends with a barrier
        if (tid < kWave) {
            const uint64_t w = tid < k ? s_list[tid] : kTopkPad;
            topk_finish(fin, b, k, tid, topk_key(w), topk_id(w));
        }
    }
}

}  // namespace fs
