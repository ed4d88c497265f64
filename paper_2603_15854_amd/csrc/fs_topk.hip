// Translation unit of the truncated-support path: the tiled stage-1 kernel with the per-tile top-k
// epilogue, the candidate reduction, the nucleus rule and the draw (fs_topk_kernels.hpp).
#include "fs_launch_tiled2.hpp"
#include "fs_topk_kernels.hpp"

namespace fs {

// Stage 1 with the per-tile top-k epilogue.  Three tile shapes (by batch size), whole K steps only.
fs_status launch_stage1_topk(const Stage1Params& p, hipStream_t st)
{
    if (p.D % 64 != 0) return FS_ERR_UNSUPPORTED;
    if (p.B <= 32) return launch_tiled2<Shape6, false, 2, false, false, false, true>(p, st);   // 512 x 32
    if (p.B <= 64) return launch_tiled2<Shape7, false, 2, false, false, false, true>(p, st);   // 512 x 64
    return launch_tiled2<Shape3, false, 2, false, false, true, true>(p, st);                   // 256 x 128, batch tiles XCD-paired
}

// Chunks a row of N candidates is cut into for the first selection pass: enough workgroups to fill
// the device at small B, never chunks shorter than 2048 elements, at most 64.
int topk_chunks(int B, int N)
{
    int want = (512 + B - 1) / B;
    const int cap = (N + 2047) / 2048;
    want = want < cap ? want : cap;
    want = want < 64 ? want : 64;
    return want < 1 ? 1 : want;
}

fs_status launch_keys_from_logits(float* logits, int B, int V, const float* tau, uint64_t seed, const uint64_t* row_seeds,
                                  int64_t row_offset, int32_t vocab_offset, int mode, uint32_t epi_flags, hipStream_t st)
{
    return launch(keys_from_logits_kernel, dim3((V + 1023) / 1024, B), dim3(256), 0, st, logits, V, tau, seed, row_seeds,
                  row_offset, vocab_offset, mode, epi_flags);
}

// The k best of every row of [B, N] candidates ((vals, ids) pairs, or keys with id = id_base +
// position when ids is null): chunks first, then the chunks' results.  tmp_* hold B * chunks * k
// pairs, fin_* B * k.
fs_status launch_topk_reduce(const float* vals, const int32_t* ids, int B, int N, int64_t row_stride, int32_t id_base,
                             int k, float* tmp_val, int32_t* tmp_idx, float* fin_val, int32_t* fin_idx, hipStream_t st)
{
    const int chunks = topk_chunks(B, N);
    const int chunk_len = (N + chunks - 1) / chunks;
    fs_status s;
    if (chunks == 1) {
        if (ids) return launch(topk_select_kernel<true>, dim3(1, B), dim3(256), 0, st, vals, ids, row_stride, N, id_base, chunk_len, k, fin_val, fin_idx);
        return launch(topk_select_kernel<false>, dim3(1, B), dim3(256), 0, st, vals, ids, row_stride, N, id_base, chunk_len, k, fin_val, fin_idx);
    }
    if (ids) s = launch(topk_select_kernel<true>, dim3(chunks, B), dim3(256), 0, st, vals, ids, row_stride, N, id_base, chunk_len, k, tmp_val, tmp_idx);
    else s = launch(topk_select_kernel<false>, dim3(chunks, B), dim3(256), 0, st, vals, ids, row_stride, N, id_base, chunk_len, k, tmp_val, tmp_idx);
    if (s != FS_OK) return s;
    const int n2 = chunks * k;
    return launch(topk_select_kernel<true>, dim3(1, B), dim3(256), 0, st, (const float*)tmp_val, (const int32_t*)tmp_idx,
                  (int64_t)n2, n2, 0, n2, k, fin_val, fin_idx);
}

fs_status launch_topk_finish(const float* fin_val, const int32_t* fin_idx, int B, int k, float top_p, int mode, uint64_t seed,
                             const uint64_t* row_seeds, int64_t row_offset, uint32_t epi_flags, int32_t* out_idx,
                             float* out_val, float* topk_val, int32_t* topk_idx, int32_t* n_kept, hipStream_t st)
{
    return launch(topk_finish_kernel, dim3(B), dim3(64), 0, st, fin_val, fin_idx, k, top_p, mode, seed, row_seeds,
                  row_offset, epi_flags, out_idx, out_val, topk_val, topk_idx, n_kept);
}

}  // namespace fs
