// Translation unit of the truncated-support path: the tiled stage-1 kernel with the per-tile top-k
// epilogue, the candidate reduction, the nucleus rule and the draw (fs_topk_kernels.hpp).
#include "fs_launch_tiled2.hpp"
#include "fs_topk_kernels.hpp"

namespace fs {

// Stage 1 with the per-tile candidate epilogue, whole K steps only.  shape = 0: the split-K kernel in
// the decode regime, else the tile shape pick_tile_shape takes for the plain path (the shape decides
// how many rounds of workgroups a launch needs: at V = 152064, B = 64 the 512 x 64 shape takes 247 us
// and the 128 x 64 shape 199 us), except that the two 128-row shapes whose waves share candidate tiles
// (256 x 128, 128 x 128) give way to the 256 x 128 form of the kernel with direct global -> LDS loads
// (C2 shape, B = 128: 196 us against 209 and 234 us; D = 3584, V = 152064: 242 us against 251 and 252 us).
// shape = 1..8, 10, 12, 13 forces that shape (tuning aid and test hook).
fs_status launch_stage1_topk(const Stage1Params& p, int shape, hipStream_t st)
{
    if (p.D % 64 != 0) return FS_ERR_UNSUPPORTED;
    if (shape == 0) {
        if (p.B <= 16 && p.D <= 4096) return launch_stage1_splitk_topk(p, st);
        int cus = 0;
        const fs_status ds = current_device(nullptr, &cus);
        if (ds != FS_OK) return ds;
        shape = pick_tile_shape(p.B, p.D, p.V, cus);
        if (shape == 3 || shape == 4) shape = 13;
    }
    switch (shape) {
    case 1: return launch_tiled2<Shape1, false, 2, false, false, false, true>(p, st);   // 128 x 32
    case 2: return launch_tiled2<Shape2, false, 2, false, false, false, true>(p, st);   // 256 x 64
    case 3: return launch_tiled2<Shape3, false, 2, false, false, true, true>(p, st);    // 256 x 128, batch tiles XCD-paired
    case 4: return launch_tiled2<Shape4, false, 2, false, false, true, true>(p, st);    // 128 x 128
    case 5: return launch_tiled2<Shape5, false, 2, false, false, false, true>(p, st);   // 128 x 64
    case 6: return launch_tiled2<Shape6, false, 2, false, false, false, true>(p, st);   // 512 x 32
    case 7: return launch_tiled2<Shape7, false, 2, false, false, false, true>(p, st);   // 512 x 64
    case 8: return launch_tiled2<Shape8, false, 2, false, false, false, true>(p, st);   // 256 x 32
    case 10: return launch_tiled2<Shape10, false, 2, false, false, false, true>(p, st); // 512 x 128
    case 12: return launch_stage1_dma_topk(p, 256, st);
    case 13: return launch_stage1_dma_topk(p, 128, st);
    default: return FS_ERR_UNSUPPORTED;
    }
}

// Selection levels for rows of N candidates: every level cuts a row into chunks of at most kSelChunk
// candidates and leaves k per chunk; the last level has one chunk.  The first level uses more (shorter)
// chunks than it must when B is small, to fill the device, as long as the next level still fits one
// workgroup.
TopkPlan topk_plan(int B, int N, int k)
{
    TopkPlan pl = {};
    int64_t n = N;
    for (int lvl = 0; lvl < TopkPlan::kMaxLevels; ++lvl) {
        int64_t c = (n + kSelChunk - 1) / kSelChunk;
        if (c > 1 && lvl == 0) {
            const int64_t one_more = kSelChunk / k;                  // chunks the next level takes in one workgroup
            int64_t want = (512 + B - 1) / B;
            const int64_t cap = (n + 1023) / 1024;
            want = want < cap ? want : cap;
            want = want < one_more ? want : one_more;
            c = c > want ? c : want;
        }
        pl.chunks[lvl] = (int)c;
        pl.n[lvl] = (int)n;
        pl.levels = lvl + 1;
        if (c == 1) break;
        n = c * k;
    }
    // outputs of levels 0, 2 go to the first buffer, of level 1 to the second (the last level writes none)
    pl.buf_words[0] = pl.levels > 1 ? (size_t)B * pl.chunks[0] * k : 0;
    pl.buf_words[1] = pl.levels > 2 ? (size_t)B * pl.chunks[1] * k : 0;
    return pl;
}

// The k best of every row of [B, N] candidates, then the nucleus rule and the draw.  buf0 / buf1:
// topk_plan's buffers.
fs_status launch_topk_reduce(const void* in, const TopkKeys* keys, int B, int N, int64_t row_stride, int32_t id_base, int k,
                             uint64_t* buf0, uint64_t* buf1, const TopkFinish& fin, const TopkCrowd* crowd, hipStream_t st)
{
    const TopkPlan pl = topk_plan(B, N, k);
    if (pl.chunks[pl.levels - 1] != 1 || B > 65535) return FS_ERR_SHAPE;
    const TopkKeys kp = keys ? *keys : TopkKeys{};
    const TopkCrowd none = {};
    const void* src = in;
    for (int lvl = 0; lvl < pl.levels; ++lvl) {
        const int c = pl.chunks[lvl], n = pl.n[lvl];
        int chunk_len = (n + c - 1) / c;
        chunk_len = (chunk_len + 3) & ~3;                  // chunks of key rows start at whole groups of four ids
        const bool last = lvl == pl.levels - 1;
        uint64_t* dst = last ? nullptr : (lvl & 1) ? buf1 : buf0;
        const bool from_keys = keys && lvl == 0;
        const int64_t stride = lvl == 0 ? row_stride : (int64_t)n;
        const int32_t base = lvl == 0 ? id_base : 0;
        fs_status s;
        const dim3 grid(c, B), block(256);
        if (from_keys && last) s = launch(topk_select_kernel<true, true>, grid, block, 0, st, src, stride, n, base, chunk_len, k, dst, kp, fin, none);
        else if (from_keys) s = launch(topk_select_kernel<true, false>, grid, block, 0, st, src, stride, n, base, chunk_len, k, dst, kp, fin, none);
        else if (last && crowd) s = launch(topk_select_kernel<false, true, true>, grid, block, 0, st, src, stride, n, base, chunk_len, k, dst, kp, fin, *crowd);
        else if (last) s = launch(topk_select_kernel<false, true>, grid, block, 0, st, src, stride, n, base, chunk_len, k, dst, kp, fin, none);
        else s = launch(topk_select_kernel<false, false>, grid, block, 0, st, src, stride, n, base, chunk_len, k, dst, kp, fin, none);
        if (s != FS_OK) return s;
        src = dst;
    }
    return FS_OK;
}

}  // namespace fs
