// Host-side launch logic of the LDS-tiled stage-1 kernel (fs_stage1_tiled2.hpp): tile-shape table,
// one-time per-device set-up, grid computation.  Included by the translation units that
// instantiate the kernel (bf16 with and without the full-transform epilogue, FP8 weights).
#pragma once

#include "fs_host.hpp"
#include "fs_stage1_tiled2.hpp"

namespace fs {

// BOTH: also build the form with cacheable W loads for launches with several batch tiles (the
// workgroups that share a W tile then run on one XCD and the second read hits its L2); without it
// such launches stream W with non-temporal loads like single-batch-tile ones.
template <class Cfg, bool FULL = false, int WB = 2, bool WCODES = false, bool KRAG = false, bool BOTH = false, bool TOPK = false,
          bool W4 = false>
fs_status launch_tiled2(const Stage1Params& p, hipStream_t st)
{
    if (!KRAG && p.D % (W4 ? 256 : WCODES ? 128 : 64) != 0) return FS_ERR_UNSUPPORTED;   // whole K steps only
    // LDS: two buffers of one K step; with codes in LDS a step carries two hidden sub-tiles (four with
    // MXFP4 codes, plus 8 scale bytes per row)
    constexpr size_t kLdsLoop = 2 * ((size_t)Cfg::kWBytes + (W4 ? 4 : WCODES ? 2 : 1) * (size_t)Cfg::kHBytes + (W4 ? Cfg::VT * 8 : 0));
    constexpr size_t kLds = kLdsLoop;
    static_assert(kLds <= kLdsPerCU, "tile shape does not fit LDS");
    const int nbt = (p.B + Cfg::BT - 1) / Cfg::BT;
    const int macro_tiles = (p.V + Cfg::VT - 1) / Cfg::VT;
    const long long grid = (long long)((macro_tiles + 7) / 8) * 8 * nbt;
    if (grid > 0x7FFFFFFFll) return FS_ERR_SHAPE;
    int dev = 0;
    const fs_status ds = current_device(&dev, nullptr);
    if (ds != FS_OK) return ds;
    auto k_stream = stage1_tiled2_kernel<Cfg, true, FULL, WB, WCODES, KRAG, TOPK, W4>;
    auto k_shared = stage1_tiled2_kernel<Cfg, !BOTH, FULL, WB, WCODES, KRAG, TOPK, W4>;   // the same kernel unless BOTH
    static PerDevice<> state;
    if (!state.attr[dev].load(std::memory_order_acquire)) {
        if (allow_lds(k_stream, kLdsPerCU) != hipSuccess) return FS_ERR_HIP;
        if (BOTH && allow_lds(k_shared, kLdsPerCU) != hipSuccess) return FS_ERR_HIP;
        state.attr[dev].store(true, std::memory_order_release);
    }
    return launch(nbt == 1 ? k_stream : k_shared, dim3((unsigned)grid), dim3(Cfg::kThreads), kLds, st, p, nbt);
}

// Tile shapes (vocabulary rows x batch rows per workgroup); numbers are those of FS_TUNE_TILE_SHAPE:
//   1: 128 x 32   4 waves, two workgroups per CU      5: 128 x 64   4 waves, two per CU
//   2: 256 x 64   8 waves, one per CU                 6: 512 x 32   8 waves, one per CU
//   3: 256 x 128  8 waves, one per CU                 7: 512 x 64   8 waves, one per CU
//   4: 128 x 128  4 waves, two per CU                 8: 256 x 32   4 waves, two per CU
//  10: 512 x 128  8 waves, one per CU, one register set of prefetch (128 accumulator VGPRs, 160 KB of LDS)
//  12: 256 x 256  4 waves, the kernel with direct global -> LDS loads of fs_stage1_dma.hpp (another
//      translation unit); 9 was the 256 x 256 shape of this kernel, which 12 replaced
//  13: 256 x 128  the same kernel with 128 batch rows per workgroup
using Shape1 = Tiled2Cfg<32, 4, 1, 4>;
using Shape2 = Tiled2Cfg<64, 4, 2, 2, 2, 256>;
using Shape3 = Tiled2Cfg<128, 4, 2, 1, 2, 256>;
using Shape4 = Tiled2Cfg<128, 2, 2, 2, 2>;
using Shape5 = Tiled2Cfg<64, 2, 2, 2, 2>;
using Shape6 = Tiled2Cfg<32, 8, 1, 1, 1, 512>;
using Shape7 = Tiled2Cfg<64, 4, 2, 1, 1, 512>;
using Shape8 = Tiled2Cfg<32, 4, 1, 1, 2, 256>;
using Shape10 = Tiled2Cfg<128, 4, 2, 1, 2, 512, 1>;

// A hidden size that is not a multiple of the K step runs on the three two-per-CU shapes, built
// with the zeroing of the last step's tail; every other shape exists for whole K steps only.
template <bool FULL, int WB = 2>
fs_status launch_tiled2_ragged(const Stage1Params& p, hipStream_t st)
{
    if (p.B <= 32) return launch_tiled2<Shape8, FULL, WB, false, true>(p, st);
    if (p.B <= 64) return launch_tiled2<Shape5, FULL, WB, false, true>(p, st);
    return launch_tiled2<Shape4, FULL, WB, false, true>(p, st);
}

// bf16 weights.  `shape` = 0 picks by pick_tile_shape; 1..8, 10, 12, 13 force one shape (tuning aid and
// tiling-invariance tests; honoured for whole-K-step hidden sizes only).
template <bool FULL>
fs_status launch_tiled2_bf16(const Stage1Params& p, int shape, hipStream_t st)
{
    if (p.D % 64 != 0) return launch_tiled2_ragged<FULL>(p, st);
    if (shape == 0) {
        int cus = 0;
        const fs_status ds = current_device(nullptr, &cus);
        if (ds != FS_OK) return ds;
        shape = pick_tile_shape(p.B, p.D, p.V, cus);
    }
    switch (shape) {
    case 1: return launch_tiled2<Shape1, FULL>(p, st);
    case 2: return launch_tiled2<Shape2, FULL>(p, st);
    case 3: return launch_tiled2<Shape3, FULL, 2, false, false, true>(p, st);
    case 4: return launch_tiled2<Shape4, FULL, 2, false, false, true>(p, st);
    case 5: return launch_tiled2<Shape5, FULL>(p, st);
    case 6: return launch_tiled2<Shape6, FULL>(p, st);
    case 7: return launch_tiled2<Shape7, FULL>(p, st);
    case 8: return launch_tiled2<Shape8, FULL>(p, st);
    case 10: return launch_tiled2<Shape10, FULL>(p, st);
    case 12: return launch_stage1_dma(p, FULL, 256, st);
    case 13: return launch_stage1_dma(p, FULL, 128, st);
    default: break;
    }
    return FS_ERR_UNSUPPORTED;
}

}  // namespace fs
