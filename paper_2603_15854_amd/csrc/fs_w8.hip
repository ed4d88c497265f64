// Translation unit of the stage-1 kernels on FP8 (E4M3) weights: one-byte W elements, otherwise
// the kernels of the bf16 path.
#include "fs_launch_splitk.hpp"
#include "fs_launch_tiled2.hpp"

namespace fs {

// variant: FS_VARIANT_AUTO, FS_VARIANT_SPLITK (tune = workgroups per CU) or FS_VARIANT_TILED2
// (tune = tile shape, 0 = automatic).
fs_status launch_stage1_w8(const Stage1Params& p, int variant, int tune, hipStream_t st)
{
    const int ksteps = (p.D + 31) / 32;
    const bool splitk_ok = p.B <= 16 && ksteps <= 32 * 8;
    if (variant == FS_VARIANT_SPLITK && !splitk_ok) return FS_ERR_UNSUPPORTED;
    if (variant != FS_VARIANT_TILED2 && splitk_ok) {
        const int wgs = variant == FS_VARIANT_SPLITK ? tune : 0;
        if (ksteps <= 32 * 4) {   // eight waves of 16 k-steps: 82 us against 90 us for four waves of 32;
            // 8-k-step stages with two register sets in flight: 84.7 us against 85.7 us at B = 16 for one
            // 16-k-step stage (more of the stream stays in flight across a tile's epilogue)
            const int nw = (ksteps + 15) / 16;
            return launch_splitk<SplitKCfg<16, 8, 2, 8, 1>>(p, (ksteps + nw - 1) / nw, nw, wgs, st);
        }
        // wide hidden sizes: eight waves of 32 k-steps, one register set of prefetch
        const int nw = (ksteps + 31) / 32;
        return launch_splitk<SplitKCfg<32, 16, 1, 8, 1>>(p, (ksteps + nw - 1) / nw, nw, wgs, st);
    }
    // Larger batches and wider hidden sizes: the tiled kernel with the codes kept in LDS.  A K step
    // is then 128 elements (the same 128-byte line of a W row as on the bf16 path); other hidden
    // sizes run on the two-per-CU shapes that widen the codes when a step is parked.
    if (p.D % 128 != 0) return launch_tiled2_ragged<false, 1>(p, st);
    int shape = variant == FS_VARIANT_TILED2 ? tune : 0;
    if (shape == 0) {
        int cus = 0;
        const fs_status ds = current_device(nullptr, &cus);
        if (ds != FS_OK) return ds;
        shape = pick_tile_shape(p.B, 0, p.V, cus);   // hidden size 0: only shapes this kernel family has
    }
    switch (shape) {
    case 1: return launch_tiled2<Tiled2Cfg<32, 4, 1, 2>, false, 1, true>(p, st);
    case 2: return launch_tiled2<Tiled2Cfg<64, 4, 2, 1, 2, 256>, false, 1, true>(p, st);
    case 4: return launch_tiled2<Tiled2Cfg<128, 2, 2, 1, 2>, false, 1, true, false, true>(p, st);
    case 5: return launch_tiled2<Tiled2Cfg<64, 2, 2, 1, 2>, false, 1, true>(p, st);
    case 6: return launch_tiled2<Tiled2Cfg<32, 8, 1, 1, 1, 512>, false, 1, true>(p, st);
    case 7: return launch_tiled2<Tiled2Cfg<64, 4, 2, 1, 1, 512, 1>, false, 1, true>(p, st);
    case 8: return launch_tiled2<Tiled2Cfg<32, 4, 1, 1, 2, 256>, false, 1, true>(p, st);
    case 3:
    case 10:   // 512 x 128 and 256 x 256 do not fit LDS with two hidden sub-tiles per step, and the
    case 12:   // direct-to-LDS kernel exists for bf16 only: all run as 256 x 128
    case 13:
        return launch_tiled2<Tiled2Cfg<128, 4, 2, 1, 2, 256>, false, 1, true, false, true>(p, st);
    default: break;
    }
    return FS_ERR_UNSUPPORTED;
}

}  // namespace fs
