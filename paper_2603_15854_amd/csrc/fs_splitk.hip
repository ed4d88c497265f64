// Translation unit of the split-K stage-1 kernel for bf16 weights (B <= 16, D <= 4096), with the
// plain and the full-transform epilogue.
#include "fs_launch_splitk.hpp"

namespace fs {

fs_status launch_stage1_splitk(const Stage1Params& p, bool full, int wgs_per_cu, hipStream_t st)
{
    // a wave keeps 32 k-steps of the hidden states (128 VGPRs) and up to four waves split K
    const int ksteps = (p.D + 31) / 32;
    if (p.B > 16 || ksteps > 32 * 4) return FS_ERR_UNSUPPORTED;
    const int nw = (ksteps + 31) / 32;
    const int kpw = (ksteps + nw - 1) / nw;
    using Cfg = SplitKCfg<32, 8, 2, 4>;   // 8-k-step LDS stages, two register sets in flight
    return full ? launch_splitk<Cfg, true>(p, kpw, nw, wgs_per_cu, st)
                : launch_splitk<Cfg, false>(p, kpw, nw, wgs_per_cu, st);
}

// The same kernel with the per-tile candidate epilogue of the truncated-support path.
fs_status launch_stage1_splitk_topk(const Stage1Params& p, hipStream_t st)
{
    const int ksteps = (p.D + 31) / 32;
    if (p.B > 16 || ksteps > 32 * 4) return FS_ERR_UNSUPPORTED;
    const int nw = (ksteps + 31) / 32;
    const int kpw = (ksteps + nw - 1) / nw;
    return launch_splitk<SplitKCfg<32, 8, 2, 4>, false, true>(p, kpw, nw, 0, st);
}

}  // namespace fs
