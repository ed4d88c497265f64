// Host-side launch logic of the persistent split-K stage-1 kernel (fs_stage1_splitk.hpp).
#pragma once

#include "fs_host.hpp"
#include "fs_stage1_splitk.hpp"

namespace fs {

// nw waves of kpw k-steps each; the grid is as many workgroups as are resident at once
// (registers and LDS decide), or wgs_per_cu_override per compute unit when that is > 0.
template <class Cfg, bool FULL = false, bool TOPK = false>
fs_status launch_splitk(const Stage1Params& p, int kpw, int nw, int wgs_per_cu_override, hipStream_t st)
{
    const size_t lds = TOPK ? Cfg::lds_bytes_topk(nw) : Cfg::lds_bytes(nw);
    if (nw > Cfg::kMaxWaves || lds > kLdsPerCU) return FS_ERR_UNSUPPORTED;
    auto kernel = stage1_splitk_kernel<Cfg, FULL, TOPK>;
    int dev = 0, cus = 0;
    const fs_status ds = current_device(&dev, &cus);
    if (ds != FS_OK) return ds;
    static PerDevice<Cfg::kMaxWaves + 1> state;
    if (!state.attr[dev].load(std::memory_order_acquire)) {
        if (allow_lds(kernel, kLdsPerCU) != hipSuccess) return FS_ERR_HIP;
        state.attr[dev].store(true, std::memory_order_release);
    }
    int per_cu = state.resident[dev][nw].load(std::memory_order_acquire);
    if (per_cu == 0) {
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, nw * kWave, lds) != hipSuccess)
            return FS_ERR_HIP;
        per_cu = occ < 1 ? 1 : occ;
        state.resident[dev][nw].store(per_cu, std::memory_order_release);
    }
    if (wgs_per_cu_override > 0) per_cu = wgs_per_cu_override;
    int grid = cus * per_cu;
    if (grid > p.T) grid = p.T;
    return launch(kernel, dim3(grid), dim3(nw * kWave), lds, st, p, nw, kpw);
}

}  // namespace fs
