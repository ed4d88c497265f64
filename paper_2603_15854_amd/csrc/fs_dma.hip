// Translation unit of the large-batch stage-1 kernel with direct global -> LDS loads
// (fs_stage1_dma.hpp), bf16 weights, plain and full-transform epilogue.
#include "fs_host.hpp"
#include "fs_stage1_dma.hpp"

namespace fs {

namespace {

template <class Cfg, bool FULL, bool TOPK = false>
fs_status launch_dma(const Stage1Params& p, hipStream_t st)
{
    if (p.D % Cfg::kKS != 0) return FS_ERR_UNSUPPORTED;   // whole K steps only
    static_assert(Cfg::lds_bytes() <= kLdsPerCU, "stages do not fit LDS");
    const int nbt = (p.B + Cfg::BT - 1) / Cfg::BT;
    const int macro_tiles = (p.V + Cfg::VT - 1) / Cfg::VT;
    const long long grid = (long long)((macro_tiles + 7) / 8) * 8 * nbt;
    if (grid > 0x7FFFFFFFll) return FS_ERR_SHAPE;
    int dev = 0;
    const fs_status ds = current_device(&dev, nullptr);
    if (ds != FS_OK) return ds;
    auto k_stream = stage1_dma_kernel<Cfg, true, FULL, TOPK>;    // one batch tile: W is read once, non-temporal
    auto k_shared = stage1_dma_kernel<Cfg, false, FULL, TOPK>;   // several: the second read of a W tile hits L2
    static PerDevice<> state;
    if (!state.attr[dev].load(std::memory_order_acquire)) {
        if (allow_lds(k_stream, kLdsPerCU) != hipSuccess) return FS_ERR_HIP;
        if (allow_lds(k_shared, kLdsPerCU) != hipSuccess) return FS_ERR_HIP;
        state.attr[dev].store(true, std::memory_order_release);
    }
    return launch(nbt == 1 ? k_stream : k_shared, dim3((unsigned)grid), dim3(Cfg::kThreads), Cfg::lds_bytes(), st, p, nbt);
}

}  // namespace

// 256 vocabulary rows x 256 (or 128) batch rows per workgroup
fs_status launch_stage1_dma(const Stage1Params& p, bool full, int batch_tile, hipStream_t st)
{
    if (batch_tile == 128) return full ? launch_dma<DmaCfg<128>, true>(p, st) : launch_dma<DmaCfg<128>, false>(p, st);
    return full ? launch_dma<DmaCfg<256>, true>(p, st) : launch_dma<DmaCfg<256>, false>(p, st);
}

// The same kernel with the per-tile candidate epilogue of the truncated-support path.
fs_status launch_stage1_dma_topk(const Stage1Params& p, int batch_tile, hipStream_t st)
{
    return batch_tile == 128 ? launch_dma<DmaCfg<128>, false, true>(p, st) : launch_dma<DmaCfg<256>, false, true>(p, st);
}

}  // namespace fs
