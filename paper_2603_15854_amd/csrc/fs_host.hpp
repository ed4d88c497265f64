// Host-side pieces shared by the translation units of the library: per-device state, the launch
// helper, and the stage-1 launchers each kernel family exports to the C ABI file.  Nothing here
// touches the data; every step of the method runs in the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>
#include <type_traits>

#include "flash_sample.h"
#include "fs_common.hpp"
#include "fs_topk_common.hpp"

namespace fs {

constexpr size_t kLdsPerCU = 160 * 1024;   // gfx950
constexpr int kMaxDevices = 64;            // device ordinals the per-device tables cover

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Compute units of the current device (cached per device).  FS_OK, FS_ERR_DEVICE when the device
// ordinal does not fit the tables, FS_ERR_HIP when the runtime fails.
fs_status current_device(int* dev_out, int* cus_out);

// Launch through hipLaunchKernel so that the status is the one of THIS launch (the sticky
// last-error slot of the runtime may hold an unrelated library's earlier failure).
template <class... KArgs, class... Args>
inline fs_status launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count");
    // one local copy per kernel parameter, converted to the parameter's exact type
    auto pack = [&](std::remove_cv_t<KArgs>... vals) {
        void* ptrs[] = {static_cast<void*>(&vals)...};
        return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds, st);
    };
    return pack(args...) == hipSuccess ? FS_OK : FS_ERR_HIP;
}

// Kernels that use more than 64 KiB of dynamic LDS must say so once per device (a function
// attribute belongs to the device that was current when it was set).
template <class K>
inline hipError_t allow_lds(K kernel, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// Per-kernel, per-device set-up state of one launcher instantiation.  The values are idempotent
// (a flag, an occupancy count), so concurrent first calls only repeat the set-up.
template <int N = 1>
struct PerDevice {
    std::atomic<bool> attr[kMaxDevices] = {};
    std::atomic<int> resident[kMaxDevices][N] = {};
};

inline int num_tiles(int V) { return (V + kVocabTile - 1) / kVocabTile; }

// Tile shape (FS_TUNE_TILE_SHAPE number) the tiled kernel takes for (B, V) on `cus` compute units.
int pick_tile_shape(int B, int D, int V, int cus);

// Stage-1 launchers, one per kernel family / translation unit.  `shape` = 0: automatic.
fs_status launch_stage1_splitk(const Stage1Params& p, bool full, int wgs_per_cu, hipStream_t st);
fs_status launch_stage1_tiled(const Stage1Params& p, int shape, hipStream_t st);
fs_status launch_stage1_tiled_full(const Stage1Params& p, int shape, hipStream_t st);
fs_status launch_stage1_dma(const Stage1Params& p, bool full, int batch_tile, hipStream_t st);
fs_status launch_stage1_w8(const Stage1Params& p, int variant, int tune, hipStream_t st);
fs_status launch_stage1_w4(const Stage1Params& p, const uint8_t* scales, int wgs_per_cu, hipStream_t st);
// truncated supports (fs_topk.hip)
fs_status launch_stage1_topk(const Stage1Params& p, int shape, hipStream_t st);
fs_status launch_stage1_dma_topk(const Stage1Params& p, int batch_tile, hipStream_t st);   // fs_dma.hip
fs_status launch_stage1_splitk_topk(const Stage1Params& p, hipStream_t st);   // fs_splitk.hip
struct TopkPlan {                 // selection levels for rows of N candidates (topk_plan)
    static constexpr int kMaxLevels = 4;
    int levels;
    int chunks[kMaxLevels];       // chunks per row at each level; 1 at the last
    int n[kMaxLevels];            // candidates per row at each level
    size_t buf_words[2];          // 64-bit words of the two intermediate buffers
};
TopkPlan topk_plan(int B, int N, int k);
// keys: how stored logits become keys (input = fp32 [B, N] logits), or null (input = packed candidates);
// crowd: the fused path's check for tiles that hold more winners than they emitted, or null
fs_status launch_topk_reduce(const void* in, const TopkKeys* keys, int B, int N, int64_t row_stride, int32_t id_base, int k,
                             uint64_t* buf0, uint64_t* buf1, const TopkFinish& fin, const TopkCrowd* crowd, hipStream_t st);
fs_status launch_mxfp4_decode(const uint32_t* codes, const uint8_t* scales, int n8, float* out, hipStream_t st);

}  // namespace fs
