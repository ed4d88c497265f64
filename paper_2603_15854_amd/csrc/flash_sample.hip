// Host side of the C ABI declared in include/flash_sample.h: argument checks, kernel choice,
// launches.  Every step of the method runs in the kernels; nothing here touches the data.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <mutex>

#include "flash_sample.h"
#include "fs_aux_kernels.hpp"
#include "fs_common.hpp"
#include "fs_grouped_kernels.hpp"
#include "fs_stage1_splitk.hpp"
#include "fs_stage1_tiled.hpp"
#include "fs_stage1_tiled2.hpp"
#include "fs_stage1_w4.hpp"

namespace {

using namespace fs;

constexpr size_t kLdsPerCU = 160 * 1024;   // gfx950
constexpr int kMaxDevices = 16;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

struct DeviceInfo {
    bool known = false;
    int cus = 256;
    void* ws = nullptr;      // workspace cache of the plain entry point
    size_t ws_bytes = 0;
};
DeviceInfo g_dev[kMaxDevices];
std::mutex g_mu;

// Compute units of the current device (cached).  Returns <= 0 on a HIP error.
int current_device_cus(int* dev_out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_dev[dev].known) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            return -1;
        g_dev[dev].cus = cus;
        g_dev[dev].known = true;
    }
    if (dev_out) *dev_out = dev;
    return g_dev[dev].cus;
}

// Kernels that use more than 64 KiB of dynamic LDS must say so once per device (a function
// attribute belongs to the device that was current when it was set).
template <class K>
hipError_t allow_lds(K kernel, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// Per-kernel, per-device set-up state of one launcher instantiation.  Written under g_mu; the
// values are idempotent, so a reader that misses a concurrent update only repeats the set-up.
template <int N = 1>
struct PerDevice {
    bool attr[kMaxDevices] = {};
    int resident[kMaxDevices][N] = {};
};

fs_status check_problem(const void* hidden, const void* W, int B, int D, int V,
                        int64_t row_offset, int32_t vocab_offset)
{
    if (B < 0 || D <= 0 || V <= 0 || (D & 7) != 0) return FS_ERR_SHAPE;
    if (vocab_offset < 0 || (int64_t)vocab_offset + (int64_t)V > (int64_t)INT32_MAX) return FS_ERR_SHAPE;
    if (row_offset < 0) return FS_ERR_SHAPE;
    if (B == 0) return FS_OK;
    if (!hidden || !W) return FS_ERR_NULL;
    if (!aligned(hidden, 16) || !aligned(W, 16)) return FS_ERR_ALIGN;
    return FS_OK;
}

inline int num_tiles(int V) { return (V + kVocabTile - 1) / kVocabTile; }
inline int num_chunks(int V) { return (V + kLogitsChunk - 1) / kLogitsChunk; }

struct Workspace {
    float* cand_val;
    int32_t* cand_idx;
};

size_t workspace_bytes(int B, int V)
{
    if (B <= 0 || V <= 0) return 0;
    const size_t per = align_up((size_t)B * (size_t)num_tiles(V) * 4, 256);
    return 2 * per;
}

Workspace carve(void* ws, int B, int V)
{
    const size_t per = align_up((size_t)B * (size_t)num_tiles(V) * 4, 256);
    Workspace w;
    w.cand_val = reinterpret_cast<float*>(ws);
    w.cand_idx = reinterpret_cast<int32_t*>(reinterpret_cast<unsigned char*>(ws) + per);
    return w;
}

// ---------------------------------------------------------------------------------------------
// stage-1 launchers

template <class Cfg, bool FULL = false>
fs_status launch_splitk(const Stage1Params& p, int kpw, int nw, int wgs_per_cu_override, hipStream_t st)
{
    const size_t lds = Cfg::lds_bytes(nw);
    if (nw > Cfg::kMaxWaves || lds > kLdsPerCU) return FS_ERR_UNSUPPORTED;
    auto kernel = stage1_splitk_kernel<Cfg, FULL>;
    int dev = 0;
    const int cus = current_device_cus(&dev);
    if (cus <= 0) return FS_ERR_HIP;
    static PerDevice<Cfg::kMaxWaves + 1> state;
    if (!state.attr[dev]) {
        if (allow_lds(kernel, kLdsPerCU) != hipSuccess) return FS_ERR_HIP;
        std::lock_guard<std::mutex> lk(g_mu);
        state.attr[dev] = true;
    }
    // persistent grid: as many workgroups as are resident at once (registers and LDS decide)
    if (state.resident[dev][nw] == 0) {
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, nw * kWave, lds) != hipSuccess)
            return FS_ERR_HIP;
        std::lock_guard<std::mutex> lk(g_mu);
        state.resident[dev][nw] = occ < 1 ? 1 : occ;
    }
    int per_cu = state.resident[dev][nw];
    if (wgs_per_cu_override > 0) per_cu = wgs_per_cu_override;
    int grid = cus * per_cu;
    if (grid > p.T) grid = p.T;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(nw * kWave), lds, st, p, nw, kpw);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

template <int NB>
fs_status launch_tiled(const Stage1Params& p, hipStream_t st)
{
    using Cfg = TiledCfg<NB>;
    auto kernel = stage1_tiled_kernel<NB>;
    int dev = 0;
    if (current_device_cus(&dev) <= 0) return FS_ERR_HIP;
    static PerDevice<> state;
    if (!state.attr[dev]) {
        if (allow_lds(kernel, kLdsPerCU) != hipSuccess) return FS_ERR_HIP;
        std::lock_guard<std::mutex> lk(g_mu);
        state.attr[dev] = true;
    }
    const int nbt = (p.B + Cfg::kBatchTile - 1) / Cfg::kBatchTile;
    const long long grid = (long long)p.T * nbt;
    if (grid > 0x7FFFFFFFll) return FS_ERR_SHAPE;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), Cfg::lds_bytes(), st, p);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

fs_status launch_tiled_auto(const Stage1Params& p, hipStream_t st)
{
    if (p.B <= 16) return launch_tiled<1>(p, st);
    if (p.B <= 32) return launch_tiled<2>(p, st);
    if (p.B <= 64) return launch_tiled<4>(p, st);
    if (p.B <= 128) return launch_tiled<8>(p, st);
    return launch_tiled<16>(p, st);
}

template <class Cfg, bool FULL = false, int WB = 2, bool WCODES = false, bool KRAG = false>
fs_status launch_tiled2(const Stage1Params& p, hipStream_t st)
{
    if (!KRAG && p.D % (WCODES ? 128 : 64) != 0) return FS_ERR_UNSUPPORTED;   // whole K steps only
    // LDS: two buffers of one K step; with codes in LDS a step carries two hidden sub-tiles
    constexpr size_t kLds = 2 * ((size_t)Cfg::kWBytes + (WCODES ? 2 : 1) * (size_t)Cfg::kHBytes);
    static_assert(kLds <= kLdsPerCU, "tile shape does not fit LDS");
    const int nbt = (p.B + Cfg::BT - 1) / Cfg::BT;
    const int macro_tiles = (p.V + Cfg::VT - 1) / Cfg::VT;
    const long long grid = (long long)((macro_tiles + 7) / 8) * 8 * nbt;
    if (grid > 0x7FFFFFFFll) return FS_ERR_SHAPE;
    int dev = 0;
    if (current_device_cus(&dev) <= 0) return FS_ERR_HIP;
    static PerDevice<> state;
    if (!state.attr[dev]) {
        if (allow_lds(stage1_tiled2_kernel<Cfg, true, FULL, WB, WCODES, KRAG>, kLdsPerCU) != hipSuccess) return FS_ERR_HIP;
        if (allow_lds(stage1_tiled2_kernel<Cfg, false, FULL, WB, WCODES, KRAG>, kLdsPerCU) != hipSuccess) return FS_ERR_HIP;
        std::lock_guard<std::mutex> lk(g_mu);
        state.attr[dev] = true;
    }
    if (nbt == 1)
        hipLaunchKernelGGL((stage1_tiled2_kernel<Cfg, true, FULL, WB, WCODES, KRAG>), dim3((unsigned)grid), dim3(Cfg::kThreads),
                           kLds, st, p, nbt);
    else
        hipLaunchKernelGGL((stage1_tiled2_kernel<Cfg, false, FULL, WB, WCODES, KRAG>), dim3((unsigned)grid), dim3(Cfg::kThreads),
                           kLds, st, p, nbt);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

// Tile shapes of the B > 16 kernel (vocabulary rows x batch rows per workgroup):
//   1: 128 x 32   4 waves, two workgroups per CU      5: 128 x 64   4 waves, two per CU
//   2: 256 x 64   8 waves, one per CU                 6: 512 x 32   8 waves, one per CU
//   3: 256 x 128  8 waves, one per CU                 7: 512 x 64   8 waves, one per CU
//   4: 128 x 128  4 waves, two per CU                 8: 256 x 32   4 waves, two per CU
//   9: 256 x 256  8 waves, one per CU (accumulators take 128 VGPRs)
//  10: 512 x 128  8 waves, one per CU, one register set of prefetch (128 accumulator VGPRs, 160 KB of LDS)
// Every workgroup re-reads its hidden tile once per W tile and the kernels are bound by the bytes
// that enter the CUs (about 14 bytes per clock and CU, whatever the kernel), so a workgroup of
// VT x BT takes time ~ (VT + BT) D, and a launch takes as long as its busiest CU:
//      cost(shape) = ceil(workgroups / CUs) x (VT + BT)
// (two workgroups per CU run side by side but share the CU's ingest rate, so they count like two
// in a row; see the one correction in the code).  More vocabulary rows per workgroup means fewer hidden re-reads per W byte, until the
// coarser grid leaves CUs idle in its last round.  The launcher takes the cheapest shape of the
// batch class, the finer one on ties (its epilogues overlap).  Measured, fused call in us at
// D = 4096 on 256 CUs (V: shapes by time, the rule's pick first):
//   B = 32   V = 128256: s6 161, s8 160, s1 165-173 | 152064: s8 187, s6 230 | 201088: s6 257, s8 277
//   B = 64   V = 50304: s2 74, s5 81, s7 108 | 100352: s7 132, s2 147, s5 150 | 152064: s5 190, s2 212, s7 247
//   B = 128  V = 50304: s3 84, s4 99, s10 136 | 100352: s10 149, s3 172, s4 187 | 128256: s10 182, s3 195-203, s4 217
//   B = 256  V = 32000: s3 84, s4 96, s9 124 | 128256: s9 301, s3 376 | 201088: s9 515, s4 570, s3 573
// and at D = 8192, V = 128256, B <= 16: s6 307, s8 315, s1 317 (the split-K kernel with 64 k-steps
// per wave: 325-335); B = 256: s9 562 against 699 for s3.
struct TileShape {
    int id, vt, bt;
};

int pick_tile_shape(int B, int V, int cus)
{
    static constexpr TileShape b32[] = {{1, 128, 32}, {8, 256, 32}, {6, 512, 32}};
    static constexpr TileShape b64[] = {{5, 128, 64}, {2, 256, 64}, {7, 512, 64}};
    static constexpr TileShape b128[] = {{4, 128, 128}, {3, 256, 128}, {10, 512, 128}};
    static constexpr TileShape big[] = {{4, 128, 128}, {3, 256, 128}, {9, 256, 256}};
    const TileShape* cand = B <= 32 ? b32 : B <= 64 ? b64 : B <= 128 ? b128 : big;
    const int n = 3;
    int best = cand[0].id;
    long long best_cost = -1;
    for (int i = 0; i < n; ++i) {   // fine to coarse; a coarser shape must be strictly cheaper
        const long long wgs = (long long)((V + cand[i].vt - 1) / cand[i].vt) * ((B + cand[i].bt - 1) / cand[i].bt);
        long long cost = ((wgs + cus - 1) / cus) * (cand[i].vt + cand[i].bt) * 10;
        // the 128-row shapes with 64 or 128 columns run two workgroups per CU and hide their
        // epilogues behind each other: measured about a tenth ahead of the count (D = 3584,
        // V = 152064, B = 128: 128 x 128 233 us, 256 x 128 247 us at equal count)
        if (cand[i].vt == 128 && cand[i].bt >= 64) cost = cost / 10 * 9;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = cand[i].id; }
    }
    return best;
}

// A hidden size that is not a multiple of the 64-element K step runs on the three two-per-CU
// shapes, built with the zeroing of the last step's tail; every other shape exists for whole K
// steps only.
template <bool FULL, int WB = 2>
fs_status launch_tiled2_ragged(const Stage1Params& p, hipStream_t st)
{
    if (p.B <= 32) return launch_tiled2<Tiled2Cfg<32, 4, 1, 1, 2, 256>, FULL, WB, false, true>(p, st);
    if (p.B <= 64) return launch_tiled2<Tiled2Cfg<64, 2, 2, 2, 2>, FULL, WB, false, true>(p, st);
    return launch_tiled2<Tiled2Cfg<128, 2, 2, 2, 2>, FULL, WB, false, true>(p, st);
}

// `shape` = 0 picks automatically; 1..9 forces one shape (tuning aid; honoured for whole-K-step
// hidden sizes only).
template <bool FULL>
fs_status launch_tiled2_auto(const Stage1Params& p, int shape, hipStream_t st)
{
    if (p.D % 64 != 0) return launch_tiled2_ragged<FULL>(p, st);
    if (shape == 0) {
        const int cus = current_device_cus(nullptr);
        if (cus <= 0) return FS_ERR_HIP;
        shape = pick_tile_shape(p.B, p.V, cus);
    }
    switch (shape) {
    case 1: return launch_tiled2<Tiled2Cfg<32, 4, 1, 4>, FULL>(p, st);
    case 2: return launch_tiled2<Tiled2Cfg<64, 4, 2, 2, 2, 256>, FULL>(p, st);
    case 3: return launch_tiled2<Tiled2Cfg<128, 4, 2, 1, 2, 256>, FULL>(p, st);
    case 4: return launch_tiled2<Tiled2Cfg<128, 2, 2, 2, 2>, FULL>(p, st);
    case 5: return launch_tiled2<Tiled2Cfg<64, 2, 2, 2, 2>, FULL>(p, st);
    case 6: return launch_tiled2<Tiled2Cfg<32, 8, 1, 1, 1, 512>, FULL>(p, st);
    case 7: return launch_tiled2<Tiled2Cfg<64, 4, 2, 1, 1, 512>, FULL>(p, st);
    case 8: return launch_tiled2<Tiled2Cfg<32, 4, 1, 1, 2, 256>, FULL>(p, st);
    case 9: return launch_tiled2<Tiled2Cfg<256, 4, 2, 1, 2, 256, 2>, FULL>(p, st);
    case 10: return launch_tiled2<Tiled2Cfg<128, 4, 2, 1, 2, 512, 1>, FULL>(p, st);
    default: break;
    }
    return FS_ERR_UNSUPPORTED;
}

// stage 1 with the full transform / log-normaliser epilogue: the default kernels only
fs_status launch_stage1_full(const Stage1Params& p, uint32_t flags, hipStream_t st)
{
    if (flags != FS_FLAG_NONE) return FS_ERR_UNSUPPORTED;
    const int ksteps = (p.D + 31) / 32;
    if (p.B <= 16 && ksteps <= 32 * 4) {
        const int nw = (ksteps + 31) / 32;
        return launch_splitk<SplitKCfg<32, 8, 2, 4>, true>(p, (ksteps + nw - 1) / nw, nw, 0, st);
    }
    return launch_tiled2_auto<true>(p, 0, st);
}

fs_status launch_stage1(const Stage1Params& p, uint32_t flags, hipStream_t st)
{
    if (flags & ~0x000FFF00u) return FS_ERR_UNSUPPORTED;
    const int variant = (int)((flags >> 8) & 0xFFu);
    const int wgs_override = (int)((flags >> 16) & 0xFu);
    const int ksteps = (p.D + 31) / 32;
    // split-K family: the hidden slice of a wave lives in registers, so the wave's k-range is
    // bounded (32 k-steps = 128 VGPRs, or 64 k-steps = 256 VGPRs at one wave per SIMD)
    auto splitk = [&](int which) -> fs_status {
        if (p.B > 16 || ksteps > 64 * 4) return FS_ERR_UNSUPPORTED;
        if (ksteps > 32 * 4) {
            const int nw = (ksteps + 63) / 64;
            const int kpw = (ksteps + nw - 1) / nw;
            return launch_splitk<SplitKCfg<64, 16, 2, 4>>(p, kpw, nw, wgs_override, st);
        }
        if (which == FS_VARIANT_SPLITK_C) {
            const int nw = (ksteps + 15) / 16;
            const int kpw = (ksteps + nw - 1) / nw;
            return launch_splitk<SplitKCfg<16, 8, 2, 8>>(p, kpw, nw, wgs_override, st);
        }
        const int nw = (ksteps + 31) / 32;
        const int kpw = (ksteps + nw - 1) / nw;
        switch (which) {
        case FS_VARIANT_SPLITK_B: return launch_splitk<SplitKCfg<32, 8, 2, 4>>(p, kpw, nw, wgs_override, st);
        case FS_VARIANT_SPLITK_D: return launch_splitk<SplitKCfg<32, 8, 4, 4>>(p, kpw, nw, wgs_override, st);
        case FS_VARIANT_SPLITK_E: return launch_splitk<SplitKCfg<32, 4, 2, 8>>(p, kpw, nw, wgs_override, st);
        default:                  return launch_splitk<SplitKCfg<32, 16, 2, 4>>(p, kpw, nw, wgs_override, st);
        }
    };
    switch (variant) {
    case FS_VARIANT_AUTO:
        // B <= 16: the split-K kernel while a wave's hidden slice fits 128 registers (D <= 4096);
        // for wider hidden sizes the tiled kernel is faster (D = 8192: 307 us against 325-335 us
        // for split-K with 64 k-steps per wave; D = 7168: 272 against 275-282)
        if (p.B <= 16 && ksteps <= 32 * 4) return splitk(FS_VARIANT_SPLITK_B);
        return launch_tiled2_auto<false>(p, 0, st);
    case FS_VARIANT_SPLITK_A:
    case FS_VARIANT_SPLITK_B:
    case FS_VARIANT_SPLITK_C:
    case FS_VARIANT_SPLITK_D:
    case FS_VARIANT_SPLITK_E:
        return splitk(variant);
    case FS_VARIANT_TILED:
        return launch_tiled_auto(p, st);
    case FS_VARIANT_TILED2:
        return launch_tiled2_auto<false>(p, wgs_override, st);
    default:
        return FS_ERR_UNSUPPORTED;
    }
}

// stage 1 on FP8 (E4M3) weights: one-byte W elements, otherwise the kernels of the bf16 path
fs_status launch_stage1_w8(const Stage1Params& p, uint32_t flags, hipStream_t st)
{
    if (flags & ~0x000FFF00u) return FS_ERR_UNSUPPORTED;
    const int variant = (int)((flags >> 8) & 0xFFu);
    const int wgs = (int)((flags >> 16) & 0xFu);
    const int ksteps = (p.D + 31) / 32;
    if (p.B <= 16 && ksteps <= 32 * 4) {
        if (variant == 2 || variant == 3) {
            const int nw = (ksteps + 15) / 16;
            const int kpw = (ksteps + nw - 1) / nw;
            if (variant == 2) return launch_splitk<SplitKCfg<16, 16, 1, 8, 1>>(p, kpw, nw, wgs, st);
            return launch_splitk<SplitKCfg<16, 8, 2, 8, 1>>(p, kpw, nw, wgs, st);
        }
        if (variant == 1) {
            const int nw = (ksteps + 31) / 32;
            return launch_splitk<SplitKCfg<32, 16, 2, 4, 1>>(p, (ksteps + nw - 1) / nw, nw, wgs, st);
        }
        if (variant == 0) {   // eight waves of 16 k-steps: 82 us against 90 us for four waves of 32
            const int nw = (ksteps + 15) / 16;
            return launch_splitk<SplitKCfg<16, 16, 1, 8, 1>>(p, (ksteps + nw - 1) / nw, nw, wgs, st);
        }
    }
    if (p.B <= 16 && ksteps <= 32 * 8 && (variant == 0 || variant == 1)) {
        // wide hidden sizes: eight waves of 32 k-steps, one register set of prefetch
        const int nw = (ksteps + 31) / 32;
        return launch_splitk<SplitKCfg<32, 16, 1, 8, 1>>(p, (ksteps + nw - 1) / nw, nw, wgs, st);
    }
    if (variant >= 1 && variant <= 3) return FS_ERR_UNSUPPORTED;   // a split-K form was asked for
    // larger batches and wider hidden sizes: the tiled kernel, shapes chosen as for bf16
    const int cus = current_device_cus(nullptr);
    if (cus <= 0) return FS_ERR_HIP;
    // variants 4..10 force tile shape 3..9 with the codes kept in LDS where that fits (128-element
    // K steps); variants 14..20 force shape 3..9 in the form that widens the codes when a step is
    // parked: there a K step covers only 64 bytes of a row, half a cache line, so the W prefetch
    // groups are twice as long as on the bf16 path (both halves of a line requested back to back)
    if (p.D % 64 != 0) return launch_tiled2_ragged<false, 1>(p, st);
    const int shape = variant >= 14 ? variant - 11 : variant >= 4 ? variant - 1 : pick_tile_shape(p.B, p.V, cus);
    if (variant < 14 && p.D % 128 == 0) {
        switch (shape) {
        case 1: return launch_tiled2<Tiled2Cfg<32, 4, 1, 2>, false, 1, true>(p, st);
        case 2: return launch_tiled2<Tiled2Cfg<64, 4, 2, 1, 2, 256>, false, 1, true>(p, st);
        case 3: return launch_tiled2<Tiled2Cfg<128, 4, 2, 1, 2, 256>, false, 1, true>(p, st);
        case 4: return launch_tiled2<Tiled2Cfg<128, 2, 2, 1, 2>, false, 1, true>(p, st);
        case 5: return launch_tiled2<Tiled2Cfg<64, 2, 2, 1, 2>, false, 1, true>(p, st);
        case 6: return launch_tiled2<Tiled2Cfg<32, 8, 1, 1, 1, 512>, false, 1, true>(p, st);
        case 7: return launch_tiled2<Tiled2Cfg<64, 4, 2, 1, 1, 512, 1>, false, 1, true>(p, st);
        case 8: return launch_tiled2<Tiled2Cfg<32, 4, 1, 1, 2, 256>, false, 1, true>(p, st);
        case 9:    // 256 x 256 and 512 x 128 do not fit LDS with two hidden sub-tiles per step:
        case 10:   // both run as shape 3 (B = 256: 299 us, no slower than the 256 x 256 park-time form)
            return launch_tiled2<Tiled2Cfg<128, 4, 2, 1, 2, 256>, false, 1, true>(p, st);
        default: break;
        }
    }
    switch (shape) {
    case 1: return launch_tiled2<Tiled2Cfg<32, 4, 1, 4>, false, 1>(p, st);
    case 2: return launch_tiled2<Tiled2Cfg<64, 4, 2, 2, 2, 256>, false, 1>(p, st);
    case 3: return launch_tiled2<Tiled2Cfg<128, 4, 2, 2, 2, 256>, false, 1>(p, st);
    case 4: return launch_tiled2<Tiled2Cfg<128, 2, 2, 4, 2>, false, 1>(p, st);
    case 5: return launch_tiled2<Tiled2Cfg<64, 2, 2, 4, 2>, false, 1>(p, st);
    case 6: return launch_tiled2<Tiled2Cfg<32, 8, 1, 2, 1, 512>, false, 1>(p, st);
    case 7: return launch_tiled2<Tiled2Cfg<64, 4, 2, 2, 1, 512>, false, 1>(p, st);
    case 8: return launch_tiled2<Tiled2Cfg<32, 4, 1, 2, 2, 256>, false, 1>(p, st);
    case 9: return launch_tiled2<Tiled2Cfg<256, 4, 2, 1, 2, 256, 1>, false, 1>(p, st);
    case 10: return launch_tiled2<Tiled2Cfg<128, 4, 2, 2, 2, 256>, false, 1>(p, st);   // 512 x 128 does not exist here
    default: return FS_ERR_UNSUPPORTED;
    }
}

template <int KPW, int MAXW, int PFD>
fs_status launch_w4(const Stage1Params& p, const uint8_t* scales, int nw, int wgs_override, hipStream_t st)
{
    const size_t lds = w4_lds_bytes(KPW, nw);
    if (nw > MAXW || lds > kLdsPerCU) return FS_ERR_UNSUPPORTED;
    auto kernel = stage1_w4_kernel<KPW, MAXW, PFD, false>;
    int dev = 0;
    const int cus = current_device_cus(&dev);
    if (cus <= 0) return FS_ERR_HIP;
    static PerDevice<MAXW + 1> state;
    if (!state.attr[dev]) {
        if (allow_lds(kernel, kLdsPerCU) != hipSuccess) return FS_ERR_HIP;
        std::lock_guard<std::mutex> lk(g_mu);
        state.attr[dev] = true;
    }
    if (state.resident[dev][nw] == 0) {
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, nw * kWave, lds) != hipSuccess)
            return FS_ERR_HIP;
        std::lock_guard<std::mutex> lk(g_mu);
        state.resident[dev][nw] = occ < 1 ? 1 : occ;
    }
    int per_cu = state.resident[dev][nw];
    if (wgs_override > 0) per_cu = wgs_override;
    int grid = cus * per_cu;
    if (grid > p.T) grid = p.T;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(nw * kWave), lds, st, p, scales, nw);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

fs_status launch_stage2(const float* cand_val, const int32_t* cand_idx, int B, int T,
                        int32_t* out_idx, float* out_val, hipStream_t st)
{
    hipLaunchKernelGGL(stage2_kernel, dim3(B), dim3(256), 0, st, cand_val, cand_idx, T, out_idx, out_val);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

}  // namespace

// =============================================================================================
extern "C" {

int flash_sample_num_tiles(int V) { return V > 0 ? num_tiles(V) : 0; }

int flash_sample_kernel_choice(int B, int D, int V, int compute_units)
{
    if (B <= 0 || D <= 0 || V <= 0 || (D & 7) != 0 || compute_units <= 0) return -1;
    if (B <= 16 && (D + 31) / 32 <= 32 * 4) return 0;
    if (D % 64 != 0) return B <= 32 ? 8 : B <= 64 ? 5 : 4;
    return pick_tile_shape(B, V, compute_units);
}

size_t flash_sample_workspace_bytes(int B, int V) { return workspace_bytes(B, V); }

const char* fs_status_string(fs_status s)
{
    switch (s) {
    case FS_OK: return "ok";
    case FS_ERR_NULL: return "a required pointer is NULL";
    case FS_ERR_SHAPE: return "bad shape: need B >= 0, D > 0, V > 0, D % 8 == 0, offsets in range";
    case FS_ERR_ALIGN: return "a pointer is not aligned as required";
    case FS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case FS_ERR_HIP: return "a HIP runtime call failed";
    case FS_ERR_UNSUPPORTED: return "unknown flag, or the requested kernel variant cannot run this shape";
    }
    return "unknown status";
}

fs_status flash_sample_stage1(const void* hidden, const void* W, int B, int D, int V,
                              const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                              int64_t row_offset, int32_t vocab_offset,
                              float* cand_val, int32_t* cand_idx, float* logits,
                              void* stream, uint32_t flags)
{
    fs_status s = check_problem(hidden, W, B, D, V, row_offset, vocab_offset);
    if (s != FS_OK || B == 0) return s;
    if ((cand_val == nullptr) != (cand_idx == nullptr)) return FS_ERR_NULL;
    if (!cand_val && !logits) return FS_ERR_NULL;
    if (cand_val && !temperature) return FS_ERR_NULL;
    if (logits && !aligned(logits, 16)) return FS_ERR_ALIGN;
    if (!aligned(cand_val, 4) || !aligned(cand_idx, 4) || !aligned(temperature, 4) ||
        !aligned(row_seeds, 8))
        return FS_ERR_ALIGN;
    Stage1Params p;
    p.H = static_cast<const uint16_t*>(hidden);
    p.W = static_cast<const uint16_t*>(W);
    p.B = B; p.D = D; p.V = V; p.T = num_tiles(V);
    p.tau = temperature;
    p.seed = seed; p.row_seeds = row_seeds;
    p.row_offset = row_offset; p.vocab_offset = vocab_offset;
    p.cand_val = cand_val; p.cand_idx = cand_idx; p.logits = logits;
    p.bias = nullptr; p.allowed = nullptr; p.mask_stride = 0; p.lse_max = nullptr; p.lse_sum = nullptr;
    return launch_stage1(p, flags, static_cast<hipStream_t>(stream));
}

fs_status flash_sample_stage2(const float* cand_val, const int32_t* cand_idx, int B, int T,
                              int32_t* out_idx, float* out_val, void* stream)
{
    if (B < 0 || T <= 0) return FS_ERR_SHAPE;
    if (B == 0) return FS_OK;
    if (!cand_val || !cand_idx || !out_idx || !out_val) return FS_ERR_NULL;
    if (!aligned(cand_val, 4) || !aligned(cand_idx, 4) || !aligned(out_idx, 4) || !aligned(out_val, 4))
        return FS_ERR_ALIGN;
    return launch_stage2(cand_val, cand_idx, B, T, out_idx, out_val, static_cast<hipStream_t>(stream));
}

fs_status flash_sample_ex(const void* hidden, const void* W, int B, int D, int V,
                          const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                          int64_t row_offset, int32_t vocab_offset,
                          int32_t* out_idx, float* out_val,
                          void* workspace, size_t workspace_bytes_given, void* stream, uint32_t flags)
{
    fs_status s = check_problem(hidden, W, B, D, V, row_offset, vocab_offset);
    if (s != FS_OK || B == 0) return s;
    if (!temperature || !out_idx || !out_val) return FS_ERR_NULL;
    if (!aligned(out_idx, 4) || !aligned(out_val, 4)) return FS_ERR_ALIGN;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < workspace_bytes(B, V))
        return FS_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, B, V);
    s = flash_sample_stage1(hidden, W, B, D, V, temperature, seed, row_seeds, row_offset, vocab_offset,
                            ws.cand_val, ws.cand_idx, nullptr, stream, flags);
    if (s != FS_OK) return s;
    return launch_stage2(ws.cand_val, ws.cand_idx, B, num_tiles(V), out_idx, out_val,
                         static_cast<hipStream_t>(stream));
}

fs_status flash_sample(const void* hidden, const void* W, int B, int D, int V,
                       const float* temperature, uint64_t seed, int32_t* out_idx, float* out_val)
{
    fs_status s = check_problem(hidden, W, B, D, V, 0, 0);
    if (s != FS_OK || B == 0) return s;
    if (!temperature || !out_idx || !out_val) return FS_ERR_NULL;
    int dev = 0;
    if (current_device_cus(&dev) <= 0) return FS_ERR_HIP;
    const size_t need = workspace_bytes(B, V);
    void* ws = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        DeviceInfo& d = g_dev[dev];
        if (d.ws_bytes < need) {
            // the old buffer may still be in use by an earlier call on the null stream
            if (d.ws) {
                if (hipStreamSynchronize(nullptr) != hipSuccess) return FS_ERR_HIP;
                (void)hipFree(d.ws);
                d.ws = nullptr;
                d.ws_bytes = 0;
            }
            if (hipMalloc(&d.ws, need) != hipSuccess) { d.ws = nullptr; return FS_ERR_HIP; }
            d.ws_bytes = need;
        }
        ws = d.ws;
    }
    return flash_sample_ex(hidden, W, B, D, V, temperature, seed, nullptr, 0, 0, out_idx, out_val,
                           ws, need, nullptr, FS_FLAG_NONE);
}

size_t flash_sample_full_workspace_bytes(int B, int V) { return 2 * workspace_bytes(B, V); }

fs_status flash_sample_full(const void* hidden, const void* W, int B, int D, int V,
                            const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                            int64_t row_offset, int32_t vocab_offset,
                            const float* bias, const uint32_t* allowed, int64_t mask_stride_words,
                            int32_t* out_idx, float* out_val, float* out_lse,
                            void* workspace, size_t workspace_bytes_given, void* stream, uint32_t flags)
{
    fs_status s = check_problem(hidden, W, B, D, V, row_offset, vocab_offset);
    if (s != FS_OK || B == 0) return s;
    if (!temperature || !out_idx || !out_val) return FS_ERR_NULL;
    if (allowed && mask_stride_words != 0 && mask_stride_words < (int64_t)((V + 31) / 32)) return FS_ERR_SHAPE;
    if (mask_stride_words < 0) return FS_ERR_SHAPE;
    if (!aligned(out_idx, 4) || !aligned(out_val, 4) || !aligned(out_lse, 4) || !aligned(temperature, 4) ||
        !aligned(row_seeds, 8) || !aligned(bias, 16) || !aligned(allowed, 4))
        return FS_ERR_ALIGN;
    const size_t half = workspace_bytes(B, V);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < 2 * half) return FS_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, B, V);
    const Workspace ws2 = carve(static_cast<unsigned char*>(workspace) + half, B, V);
    Stage1Params p;
    p.H = static_cast<const uint16_t*>(hidden);
    p.W = static_cast<const uint16_t*>(W);
    p.B = B; p.D = D; p.V = V; p.T = num_tiles(V);
    p.tau = temperature;
    p.seed = seed; p.row_seeds = row_seeds;
    p.row_offset = row_offset; p.vocab_offset = vocab_offset;
    p.cand_val = ws.cand_val; p.cand_idx = ws.cand_idx; p.logits = nullptr;
    p.bias = bias; p.allowed = allowed; p.mask_stride = mask_stride_words;
    p.lse_max = out_lse ? ws2.cand_val : nullptr;
    p.lse_sum = out_lse ? reinterpret_cast<float*>(ws2.cand_idx) : nullptr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    s = launch_stage1_full(p, flags, st);
    if (s != FS_OK) return s;
    s = launch_stage2(ws.cand_val, ws.cand_idx, B, p.T, out_idx, out_val, st);
    if (s != FS_OK || !out_lse) return s;
    hipLaunchKernelGGL(lse_reduce_kernel, dim3(B), dim3(256), 0, st, p.lse_max, p.lse_sum, p.T, out_lse);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

int flash_sample_num_groups(int V, int group_tiles)
{
    if (V <= 0 || group_tiles <= 0) return 0;
    return (num_tiles(V) + group_tiles - 1) / group_tiles;
}

namespace {

fs_status launch_group_choose(const GroupInputs& in, int B, int m, int mode, uint64_t seed,
                              const uint64_t* row_seeds, int64_t row_offset, int64_t group_offset,
                              int32_t* out_idx, float* out_lse, float* group_log_mass,
                              int32_t* group_sample, hipStream_t st)
{
    if (mode == FS_GROUPED_PARALLEL)
        hipLaunchKernelGGL(group_choose_kernel<0>, dim3(B), dim3(256), 0, st, in, m, seed, row_seeds,
                           row_offset, (uint32_t)group_offset, out_idx, out_lse, group_log_mass, group_sample);
    else
        hipLaunchKernelGGL(group_choose_kernel<1>, dim3(B), dim3(256), 0, st, in, m, seed, row_seeds,
                           row_offset, (uint32_t)group_offset, out_idx, out_lse, group_log_mass, group_sample);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

}  // namespace

fs_status flash_sample_grouped(const void* hidden, const void* W, int B, int D, int V,
                               const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                               int64_t row_offset, int32_t vocab_offset,
                               const float* bias, const uint32_t* allowed, int64_t mask_stride_words,
                               int group_tiles, int mode,
                               int32_t* out_idx, float* out_lse,
                               float* group_log_mass, int32_t* group_sample,
                               void* workspace, size_t workspace_bytes_given, void* stream, uint32_t flags)
{
    fs_status s = check_problem(hidden, W, B, D, V, row_offset, vocab_offset);
    if (s != FS_OK) return s;
    if (group_tiles < 1 || (mode != FS_GROUPED_PARALLEL && mode != FS_GROUPED_ONLINE)) return FS_ERR_SHAPE;
    const int64_t group_ids = (int64_t)kVocabTile * (int64_t)group_tiles;
    if ((int64_t)vocab_offset % group_ids != 0) return FS_ERR_SHAPE;
    if (B == 0) return FS_OK;
    if (!temperature || !out_idx) return FS_ERR_NULL;
    if (allowed && mask_stride_words != 0 && mask_stride_words < (int64_t)((V + 31) / 32)) return FS_ERR_SHAPE;
    if (mask_stride_words < 0) return FS_ERR_SHAPE;
    if (!aligned(out_idx, 4) || !aligned(out_lse, 4) || !aligned(temperature, 4) || !aligned(row_seeds, 8) ||
        !aligned(bias, 16) || !aligned(allowed, 4) || !aligned(group_log_mass, 4) || !aligned(group_sample, 4))
        return FS_ERR_ALIGN;
    const size_t half = workspace_bytes(B, V);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < 2 * half) return FS_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, B, V);
    const Workspace ws2 = carve(static_cast<unsigned char*>(workspace) + half, B, V);
    Stage1Params p;
    p.H = static_cast<const uint16_t*>(hidden);
    p.W = static_cast<const uint16_t*>(W);
    p.B = B; p.D = D; p.V = V; p.T = num_tiles(V);
    p.tau = temperature;
    p.seed = seed; p.row_seeds = row_seeds;
    p.row_offset = row_offset; p.vocab_offset = vocab_offset;
    p.cand_val = ws.cand_val; p.cand_idx = ws.cand_idx; p.logits = nullptr;
    p.bias = bias; p.allowed = allowed; p.mask_stride = mask_stride_words;
    p.lse_max = ws2.cand_val;
    p.lse_sum = reinterpret_cast<float*>(ws2.cand_idx);
    hipStream_t st = static_cast<hipStream_t>(stream);
    s = launch_stage1_full(p, flags, st);
    if (s != FS_OK) return s;
    GroupInputs in;
    in.cand_val = ws.cand_val; in.cand_idx = ws.cand_idx;
    in.lse_max = p.lse_max; in.lse_sum = p.lse_sum;
    in.T = p.T; in.gt = group_tiles;
    const int m = (p.T + group_tiles - 1) / group_tiles;
    return launch_group_choose(in, B, m, mode, seed, row_seeds, row_offset, (int64_t)vocab_offset / group_ids,
                               out_idx, out_lse, group_log_mass, group_sample, st);
}

fs_status flash_group_choose(const float* group_log_mass, const int32_t* group_sample, int B, int m,
                             int mode, uint64_t seed, const uint64_t* row_seeds, int64_t row_offset,
                             int64_t group_offset, int32_t* out_idx, float* out_lse, void* stream)
{
    if (B < 0 || m <= 0 || row_offset < 0 || group_offset < 0 || group_offset + (int64_t)m > 0xFFFFFFFFll)
        return FS_ERR_SHAPE;
    if (mode != FS_GROUPED_PARALLEL && mode != FS_GROUPED_ONLINE) return FS_ERR_SHAPE;
    if (B == 0) return FS_OK;
    if (!group_log_mass || !group_sample || !out_idx) return FS_ERR_NULL;
    if (!aligned(group_log_mass, 4) || !aligned(group_sample, 4) || !aligned(out_idx, 4) ||
        !aligned(out_lse, 4) || !aligned(row_seeds, 8))
        return FS_ERR_ALIGN;
    GroupInputs in;
    in.cand_val = nullptr; in.cand_idx = group_sample;
    in.lse_max = group_log_mass; in.lse_sum = nullptr;
    in.T = m; in.gt = 1;
    return launch_group_choose(in, B, m, mode, seed, row_seeds, row_offset, group_offset, out_idx, out_lse,
                               nullptr, nullptr, static_cast<hipStream_t>(stream));
}

fs_status flash_sample_w8(const void* hidden, const void* W8, const float* w_scale, int B, int D, int V,
                          const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                          int64_t row_offset, int32_t vocab_offset, float* logits,
                          int32_t* out_idx, float* out_val,
                          void* workspace, size_t workspace_bytes_given, void* stream, uint32_t flags)
{
    fs_status s = check_problem(hidden, W8, B, D, V, row_offset, vocab_offset);
    if (s != FS_OK) return s;
    if ((D & 15) != 0) return FS_ERR_SHAPE;
    if (B == 0) return FS_OK;
    if (!temperature || !out_idx || !out_val) return FS_ERR_NULL;
    if (!aligned(out_idx, 4) || !aligned(out_val, 4) || !aligned(temperature, 4) || !aligned(row_seeds, 8) ||
        !aligned(w_scale, 16) || !aligned(logits, 16))
        return FS_ERR_ALIGN;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < workspace_bytes(B, V))
        return FS_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, B, V);
    Stage1Params p;
    p.H = static_cast<const uint16_t*>(hidden);
    p.W = static_cast<const uint16_t*>(W8);
    p.B = B; p.D = D; p.V = V; p.T = num_tiles(V);
    p.tau = temperature;
    p.seed = seed; p.row_seeds = row_seeds;
    p.row_offset = row_offset; p.vocab_offset = vocab_offset;
    p.cand_val = ws.cand_val; p.cand_idx = ws.cand_idx; p.logits = logits;
    p.bias = nullptr; p.allowed = nullptr; p.mask_stride = 0;
    p.lse_max = nullptr; p.lse_sum = nullptr;
    p.w_scale = w_scale;
    hipStream_t st = static_cast<hipStream_t>(stream);
    s = launch_stage1_w8(p, flags, st);
    if (s != FS_OK) return s;
    return launch_stage2(ws.cand_val, ws.cand_idx, B, p.T, out_idx, out_val, st);
}

fs_status flash_sample_w4(const void* hidden, const void* W4, const void* w_scales, int B, int D, int V,
                          const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                          int64_t row_offset, int32_t vocab_offset, float* logits,
                          int32_t* out_idx, float* out_val,
                          void* workspace, size_t workspace_bytes_given, void* stream, uint32_t flags)
{
    fs_status s = check_problem(hidden, W4, B, D, V, row_offset, vocab_offset);
    if (s != FS_OK) return s;
    if (flags & ~0x000FFF00u) return FS_ERR_UNSUPPORTED;
    if (B == 0) return FS_OK;
    if (B > 16 || (D & 511) != 0 || D > 8192) return FS_ERR_UNSUPPORTED;
    if (!w_scales || !temperature || !out_idx || !out_val) return FS_ERR_NULL;
    if (!aligned(w_scales, 16) || !aligned(out_idx, 4) || !aligned(out_val, 4) || !aligned(temperature, 4) ||
        !aligned(row_seeds, 8) || !aligned(logits, 16))
        return FS_ERR_ALIGN;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < workspace_bytes(B, V))
        return FS_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, B, V);
    Stage1Params p;
    p.H = static_cast<const uint16_t*>(hidden);
    p.W = static_cast<const uint16_t*>(W4);
    p.B = B; p.D = D; p.V = V; p.T = num_tiles(V);
    p.tau = temperature;
    p.seed = seed; p.row_seeds = row_seeds;
    p.row_offset = row_offset; p.vocab_offset = vocab_offset;
    p.cand_val = ws.cand_val; p.cand_idx = ws.cand_idx; p.logits = logits;
    p.bias = nullptr; p.allowed = nullptr; p.mask_stride = 0;
    p.lse_max = nullptr; p.lse_sum = nullptr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t* sc = static_cast<const uint8_t*>(w_scales);
    const int variant = (int)((flags >> 8) & 0xFFu);
    const int wgs = (int)((flags >> 16) & 0xFu);
    if (D <= 4096 && variant < 8) {   // eight waves of 16 K steps
        switch (variant) {
        case 0: case 2: s = launch_w4<16, 8, 2>(p, sc, D / 512, wgs, st); break;
        case 1: s = launch_w4<16, 8, 1>(p, sc, D / 512, wgs, st); break;
        case 4: s = launch_w4<16, 8, 4>(p, sc, D / 512, wgs, st); break;
        default: return FS_ERR_UNSUPPORTED;
        }
    } else {                          // 32 K steps per wave (D % 1024 == 0 then)
        if ((D & 1023) != 0) return FS_ERR_UNSUPPORTED;
        switch (variant) {
        case 0: case 1: case 9: s = launch_w4<32, 8, 1>(p, sc, D / 1024, wgs, st); break;
        case 2: case 10: s = launch_w4<32, 8, 2>(p, sc, D / 1024, wgs, st); break;
        default: return FS_ERR_UNSUPPORTED;
        }
    }
    if (s != FS_OK) return s;
    return launch_stage2(ws.cand_val, ws.cand_idx, B, p.T, out_idx, out_val, st);
}

fs_status flash_sample_mxfp4_decode(const void* codes, const uint8_t* scales, int n8, float* out, void* stream)
{
    if (n8 < 0) return FS_ERR_SHAPE;
    if (n8 == 0) return FS_OK;
    if (!codes || !scales || !out) return FS_ERR_NULL;
    if (!aligned(codes, 4) || !aligned(out, 4)) return FS_ERR_ALIGN;
    hipLaunchKernelGGL(mxfp4_decode_kernel, dim3((n8 + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint32_t*>(codes), scales, n8, out);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

fs_status flash_sample_e4m3_decode(const uint8_t* codes, int n, float* out, void* stream)
{
    if (n < 0 || (n & 7) != 0) return FS_ERR_SHAPE;
    if (n == 0) return FS_OK;
    if (!codes || !out) return FS_ERR_NULL;
    if (!aligned(codes, 8) || !aligned(out, 4)) return FS_ERR_ALIGN;
    hipLaunchKernelGGL(e4m3_decode_kernel, dim3((n / 8 + 255) / 256), dim3(256), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<const uint32_t*>(codes), n / 8, out);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

fs_status flash_lm_head_logits(const void* hidden, const void* W, int B, int D, int V,
                               float* logits, void* stream, uint32_t flags)
{
    if (B > 0 && !logits) return FS_ERR_NULL;
    return flash_sample_stage1(hidden, W, B, D, V, nullptr, 0, nullptr, 0, 0, nullptr, nullptr, logits,
                               stream, flags);
}

fs_status flash_gumbel_argmax_logits(const float* logits, int B, int V, const float* temperature,
                                     uint64_t seed, const uint64_t* row_seeds, int64_t row_offset,
                                     int32_t vocab_offset, int32_t* out_idx, float* out_val,
                                     void* workspace, size_t workspace_bytes_given, void* stream)
{
    if (B < 0 || V <= 0 || row_offset < 0 || vocab_offset < 0 ||
        (int64_t)vocab_offset + (int64_t)V > (int64_t)INT32_MAX || B > 65535)
        return FS_ERR_SHAPE;
    if (B == 0) return FS_OK;
    if (!logits || !temperature || !out_idx || !out_val) return FS_ERR_NULL;
    if (!aligned(logits, 16) || !aligned(out_idx, 4) || !aligned(out_val, 4) || !aligned(row_seeds, 8))
        return FS_ERR_ALIGN;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < workspace_bytes(B, V))
        return FS_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, B, V);   // [B, TC] fits inside [B, T]: TC <= T
    const int TC = num_chunks(V);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(gumbel_argmax_logits_kernel, dim3(TC, B), dim3(256), 0, st, logits, V, TC,
                       temperature, seed, row_seeds, row_offset, vocab_offset, ws.cand_val, ws.cand_idx);
    if (hipGetLastError() != hipSuccess) return FS_ERR_HIP;
    return launch_stage2(ws.cand_val, ws.cand_idx, B, TC, out_idx, out_val, st);
}

fs_status flash_sample_unfused(const void* hidden, const void* W, int B, int D, int V,
                               const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                               int64_t row_offset, int32_t vocab_offset, float* logits,
                               int32_t* out_idx, float* out_val,
                               void* workspace, size_t workspace_bytes_given, void* stream, uint32_t flags)
{
    fs_status s = check_problem(hidden, W, B, D, V, row_offset, vocab_offset);
    if (s != FS_OK || B == 0) return s;
    if (!logits || !temperature || !out_idx || !out_val) return FS_ERR_NULL;
    if (B > 65535) return FS_ERR_SHAPE;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < workspace_bytes(B, V))
        return FS_ERR_WORKSPACE;
    s = flash_lm_head_logits(hidden, W, B, D, V, logits, stream, flags);
    if (s != FS_OK) return s;
    return flash_gumbel_argmax_logits(logits, B, V, temperature, seed, row_seeds, row_offset, vocab_offset,
                                      out_idx, out_val, workspace, workspace_bytes_given, stream);
}

fs_status flash_sample_noise(uint64_t seed, int64_t row, int32_t v0, int n, float* g_out, void* stream)
{
    if (n < 0 || v0 < 0 || row < 0 || (int64_t)v0 + n > (int64_t)INT32_MAX) return FS_ERR_SHAPE;
    if (n == 0) return FS_OK;
    if (!g_out) return FS_ERR_NULL;
    if (!aligned(g_out, 4)) return FS_ERR_ALIGN;
    hipLaunchKernelGGL(noise_kernel, dim3((n + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       seed, (uint32_t)(uint64_t)row, v0, n, g_out);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

fs_status flash_sample_gumbel_transform(const uint32_t* words, int n, float* g_out, void* stream)
{
    if (n < 0) return FS_ERR_SHAPE;
    if (n == 0) return FS_OK;
    if (!words || !g_out) return FS_ERR_NULL;
    if (!aligned(words, 4) || !aligned(g_out, 4)) return FS_ERR_ALIGN;
    hipLaunchKernelGGL(gumbel_transform_kernel, dim3((n + 255) / 256), dim3(256), 0,
                       static_cast<hipStream_t>(stream), words, n, g_out);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

fs_status flash_sample_stream_probe(void* dst, const void* src, size_t bytes, uint32_t* sink, void* stream)
{
    if ((bytes & 15) != 0) return FS_ERR_SHAPE;
    if (bytes == 0) return FS_OK;
    if (!src) return FS_ERR_NULL;
    if (!aligned(src, 16) || !aligned(dst, 16) || !aligned(sink, 4)) return FS_ERR_ALIGN;
    const int cus = current_device_cus(nullptr);
    if (cus <= 0) return FS_ERR_HIP;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    const size_t cap = (size_t)cus * 8;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(stream_probe_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<uint4*>(dst),
                       static_cast<const uint4*>(src), n16, sink);
    return hipGetLastError() == hipSuccess ? FS_OK : FS_ERR_HIP;
}

}  // extern "C"
