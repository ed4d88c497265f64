// Host side of the C ABI declared in include/flash_sample.h: argument checks, kernel choice,
// launches.  Every step of the method runs in the kernels; nothing here touches the data.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <mutex>

#include "flash_sample.h"
#include "flash_sample_measure.h"
#include "fs_aux_kernels.hpp"
#include "fs_common.hpp"
#include "fs_grouped_kernels.hpp"
#include "fs_host.hpp"

namespace fs {

namespace {
struct DeviceInfo {
    std::atomic<int> cus{0};   // 0 = not queried yet
};
DeviceInfo g_dev[kMaxDevices];
}  // namespace

fs_status current_device(int* dev_out, int* cus_out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return FS_ERR_HIP;
    if (dev >= kMaxDevices) return FS_ERR_DEVICE;
    int cus = g_dev[dev].cus.load(std::memory_order_acquire);
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            return FS_ERR_HIP;
        g_dev[dev].cus.store(cus, std::memory_order_release);
    }
    if (dev_out) *dev_out = dev;
    if (cus_out) *cus_out = cus;
    return FS_OK;
}

// Every workgroup of the tiled kernel re-reads its hidden tile once per W tile and the kernels are
// bound by the bytes that enter the CUs (about 14 bytes per clock and CU, whatever the kernel), so
// a workgroup of VT x BT takes time ~ (VT + BT) D, and a launch takes as long as its busiest CU:
//      cost(shape) = ceil(workgroups / CUs) x (VT + BT)
// (two workgroups per CU run side by side but share the CU's ingest rate, so they count like two
// in a row; see the one correction in the code).  More vocabulary rows per workgroup means fewer
// hidden re-reads per W byte, until the coarser grid leaves CUs idle in its last round.  The
// launcher takes the cheapest shape of the batch class, the finer one on ties (its epilogues
// overlap).  Measured, fused call in us at D = 4096 on 256 CUs (V: shapes by time, the rule's pick
// first; shape numbers as in fs_launch_tiled2.hpp):
//   B = 32   V = 128256: s6 161, s8 160, s1 165-173 | 152064: s8 187, s6 230 | 201088: s6 257, s8 277
//   B = 64   V = 50304: s2 74, s5 81, s7 108 | 100352: s7 132, s2 147, s5 150 | 152064: s5 190, s2 212, s7 247
//   B = 128  V = 50304: s3 84, s4 99, s10 136 | 100352: s10 149, s3 172, s4 187 | 128256: s10 182, s3 195-203, s4 217
//   B = 256  V = 32000: s3 84, s4 96 | 128256: s12 259, s3 346 | D = 8192: s12 488, s3 648
// (s12 is the 256 x 256 kernel with direct global -> LDS loads; the 256 x 256 shape of the tiled
// kernel it replaced ran at 301 and 566) and at D = 8192, V = 128256, B <= 16: s6 307, s8 315, s1 317.
int pick_tile_shape(int B, int D, int V, int cus)
{
    if (B > 128) {
        // The kernel with direct global -> LDS loads, 256 x 256 or 256 x 128 tiles.  A round of 256 x 256
        // workgroups takes 123 us and one of 256 x 128 workgroups 73 us at D = 4096 (the ratio holds at
        // D = 8192); the launch lasts rounds x that.  256 x 128 wins where the last 256-row batch tile
        // would be at most half full (B = 320, 384: 10-20 % ahead) and where 256-row tiles leave CUs
        // without work (V = 32000 at B <= 256); checked against a sweep over V in {32000 .. 256000} x
        // B in {160, 256, 320, 384, 512, 768}.  On near-ties the larger tile (fewer bytes into the CUs).
        const long long mt = (V + 255) / 256;
        const long long r256 = (mt * ((B + 255) / 256) + cus - 1) / cus;
        const long long r128 = (mt * ((B + 127) / 128) + cus - 1) / cus;
        return r128 * 73 * 100 < r256 * 123 * 97 ? 13 : 12;
    }
    struct TileShape { int id, vt, bt; };
    static constexpr TileShape b32[] = {{1, 128, 32}, {8, 256, 32}, {6, 512, 32}};
    static constexpr TileShape b64[] = {{5, 128, 64}, {2, 256, 64}, {7, 512, 64}};
    static constexpr TileShape b128[] = {{4, 128, 128}, {3, 256, 128}, {10, 512, 128}};
    const TileShape* cand = B <= 32 ? b32 : B <= 64 ? b64 : b128;
    int best = cand[0].id;
    long long best_cost = -1;
    for (int i = 0; i < 3; ++i) {   // fine to coarse; a coarser shape must be strictly cheaper
        const long long wgs = (long long)((V + cand[i].vt - 1) / cand[i].vt) * ((B + cand[i].bt - 1) / cand[i].bt);
        long long cost = ((wgs + cus - 1) / cus) * (cand[i].vt + cand[i].bt) * 10;
        // the 128-row shapes with 64 or 128 columns run two workgroups per CU and hide their
        // epilogues behind each other: measured about a tenth ahead of the count (D = 3584,
        // V = 152064, B = 128: 128 x 128 233 us, 256 x 128 247 us at equal count)
        if (cand[i].vt == 128 && cand[i].bt >= 64) cost = cost / 10 * 9;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = cand[i].id; }
    }
    // wide hidden sizes at 64 < B <= 128: the kernel with direct global -> LDS loads in its 256 x 128
    // form is 2-4 % ahead of the 512 x 128 shape (D = 8192: 340 vs 354 us, D = 7168: 322 vs 328 us)
    if (best == 10 && D >= 6144) best = 13;
    return best;
}

}  // namespace fs

namespace {

using namespace fs;

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

constexpr uint32_t kVariantMask = 0x0000FF00u, kTuneMask = 0x000F0000u;
constexpr uint32_t kEpiMask = FS_FLAG_GREEDY | FS_FLAG_EXACT_LOG;

// bits of `flags` that go to the kernels' epilogue
inline uint32_t epi_bits(uint32_t flags) { return flags & kEpiMask; }

// bf16 weights.  The split-K kernel while a wave's hidden slice fits 128 registers (B <= 16,
// D <= 4096); for wider hidden sizes and larger batches the tiled kernel (at D = 8192, B <= 16
// it runs at 307 us against 325-335 us for a split-K form with 64 k-steps per wave).
fs_status launch_stage1(const Stage1Params& p, bool full, uint32_t flags, hipStream_t st)
{
    if (flags & ~(kVariantMask | kTuneMask | kEpiMask)) return FS_ERR_UNSUPPORTED;
    const int variant = (int)((flags & kVariantMask) >> 8);
    const int tune = (int)((flags & kTuneMask) >> 16);
    const bool splitk_ok = p.B <= 16 && (p.D + 31) / 32 <= 32 * 4;
    switch (variant) {
    case FS_VARIANT_AUTO:
        if (splitk_ok) return launch_stage1_splitk(p, full, 0, st);
        return full ? launch_stage1_tiled_full(p, 0, st) : launch_stage1_tiled(p, 0, st);
    case FS_VARIANT_SPLITK:
        if (!splitk_ok) return FS_ERR_UNSUPPORTED;
        return launch_stage1_splitk(p, full, tune, st);
    case FS_VARIANT_TILED2:
        return full ? launch_stage1_tiled_full(p, tune, st) : launch_stage1_tiled(p, tune, st);
    default:
        return FS_ERR_UNSUPPORTED;
    }
}

fs_status launch_stage2(const float* cand_val, const int32_t* cand_idx, int B, int T,
                        int32_t* out_idx, float* out_val, hipStream_t st)
{
    return launch(stage2_kernel, dim3(B), dim3(256), 0, st, cand_val, cand_idx, T, out_idx, out_val);
}

Stage1Params make_params(const void* hidden, const void* W, int B, int D, int V, const float* temperature,
                         uint64_t seed, const uint64_t* row_seeds, int64_t row_offset, int32_t vocab_offset,
                         uint32_t flags)
{
    Stage1Params p;
    p.H = static_cast<const uint16_t*>(hidden);
    p.W = static_cast<const uint16_t*>(W);
    p.B = B; p.D = D; p.V = V; p.T = num_tiles(V);
    p.tau = temperature;
    p.seed = seed; p.row_seeds = row_seeds;
    p.row_offset = row_offset; p.vocab_offset = vocab_offset;
    p.cand_val = nullptr; p.cand_idx = nullptr; p.logits = nullptr;
    p.bias = nullptr; p.allowed = nullptr; p.mask_stride = 0; p.lse_max = nullptr; p.lse_sum = nullptr;
    p.w_scale = nullptr;
    p.epi_flags = epi_bits(flags);
    return p;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Scratch of flash_sample_static: the candidate buffer of Alg. 1 in a file-scope device array, for
// callers that cannot allocate.  In host code the array's name is only a stand-in; its device
// address is looked up once per device (each device holds its own copy) and used from then on.
static __device__ __align__(256) unsigned char scratch[FS_STATIC_SCRATCH_BYTES];

namespace {

std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (first call on a device: one symbol lookup).
fs_status static_scratch(void** out)
{
    int dev = 0;
    const fs_status ds = current_device(&dev, nullptr);
    if (ds != FS_OK) return ds;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return FS_ERR_HIP;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return FS_OK;
}

// workspace cache of the plain entry point, one per device; g_ws_mu is held across the launch so
// that a concurrent call cannot free the buffer between another thread's lookup and its launch
struct WsCache {
    void* ws = nullptr;
    size_t bytes = 0;
};
WsCache g_ws[kMaxDevices];
std::mutex g_ws_mu;

}  // namespace

// =============================================================================================
extern "C" {

int flash_sample_num_tiles(int V) { return V > 0 ? num_tiles(V) : 0; }

size_t flash_sample_workspace_bytes(int B, int V) { return workspace_bytes(B, V); }

const char* fs_status_string(fs_status s)
{
    switch (s) {
    case FS_OK: return "ok";
    case FS_ERR_NULL: return "a required pointer is NULL";
    case FS_ERR_SHAPE: return "bad shape: need B >= 0, D > 0, V > 0, D % 8 == 0, offsets and sizes in range";
    case FS_ERR_ALIGN: return "a pointer is not aligned as required";
    case FS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case FS_ERR_HIP: return "a HIP runtime call failed";
    case FS_ERR_UNSUPPORTED: return "unknown flag, or the requested kernel variant cannot run this shape";
    case FS_ERR_DEVICE: return "the current device ordinal is beyond the library's per-device tables (64 devices)";
    case FS_ERR_SCRATCH_LIMIT: return "the problem needs more than the built-in scratch of flash_sample_static "
                                      "(8 B T bytes > FS_STATIC_SCRATCH_BYTES): use flash_sample_ex with a workspace";
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
    Stage1Params p = make_params(hidden, W, B, D, V, temperature, seed, row_seeds, row_offset, vocab_offset, flags);
    p.cand_val = cand_val; p.cand_idx = cand_idx; p.logits = logits;
    return launch_stage1(p, false, flags, static_cast<hipStream_t>(stream));
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
    s = current_device(&dev, nullptr);
    if (s != FS_OK) return s;
    const size_t need = workspace_bytes(B, V);
    std::lock_guard<std::mutex> lk(g_ws_mu);   // held until the kernels are enqueued
    WsCache& c = g_ws[dev];
    if (c.bytes < need) {
        if (c.ws) {   // the old buffer may still be in use by an earlier call on the null stream
            if (hipStreamSynchronize(nullptr) != hipSuccess) return FS_ERR_HIP;
            (void)hipFree(c.ws);
            c.ws = nullptr;
            c.bytes = 0;
        }
        if (hipMalloc(&c.ws, need) != hipSuccess) { c.ws = nullptr; return FS_ERR_HIP; }
        c.bytes = need;
    }
    return flash_sample_ex(hidden, W, B, D, V, temperature, seed, nullptr, 0, 0, out_idx, out_val,
                           c.ws, need, nullptr, FS_FLAG_NONE);
}

fs_status flash_sample_static(const void* hidden, const void* W, int B, int D, int V,
                              const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                              int64_t row_offset, int32_t vocab_offset,
                              int32_t* out_idx, float* out_val, void* stream, uint32_t flags)
{
    fs_status s = check_problem(hidden, W, B, D, V, row_offset, vocab_offset);
    if (s != FS_OK || B == 0) return s;
    if (workspace_bytes(B, V) > (size_t)FS_STATIC_SCRATCH_BYTES) return FS_ERR_SCRATCH_LIMIT;
    void* ptr = nullptr;
    s = static_scratch(&ptr);
    if (s != FS_OK) return s;
    // every (row, tile) entry of the candidate buffer is written by stage 1 before stage 2 reads
    // it, so nothing in the scratch has to start at zero
    return flash_sample_ex(hidden, W, B, D, V, temperature, seed, row_seeds, row_offset, vocab_offset,
                           out_idx, out_val, ptr, (size_t)FS_STATIC_SCRATCH_BYTES, stream, flags);
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
    if (flags & ~kEpiMask) return FS_ERR_UNSUPPORTED;   // the automatic kernel choice only
    const size_t half = workspace_bytes(B, V);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < 2 * half) return FS_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, B, V);
    const Workspace ws2 = carve(static_cast<unsigned char*>(workspace) + half, B, V);
    Stage1Params p = make_params(hidden, W, B, D, V, temperature, seed, row_seeds, row_offset, vocab_offset, flags);
    p.cand_val = ws.cand_val; p.cand_idx = ws.cand_idx;
    p.bias = bias; p.allowed = allowed; p.mask_stride = mask_stride_words;
    p.lse_max = out_lse ? ws2.cand_val : nullptr;
    p.lse_sum = out_lse ? reinterpret_cast<float*>(ws2.cand_idx) : nullptr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    s = launch_stage1(p, true, flags, st);
    if (s != FS_OK) return s;
    s = launch_stage2(ws.cand_val, ws.cand_idx, B, p.T, out_idx, out_val, st);
    if (s != FS_OK || !out_lse) return s;
    return launch(lse_reduce_kernel, dim3(B), dim3(256), 0, st, p.lse_max, p.lse_sum, p.T, out_lse);
}

int flash_sample_num_groups(int V, int group_tiles)
{
    if (V <= 0 || group_tiles <= 0) return 0;
    return (num_tiles(V) + group_tiles - 1) / group_tiles;
}

}  // extern "C"

namespace {

fs_status launch_group_choose(const GroupInputs& in, int B, int m, int mode, uint64_t seed,
                              const uint64_t* row_seeds, int64_t row_offset, int64_t group_offset,
                              int32_t* out_idx, float* out_lse, float* group_log_mass,
                              int32_t* group_sample, hipStream_t st)
{
    if (mode == FS_GROUPED_PARALLEL)
        return launch(group_choose_kernel<0>, dim3(B), dim3(256), 0, st, in, m, seed, row_seeds,
                      row_offset, (uint32_t)group_offset, out_idx, out_lse, group_log_mass, group_sample);
    return launch(group_choose_kernel<1>, dim3(B), dim3(256), 0, st, in, m, seed, row_seeds,
                  row_offset, (uint32_t)group_offset, out_idx, out_lse, group_log_mass, group_sample);
}

}  // namespace

extern "C" {

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
    if (flags != FS_FLAG_NONE) return FS_ERR_UNSUPPORTED;
    const size_t half = workspace_bytes(B, V);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < 2 * half) return FS_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, B, V);
    const Workspace ws2 = carve(static_cast<unsigned char*>(workspace) + half, B, V);
    Stage1Params p = make_params(hidden, W, B, D, V, temperature, seed, row_seeds, row_offset, vocab_offset, flags);
    p.cand_val = ws.cand_val; p.cand_idx = ws.cand_idx;
    p.bias = bias; p.allowed = allowed; p.mask_stride = mask_stride_words;
    p.lse_max = ws2.cand_val;
    p.lse_sum = reinterpret_cast<float*>(ws2.cand_idx);
    hipStream_t st = static_cast<hipStream_t>(stream);
    s = launch_stage1(p, true, flags, st);
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
    if (flags & ~(kVariantMask | kTuneMask | kEpiMask)) return FS_ERR_UNSUPPORTED;
    if (B == 0) return FS_OK;
    if (!temperature || !out_idx || !out_val) return FS_ERR_NULL;
    if (!aligned(out_idx, 4) || !aligned(out_val, 4) || !aligned(temperature, 4) || !aligned(row_seeds, 8) ||
        !aligned(w_scale, 16) || !aligned(logits, 16))
        return FS_ERR_ALIGN;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < workspace_bytes(B, V))
        return FS_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, B, V);
    Stage1Params p = make_params(hidden, W8, B, D, V, temperature, seed, row_seeds, row_offset, vocab_offset, flags);
    p.cand_val = ws.cand_val; p.cand_idx = ws.cand_idx; p.logits = logits;
    p.w_scale = w_scale;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int variant = (int)((flags & kVariantMask) >> 8);
    if (variant != FS_VARIANT_AUTO && variant != FS_VARIANT_SPLITK && variant != FS_VARIANT_TILED2)
        return FS_ERR_UNSUPPORTED;
    s = launch_stage1_w8(p, variant, (int)((flags & kTuneMask) >> 16), st);
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
    if (flags & ~(kTuneMask | kEpiMask)) return FS_ERR_UNSUPPORTED;
    if (B == 0) return FS_OK;
    if ((D & 255) != 0) return FS_ERR_UNSUPPORTED;          // whole blocks of 32 and whole K steps of the tiled form
    if (!w_scales || !temperature || !out_idx || !out_val) return FS_ERR_NULL;
    if (!aligned(w_scales, 16) || !aligned(out_idx, 4) || !aligned(out_val, 4) || !aligned(temperature, 4) ||
        !aligned(row_seeds, 8) || !aligned(logits, 16))
        return FS_ERR_ALIGN;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < workspace_bytes(B, V))
        return FS_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, B, V);
    Stage1Params p = make_params(hidden, W4, B, D, V, temperature, seed, row_seeds, row_offset, vocab_offset, flags);
    p.cand_val = ws.cand_val; p.cand_idx = ws.cand_idx; p.logits = logits;
    hipStream_t st = static_cast<hipStream_t>(stream);
    s = launch_stage1_w4(p, static_cast<const uint8_t*>(w_scales), (int)((flags & kTuneMask) >> 16), st);
    if (s != FS_OK) return s;
    return launch_stage2(ws.cand_val, ws.cand_idx, B, p.T, out_idx, out_val, st);
}

fs_status flash_sample_mxfp4_decode(const void* codes, const uint8_t* scales, int n8, float* out, void* stream)
{
    if (n8 < 0) return FS_ERR_SHAPE;
    if (n8 == 0) return FS_OK;
    if (!codes || !scales || !out) return FS_ERR_NULL;
    if (!aligned(codes, 4) || !aligned(out, 4)) return FS_ERR_ALIGN;
    return launch_mxfp4_decode(static_cast<const uint32_t*>(codes), scales, n8, out, static_cast<hipStream_t>(stream));
}

fs_status flash_sample_e4m3_decode(const uint8_t* codes, int n, float* out, void* stream)
{
    if (n < 0 || (n & 7) != 0) return FS_ERR_SHAPE;
    if (n == 0) return FS_OK;
    if (!codes || !out) return FS_ERR_NULL;
    if (!aligned(codes, 8) || !aligned(out, 4)) return FS_ERR_ALIGN;
    return launch(e4m3_decode_kernel, dim3((n / 8 + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                  reinterpret_cast<const uint32_t*>(codes), n / 8, out);
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
    fs_status s = launch(gumbel_argmax_logits_kernel, dim3(TC, B), dim3(256), 0, st, logits, V, TC,
                         temperature, seed, row_seeds, row_offset, vocab_offset, ws.cand_val, ws.cand_idx);
    if (s != FS_OK) return s;
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
    return launch(noise_kernel, dim3((n + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                  seed, (uint32_t)(uint64_t)row, v0, n, g_out);
}

fs_status flash_sample_gumbel_transform(const uint32_t* words, int n, float* g_out, void* stream, uint32_t flags)
{
    if (n < 0) return FS_ERR_SHAPE;
    if (flags & ~(uint32_t)FS_FLAG_EXACT_LOG) return FS_ERR_UNSUPPORTED;
    if (n == 0) return FS_OK;
    if (!words || !g_out) return FS_ERR_NULL;
    if (!aligned(words, 4) || !aligned(g_out, 4)) return FS_ERR_ALIGN;
    return launch(gumbel_transform_kernel, dim3((n + 255) / 256), dim3(256), 0,
                  static_cast<hipStream_t>(stream), words, n, g_out, flags);
}

// ---- truncated supports

namespace {

struct TopkWs {
    uint64_t* cand;        // [B, T * m]   stage-1 candidates (fused path only)
    uint64_t* buf[2];      // intermediate selection levels
    size_t bytes;
};

// candidates a tile emits in the fused form
int topk_tile_m(int k, int B)
{
    const int m = B <= 32 ? kTopkTileM : kTopkTileMLargeB;
    return k < m ? k : m;
}

TopkWs carve_topk(void* ws, int B, int V, int k, bool fused)
{
    const int n_cand = fused ? num_tiles(V) * topk_tile_m(k, B) : V;
    const TopkPlan pl = topk_plan(B, n_cand, k);
    const size_t cand = fused ? align_up((size_t)B * (size_t)n_cand * 8, 256) : 0;
    const size_t b0 = align_up(pl.buf_words[0] * 8, 256), b1 = align_up(pl.buf_words[1] * 8, 256);
    unsigned char* q = static_cast<unsigned char*>(ws);
    TopkWs w;
    w.cand = reinterpret_cast<uint64_t*>(q);
    w.buf[0] = reinterpret_cast<uint64_t*>(q + cand);
    w.buf[1] = reinterpret_cast<uint64_t*>(q + cand + b0);
    w.bytes = cand + b0 + b1;
    return w;
}

fs_status check_topk(int B, int k, float top_p, int mode, uint32_t flags, const void* temperature, const void* out_idx,
                     const void* out_val, const void* topk_val, const void* topk_idx, const void* n_kept,
                     const void* row_seeds, uint32_t tune_bits = 0u)
{
    if (k < 1 || k > FS_TOPK_MAX_K) return FS_ERR_SHAPE;
    if (mode != FS_TOPK_TRUNCATE && mode != FS_TOPK_GUMBEL) return FS_ERR_SHAPE;
    if (!(top_p > 0.0f) || top_p > 1.0f) return FS_ERR_SHAPE;                 // also rejects NaN
    if (mode == FS_TOPK_GUMBEL && top_p != 1.0f) return FS_ERR_SHAPE;         // the candidates are the draw: nothing to cut
    if (flags & ~((uint32_t)FS_FLAG_EXACT_LOG | tune_bits)) return FS_ERR_UNSUPPORTED;
    if (B == 0) return FS_OK;
    if (!temperature || !out_idx || !out_val) return FS_ERR_NULL;
    if (!aligned(temperature, 4) || !aligned(out_idx, 4) || !aligned(out_val, 4) || !aligned(topk_val, 4) ||
        !aligned(topk_idx, 4) || !aligned(n_kept, 4) || !aligned(row_seeds, 8))
        return FS_ERR_ALIGN;
    return FS_OK;
}

}  // namespace

size_t flash_sample_topk_workspace_bytes(int B, int V, int k)
{
    if (B <= 0 || V <= 0 || k < 1 || k > FS_TOPK_MAX_K) return 0;
    const size_t fused = carve_topk(nullptr, B, V, k, true).bytes, unfused = carve_topk(nullptr, B, V, k, false).bytes;
    return fused > unfused ? fused : unfused;
}

fs_status flash_sample_topk(const void* hidden, const void* W, int B, int D, int V,
                            const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                            int64_t row_offset, int32_t vocab_offset, int k, float top_p, int mode,
                            int32_t* out_idx, float* out_val, float* topk_val, int32_t* topk_idx, int32_t* n_kept,
                            void* workspace, size_t workspace_bytes_given, void* stream, uint32_t flags)
{
    fs_status s = check_problem(hidden, W, B, D, V, row_offset, vocab_offset);
    if (s != FS_OK) return s;
    s = check_topk(B, k, top_p, mode, flags, temperature, out_idx, out_val, topk_val, topk_idx, n_kept, row_seeds, kTuneMask);
    if (s != FS_OK || B == 0) return s;
    if (D % 64 != 0) return FS_ERR_UNSUPPORTED;      // the per-tile top-k epilogue exists for whole K steps only
    const TopkWs ws = carve_topk(workspace, B, V, k, true);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < ws.bytes) return FS_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int m = topk_tile_m(k, B);
    Stage1Params p = make_params(hidden, W, B, D, V, temperature, seed, row_seeds, row_offset, vocab_offset, flags);
    p.topk_out = ws.cand; p.topk_k = m; p.topk_mode = mode;
    s = launch_stage1_topk(p, (int)((flags & kTuneMask) >> 16), st);
    if (s != FS_OK) return s;
    const int n_cand = p.T * m;
    const TopkFinish fin = {top_p, mode, seed, row_seeds, row_offset, epi_bits(flags), out_idx, out_val, topk_val, topk_idx, n_kept};
    // more than m wanted: the last selection level checks for tiles that hold more winners than they emitted
    const TopkCrowd crowd = {ws.cand, p.T, m, vocab_offset, p.H, p.W, D, V, temperature};
    return launch_topk_reduce(ws.cand, nullptr, B, n_cand, (int64_t)n_cand, 0, k, ws.buf[0], ws.buf[1], fin, k > m ? &crowd : nullptr, st);
}

fs_status flash_sample_topk_unfused(const void* hidden, const void* W, int B, int D, int V,
                                    const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                                    int64_t row_offset, int32_t vocab_offset, int k, float top_p, int mode,
                                    float* logits, int32_t* out_idx, float* out_val, float* topk_val,
                                    int32_t* topk_idx, int32_t* n_kept,
                                    void* workspace, size_t workspace_bytes_given, void* stream, uint32_t flags)
{
    fs_status s = check_problem(hidden, W, B, D, V, row_offset, vocab_offset);
    if (s != FS_OK) return s;
    s = check_topk(B, k, top_p, mode, flags, temperature, out_idx, out_val, topk_val, topk_idx, n_kept, row_seeds);
    if (s != FS_OK || B == 0) return s;
    if (!logits) return FS_ERR_NULL;
    if (!aligned(logits, 16)) return FS_ERR_ALIGN;
    if (B > 65535) return FS_ERR_SHAPE;
    const TopkWs ws = carve_topk(workspace, B, V, k, false);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes_given < ws.bytes) return FS_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    s = flash_lm_head_logits(hidden, W, B, D, V, logits, stream, FS_FLAG_NONE);
    if (s != FS_OK) return s;
    const TopkKeys keys = {temperature, seed, row_seeds, row_offset, mode, epi_bits(flags)};
    const TopkFinish fin = {top_p, mode, seed, row_seeds, row_offset, epi_bits(flags), out_idx, out_val, topk_val, topk_idx, n_kept};
    return launch_topk_reduce(logits, &keys, B, V, (int64_t)V, vocab_offset, k, ws.buf[0], ws.buf[1], fin, nullptr, st);
}

// ---- include/flash_sample_measure.h

int flash_measure_kernel_choice(int B, int D, int V, int compute_units)
{
    if (B <= 0 || D <= 0 || V <= 0 || (D & 7) != 0 || compute_units <= 0) return -1;
    if (B <= 16 && (D + 31) / 32 <= 32 * 4) return 0;
    if (D % 64 != 0) return B <= 32 ? 8 : B <= 64 ? 5 : 4;
    return pick_tile_shape(B, D, V, compute_units);
}

fs_status flash_measure_stream_probe(void* dst, const void* src, size_t bytes, uint32_t* sink, void* stream)
{
    if ((bytes & 15) != 0) return FS_ERR_SHAPE;
    if (bytes == 0) return FS_OK;
    if (!src) return FS_ERR_NULL;
    if (!aligned(src, 16) || !aligned(dst, 16) || !aligned(sink, 4)) return FS_ERR_ALIGN;
    int cus = 0;
    const fs_status ds = current_device(nullptr, &cus);
    if (ds != FS_OK) return ds;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    const size_t cap = (size_t)cus * 8;
    if (blocks > cap) blocks = cap;
    return launch(stream_probe_kernel, dim3((unsigned)blocks), dim3(256), 0,
                  static_cast<hipStream_t>(stream), static_cast<uint4*>(dst),
                  static_cast<const uint4*>(src), n16, sink);
}

}  // extern "C"
