// Translation unit of the stage-1 kernels on MXFP4 weights: the split-K form of the decode regime
// (B <= 16) and the tiled form with the codes kept in LDS (larger batches, other hidden sizes).
#include "fs_launch_tiled2.hpp"
#include "fs_stage1_w4.hpp"

namespace fs {

namespace {

template <int KPW, int MAXW, int PFD>
fs_status launch_w4(const Stage1Params& p, const uint8_t* scales, int nw, int wgs_override, hipStream_t st)
{
    const size_t lds = w4_lds_bytes(KPW, nw);
    if (nw > MAXW || lds > kLdsPerCU) return FS_ERR_UNSUPPORTED;
    auto kernel = stage1_w4_kernel<KPW, MAXW, PFD, false>;
    int dev = 0, cus = 0;
    const fs_status ds = current_device(&dev, &cus);
    if (ds != FS_OK) return ds;
    static PerDevice<MAXW + 1> state;
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
    if (wgs_override > 0) per_cu = wgs_override;
    int grid = cus * per_cu;
    if (grid > p.T) grid = p.T;
    return launch(kernel, dim3(grid), dim3(nw * kWave), lds, st, p, scales, nw);
}

}  // namespace

// B <= 16: split-K.  D % 512 == 0 and D <= 4096: eight waves of 16 K steps, two row-tiles in flight;
// D % 1024 == 0 and D <= 8192: 32 K steps per wave, one row-tile in flight.
// Otherwise (D % 256 == 0): the tiled kernel, 256 x 32 tiles up to 32 rows, 256 x 64 above (more rows
// per workgroup do not fit LDS beside four hidden sub-tiles per step; larger batches run as several
// batch tiles that share each W tile through L2).
fs_status launch_stage1_w4(const Stage1Params& p, const uint8_t* scales, int wgs_per_cu, hipStream_t st)
{
    const bool splitk = p.B <= 16 && (p.D & 511) == 0 && (p.D <= 4096 || (p.D <= 8192 && (p.D & 1023) == 0));
    if (splitk) {
        if (p.D <= 4096) return launch_w4<16, 8, 2>(p, scales, p.D / 512, wgs_per_cu, st);
        return launch_w4<32, 8, 1>(p, scales, p.D / 1024, wgs_per_cu, st);
    }
    if ((p.D & 255) != 0) return FS_ERR_UNSUPPORTED;
    Stage1Params q = p;
    q.w4_scales = scales;
    if (p.B <= 32) return launch_tiled2<Tiled2Cfg<32, 4, 1, 1, 2, 256>, false, 1, true, false, true, false, true>(q, st);
    return launch_tiled2<Tiled2Cfg<64, 4, 2, 1, 2, 256>, false, 1, true, false, true, false, true>(q, st);
}

fs_status launch_mxfp4_decode(const uint32_t* codes, const uint8_t* scales, int n8, float* out, hipStream_t st)
{
    return launch(mxfp4_decode_kernel, dim3((n8 + 255) / 256), dim3(256), 0, st, codes, scales, n8, out);
}

}  // namespace fs
