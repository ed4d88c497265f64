// Translation unit of the LDS-tiled stage-1 kernel, bf16 weights, full-transform epilogue (bias,
// allowed-id mask, online log-sum-exp).
#include "fs_launch_tiled2.hpp"

namespace fs {

fs_status launch_stage1_tiled_full(const Stage1Params& p, int shape, hipStream_t st)
{
    return launch_tiled2_bf16<true>(p, shape, st);
}

}  // namespace fs
