// Translation unit of the LDS-tiled stage-1 kernel, bf16 weights, plain epilogue (1/tau scaling).
#include "fs_launch_tiled2.hpp"

namespace fs {

fs_status launch_stage1_tiled(const Stage1Params& p, int shape, hipStream_t st)
{
    return launch_tiled2_bf16<false>(p, shape, st);
}

}  // namespace fs
