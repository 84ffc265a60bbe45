// Grouped expert GEMM, down projection, bf16: the kernel instantiations of moe_gemm_kernel.hpp
// for this operand type (one translation unit per type, so that they compile side by side).
#include "moe_gemm_kernel.hpp"

namespace moe {

int launch_gemm_down_bf16(int tile_rows, const GemmArgs &g, const moe_tile *tiles, const int32_t *sched, int max_tiles,
                       int est_tiles, hipStream_t s)
{
    return launch_by_tile_rows<false, false>(tile_rows, g, tiles, sched, max_tiles, est_tiles, s);
}

}  // namespace moe
