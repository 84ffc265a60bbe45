// Host side of the grouped expert GEMMs (paper Sec. 4.5 "Expert FFN computation"): the per-type
// dispatch.  The operand description and the choices that depend on the problem statement alone
// are in moe_internal.hpp (gateup_args, down_args, gemm_width); the kernels live in
// moe_gemm_kernel.hpp and are instantiated per operand type in moe_gemm_{gateup,down}_{bf16,fp8}.hip.
#include "moe_internal.hpp"

namespace moe {

int launch_gemm_swiglu(const moe_config &c, int tile_rows, int max_tiles, const void *x,
                       const float *x_scale, const void *w1, const float *w1_scale, const int32_t *sorted_pair,
                       const moe_tile *tiles, const int32_t *sched, void *act, float *act_scale, hipStream_t s)
{
    const GemmArgs g = gateup_args(c, x, x_scale, w1, w1_scale, sorted_pair, act, act_scale);
    if (c.dtype == MOE_DTYPE_FP8_E4M3)
        return launch_gemm_gateup_fp8(tile_rows, g, tiles, sched, max_tiles, expected_tiles(c), s);
    return launch_gemm_gateup_bf16(tile_rows, g, tiles, sched, max_tiles, expected_tiles(c), s);
}

int launch_gemm_down(const moe_config &c, int tile_rows, int max_tiles, int k_split, const void *act,
                     const float *act_scale, const void *w2, const float *w2_scale, const moe_tile *tiles,
                     const int32_t *sched, void *y, hipStream_t s)
{
    const GemmArgs g = down_args(c, act, act_scale, w2, w2_scale, y, k_split);
    if (c.dtype == MOE_DTYPE_FP8_E4M3)
        return launch_gemm_down_fp8(tile_rows, g, tiles, sched, max_tiles, expected_tiles(c), s);
    return launch_gemm_down_bf16(tile_rows, g, tiles, sched, max_tiles, expected_tiles(c), s);
}

}  // namespace moe
