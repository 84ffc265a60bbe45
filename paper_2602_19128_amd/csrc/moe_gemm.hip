// Host side of the grouped expert GEMMs (paper Sec. 4.5 "Expert FFN computation"): operand
// description and the choices that depend on the problem statement only.  The kernels live in
// moe_gemm_kernel.hpp and are instantiated per operand type in moe_gemm_{gateup,down}_{bf16,fp8}.hip.
#include "moe_internal.hpp"

namespace moe {
namespace {

// Tiles a balanced router is expected to produce (host-side estimate used only to pick the
// workgroup width; the kernels read the real count from device memory).
int expected_tiles(const moe_config &c)
{
    const long pairs = (long)c.T * c.top_k;
    const int el = local_experts(c);
    return (int)(pairs < el ? pairs : el);
}

// Number of distinct K-loop starting points for rows of `row_bytes` bytes: every K step its own
// when the row stride is a multiple of 4 KiB (measured: such strides lose 10-15% of the stream rate
// when all workgroups walk K in step; other strides gain nothing and only spread the token rows
// over more of L2).
int k_groups_for(int row_bytes)
{
    return row_bytes % 4096 == 0 ? row_bytes / GM_STEP_BYTES : 1;
}

// An output that does not fit the L2s (8 x 4 MiB) anyway is written with non-temporal stores:
// cached stores of such a stream push the token rows the workgroups share out of L2 (measured
// -4..6 % on the gate/up GEMM); a small output stays cached for the kernel that reads it next.
int nt_output(size_t bytes) { return bytes > (size_t)32 << 20 ? 1 : 0; }

}  // namespace

int launch_gemm_swiglu(const moe_config &c, int tile_rows, int max_tiles, const void *x,
                       const float *x_scale, const void *w1, const float *w1_scale, const int32_t *sorted_pair,
                       const moe_tile *tiles, const int32_t *sched, void *act, float *act_scale, hipStream_t s)
{
    GemmArgs g{static_cast<const unsigned char *>(x), x_scale, static_cast<const unsigned char *>(w1), w1_scale,
               sorted_pair, static_cast<unsigned char *>(act), act_scale, c.H, c.I, c.top_k,
               k_groups_for(c.H * (c.dtype == MOE_DTYPE_FP8_E4M3 ? 1 : 2)),
               nt_output((size_t)c.T * c.top_k * c.I * (c.dtype == MOE_DTYPE_FP8_E4M3 ? 1 : 2))};
    if (c.dtype == MOE_DTYPE_FP8_E4M3) {
        return launch_gemm_gateup_fp8(tile_rows, g, tiles, sched, max_tiles, expected_tiles(c), s);
    }
    return launch_gemm_gateup_bf16(tile_rows, g, tiles, sched, max_tiles, expected_tiles(c), s);
}

int launch_gemm_down(const moe_config &c, int tile_rows, int max_tiles, const void *act, const float *act_scale,
                     const void *w2, const float *w2_scale, const moe_tile *tiles, const int32_t *sched, void *y,
                     hipStream_t s)
{
    GemmArgs g{static_cast<const unsigned char *>(act), act_scale, static_cast<const unsigned char *>(w2), w2_scale,
               nullptr, static_cast<unsigned char *>(y), nullptr, c.I, c.H, c.top_k,
               k_groups_for(c.I * (c.dtype == MOE_DTYPE_FP8_E4M3 ? 1 : 2)),
               nt_output((size_t)c.T * c.top_k * c.H * 2)};
    if (c.dtype == MOE_DTYPE_FP8_E4M3) {
        return launch_gemm_down_fp8(tile_rows, g, tiles, sched, max_tiles, expected_tiles(c), s);
    }
    return launch_gemm_down_bf16(tile_rows, g, tiles, sched, max_tiles, expected_tiles(c), s);
}

}  // namespace moe
