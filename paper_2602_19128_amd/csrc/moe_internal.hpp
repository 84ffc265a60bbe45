// Internal declarations shared by the HIP translation units of the MoE library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe.h"

namespace moe {

constexpr int kWave = 64;            // gfx950 wavefront width
constexpr int kMaxExperts = 512;
constexpr int kMaxTopK = 64;
constexpr int kQBlock = 128;         // edge of an fp8 scale block

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- bf16 helpers (bf16 = upper half of an IEEE binary32) ------------------
__device__ inline float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even; NaN stays NaN
__device__ inline uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// Experts whose weights a call holds (local-expert mode), and the first of them.
__host__ __device__ inline int local_experts(const moe_config &c) { return c.num_local_experts > 0 ? c.num_local_experts : c.E; }

// ---- launch helpers ----------------------------------------------------------
void set_last_hip_error(hipError_t e);
inline int check_launch()
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_last_hip_error(e); return MOE_ERR_HIP; }
    return MOE_OK;
}

// ---- per-step launchers (arguments already validated by the C ABI layer) -----
size_t route_workspace_bytes(const moe_config &c);
int launch_route(const moe_config &c, const void *x, const float *x_scale, const float *router_w,
                 const float *bias, int32_t *ids, float *w, void *ws, hipStream_t s);
int launch_quantize_act(const moe_config &c, const void *x, void *xq, float *x_scale, hipStream_t s);
int launch_permute(const moe_config &c, int tile_rows, int max_tiles, const int32_t *ids,
                   int32_t *offsets, int32_t *sorted_pair, int32_t *inv, moe_tile *tiles,
                   int32_t *sched, hipStream_t s);
int launch_gemm_swiglu(const moe_config &c, int tile_rows, int max_tiles, const void *x,
                       const float *x_scale, const void *w1, const float *w1_scale,
                       const int32_t *sorted_pair, const moe_tile *tiles, const int32_t *sched,
                       void *act, float *act_scale, hipStream_t s);
int launch_gemm_down(const moe_config &c, int tile_rows, int max_tiles, const void *act,
                     const float *act_scale, const void *w2, const float *w2_scale,
                     const moe_tile *tiles, const int32_t *sched, void *y, hipStream_t s);
int launch_combine(const moe_config &c, const void *y, const float *w, const int32_t *inv, void *out,
                   hipStream_t s);

}  // namespace moe
