// Internal declarations shared by the HIP translation units of the MoE library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "moe.h"

namespace moe {

constexpr int kWave = 64;            // gfx950 wavefront width
constexpr int kMaxExperts = 512;
constexpr int kMaxTopK = 64;
constexpr int kQBlock = 128;         // edge of an fp8 scale block
constexpr int kMaxScaleBlocks = 128; // fp8: scale blocks along a contraction (H or I up to 16384)

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

// One-time set-up per device (e.g. a kernel's dynamic-LDS limit), safe to reach from several host
// threads: the set-up must be idempotent, since two threads may both run it before either has
// marked it done; a failed set-up is tried again by the next call.
constexpr int kMaxDevices = 64;
struct DeviceOnce {
    std::atomic<int> done[kMaxDevices];
    DeviceOnce() { for (auto &d : done) d.store(0, std::memory_order_relaxed); }
    template <class F> int run(F &&setup)
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return setup();
        if (done[dev].load(std::memory_order_acquire)) return MOE_OK;
        const int rc = setup();
        if (rc == MOE_OK) done[dev].store(1, std::memory_order_release);
        return rc;
    }
};

// Raises a kernel's dynamic-LDS limit, once per device.
inline int set_dynamic_lds(DeviceOnce &once, const void *kern, int bytes)
{
    return once.run([&]() {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) { set_last_hip_error(e); return MOE_ERR_HIP; }
        return MOE_OK;
    });
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
// (k_split: see down_k_split; y then receives the partial sums)
int launch_gemm_down(const moe_config &c, int tile_rows, int max_tiles, int k_split, const void *act,
                     const float *act_scale, const void *w2, const float *w2_scale,
                     const moe_tile *tiles, const int32_t *sched, void *y, hipStream_t s);
// (k_split = 2: y holds the fp32 partial sums of a K-split down projection, [2][P,H])
int launch_combine(const moe_config &c, const void *y, const float *w, const int32_t *inv, void *out,
                   hipStream_t s, int k_split = 1);

// ---- single-launch forward (moe_fused.hip) -----------------------------------------------------
void set_single_launch(int enable);
int single_launch_mode(const moe_config &c, int tile_rows);
int single_launch_timeouts(unsigned *out);
int launch_fused(const moe_config &c, int tile_rows, int max_tiles, const void *x, const float *router_w,
                 const float *bias, void *route_ws, int32_t *ids, float *w, int32_t *offsets, int32_t *sorted_pair,
                 int32_t *inv, moe_tile *tiles, int32_t *sched, const void *w1, const void *w2, void *act, void *y,
                 void *out, hipStream_t s);

// ---- grouped GEMMs: operand description shared by the host side and the kernel instantiations ----
constexpr int GM_STEP_BYTES = 128;        // bytes of every row consumed per K step

struct GemmArgs {
    const unsigned char *A;       // gate/up: x [T,K]; down: act [P,K]
    const float *a_scale;         // fp8: [T or P, K/128]
    const unsigned char *W;       // [E, w_rows, K]
    const float *w_scale;         // fp8: [E, w_rows/128, K/128]
    const int32_t *sorted_pair;   // gate/up only
    unsigned char *out;           // gate/up: act [P,n_out] (bf16 / fp8); down: y [P,n_out] bf16
    float *out_scale;             // fp8 gate/up: act_scale [P, n_out/128]
    int K, n_out, top_k;
    int k_groups;                 // distinct K-loop starting points spread over the workgroups (1 = all start at 0)
    int nt_out;                   // write the output with non-temporal stores (it is too large to stay in L2 anyway)
    int k_split;                  // down only: 1, or 2 = K is cut in halves, each with items of its own, and `out`
                                  // holds the halves' fp32 partial sums, [2][P,n_out], split_stride bytes apart
    size_t split_stride;
};

// Workgroup width of a grouped GEMM launch, from the problem statement alone (est_tiles: tiles a
// balanced router is expected to produce; the kernels read the real count from device memory).
//   wide    8 wavefronts, two 16-row weight blocks each: 128 gate/up or 256 down columns per workgroup.
//   narrow  4 wavefronts (half the columns) when the wide ones would leave compute units without
//           work; not for the fp8 gate/up GEMM, whose epilogue re-quantises a whole 128-column
//           block per workgroup.
//   wide4   down projection of low tiles (32 or 64 rows): four weight blocks per wavefront, 512
//           columns per workgroup.  Its K loop is short (16 steps for fp8 with I = 2048), so a
//           workgroup's fixed costs are a third of its life, and the accumulators of a low tile
//           leave the registers for it (fp8 prefill: down GEMM -4 %).  Not for 16-row tiles, where
//           two workgroups per compute unit already overlap those costs (decode shape: +0.5 %).
enum GemmWidth { GEMM_NARROW = 0, GEMM_WIDE = 1, GEMM_WIDE4 = 2 };
constexpr int kComputeUnits = 256;
inline GemmWidth gemm_width(int mb_max, bool swiglu, bool fp8, int n_out, int est_tiles)
{
    const int wide_cols = swiglu ? 128 : 256;
    if (!swiglu && (mb_max == 2 || mb_max == 4) && (long)est_tiles * ceil_div(n_out, 512) >= 4 * kComputeUnits)
        return GEMM_WIDE4;
    if (!(fp8 && swiglu) && (long)est_tiles * ceil_div(n_out, wide_cols) < 2 * kComputeUnits) return GEMM_NARROW;
    return GEMM_WIDE;
}
// Tiles a balanced router is expected to produce.
inline int expected_tiles(const moe_config &c)
{
    const long pairs = (long)c.T * c.top_k;
    const int el = local_experts(c);
    return (int)(pairs < el ? pairs : el);
}

// Down projection of a layer with few experts and tall tiles (Mixtral-shaped prefill): the narrow
// workgroups such a launch would take own 128 output columns each and pull more token bytes than
// weight bytes through the compute unit's memory pipeline, which then runs at its own limit (about
// 50 GB/s) instead of the chip's.  Cutting K in two instead gives as many items of 256 columns: half
// the token bytes per weight byte (measured 192 -> 163 us at 512 Mixtral tokens).  The halves' fp32
// partial sums go to the workspace and the combine adds them, first half first, before it rounds a
// row to bf16, so the result has one fixed order.  bf16 only; the K loop must stay long.
inline int down_k_split(const moe_config &c, int tile_rows)
{
    if (c.dtype != MOE_DTYPE_BF16 || tile_rows < 128) return 1;
    if (gemm_width(tile_rows / 16, false, false, c.H, expected_tiles(c)) != GEMM_NARROW) return 1;
    const int nk = c.I * 2 / 128;                            // K steps of the whole reduction
    return (nk >= 64 && nk % 2 == 0) ? 2 : 1;
}

// Number of distinct K-loop starting points for rows of `row_bytes` bytes: every K step its own
// when the row stride is a multiple of 4 KiB (measured: such strides lose 10-15% of the stream rate
// when all workgroups walk K in step; other strides gain nothing and only spread the token rows
// over more of L2).
inline int k_groups_for(int row_bytes) { return row_bytes % 4096 == 0 ? row_bytes / GM_STEP_BYTES : 1; }

// An output that does not fit the L2s (8 x 4 MiB) anyway is written with non-temporal stores:
// cached stores of such a stream push the token rows the workgroups share out of L2 (measured
// -4..6 % on the gate/up GEMM); a small output stays cached for the kernel that reads it next.
inline int nt_output(size_t bytes) { return bytes > (size_t)32 << 20 ? 1 : 0; }

inline GemmArgs gateup_args(const moe_config &c, const void *x, const float *x_scale, const void *w1,
                            const float *w1_scale, const int32_t *sorted_pair, void *act, float *act_scale)
{
    const int es = c.dtype == MOE_DTYPE_FP8_E4M3 ? 1 : 2;
    return GemmArgs{static_cast<const unsigned char *>(x), x_scale, static_cast<const unsigned char *>(w1), w1_scale,
                    sorted_pair, static_cast<unsigned char *>(act), act_scale, c.H, c.I, c.top_k,
                    k_groups_for(c.H * es), nt_output((size_t)c.T * c.top_k * c.I * es), 1, 0};
}

// y: the bf16 output [P,H]; with k_split = 2 the fp32 partial sums [2][P,H] instead.
inline GemmArgs down_args(const moe_config &c, const void *act, const float *act_scale, const void *w2,
                          const float *w2_scale, void *y, int k_split)
{
    const int es = c.dtype == MOE_DTYPE_FP8_E4M3 ? 1 : 2;
    const size_t out_bytes = (size_t)c.T * c.top_k * c.H * (k_split > 1 ? 4 : 2);
    return GemmArgs{static_cast<const unsigned char *>(act), act_scale, static_cast<const unsigned char *>(w2), w2_scale,
                    nullptr, static_cast<unsigned char *>(y), nullptr, c.I, c.H, c.top_k,
                    k_groups_for(c.I * es), nt_output(out_bytes * k_split), k_split, out_bytes};
}

// kernel instantiations per operand type (moe_gemm_{gateup,down}_{bf16,fp8}.hip)
int launch_gemm_gateup_bf16(int tile_rows, const GemmArgs &g, const moe_tile *tiles, const int32_t *sched,
                            int max_tiles, int est_tiles, hipStream_t s);
int launch_gemm_gateup_fp8(int tile_rows, const GemmArgs &g, const moe_tile *tiles, const int32_t *sched,
                           int max_tiles, int est_tiles, hipStream_t s);
int launch_gemm_down_bf16(int tile_rows, const GemmArgs &g, const moe_tile *tiles, const int32_t *sched,
                          int max_tiles, int est_tiles, hipStream_t s);
int launch_gemm_down_fp8(int tile_rows, const GemmArgs &g, const moe_tile *tiles, const int32_t *sched,
                         int max_tiles, int est_tiles, hipStream_t s);

}  // namespace moe
