// Sort-scatter kernel (paper Sec. 4.5: tokens reordered by expert into contiguous memory); the
// algorithm is described with its device code in moe_permute_device.hpp.
#include "moe_permute_device.hpp"

namespace moe {
namespace {

constexpr int PM_THREADS = 1024;

__global__ __launch_bounds__(PM_THREADS) void permute_kernel(const int32_t *__restrict__ ids, int P, int E,
                                                             int e_first, int tile_rows, int max_tiles,
                                                             int32_t *__restrict__ offsets,
                                                             int32_t *__restrict__ sorted_pair,
                                                             int32_t *__restrict__ inv,
                                                             moe_tile *__restrict__ tiles,
                                                             int32_t *__restrict__ sched)
{
    extern __shared__ int lds[];
    permute_block<PM_THREADS>(ids, P, E, e_first, tile_rows, max_tiles, offsets, sorted_pair, inv, tiles, sched, lds,
                              (int)blockIdx.x, (int)gridDim.x);
}

}  // namespace

int launch_permute(const moe_config &c, int tile_rows, int max_tiles, const int32_t *ids,
                   int32_t *offsets, int32_t *sorted_pair, int32_t *inv, moe_tile *tiles,
                   int32_t *sched, hipStream_t s)
{
    const int P = c.T * c.top_k;
    const int el = local_experts(c);
    const size_t lds = sizeof(int) * permute_lds_ints(PM_THREADS, el);
    const int wgs = min(PM_MAX_WGS, max(1, ceil_div(P, PM_SLICE)));
    hipLaunchKernelGGL(permute_kernel, dim3(wgs), dim3(PM_THREADS), lds, s, ids, P, el, c.local_expert_offset,
                       tile_rows, max_tiles,
                       offsets, sorted_pair, inv, tiles, sched);
    return check_launch();
}

}  // namespace moe
