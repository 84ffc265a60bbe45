// Weighted combine kernel; the arithmetic is in moe_combine_device.hpp.
#include "moe_combine_device.hpp"

namespace moe {
namespace {

template <bool NT, bool SPLIT>
__global__ __launch_bounds__(256) void combine_kernel(const uint16_t *__restrict__ y,
                                                      const float *__restrict__ w,
                                                      const int32_t *__restrict__ inv,
                                                      uint16_t *__restrict__ out, int T, int H, int k,
                                                      size_t split_stride)
{
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)T * (H / 8)) return;
    combine_chunk<NT, SPLIT>(y, w, inv, out, H, k, idx, split_stride);
}

}  // namespace

int launch_combine(const moe_config &c, const void *y, const float *w, const int32_t *inv, void *out,
                   hipStream_t s, int k_split)
{
    const long long work = (long long)c.T * (c.H / 8);
    const unsigned blocks = (unsigned)((work + 255) / 256);
    const bool streamed = combine_streams(c);
    const size_t split_stride = (size_t)c.T * c.top_k * c.H * sizeof(float);
    if (k_split > 1)
        hipLaunchKernelGGL((combine_kernel<false, true>), dim3(blocks), dim3(256), 0, s, static_cast<const uint16_t *>(y), w,
                           inv, static_cast<uint16_t *>(out), c.T, c.H, c.top_k, split_stride);
    else if (streamed)
        hipLaunchKernelGGL((combine_kernel<true, false>), dim3(blocks), dim3(256), 0, s, static_cast<const uint16_t *>(y), w,
                           inv, static_cast<uint16_t *>(out), c.T, c.H, c.top_k, (size_t)0);
    else
        hipLaunchKernelGGL((combine_kernel<false, false>), dim3(blocks), dim3(256), 0, s, static_cast<const uint16_t *>(y), w,
                           inv, static_cast<uint16_t *>(out), c.T, c.H, c.top_k, (size_t)0);
    return check_launch();
}

}  // namespace moe
