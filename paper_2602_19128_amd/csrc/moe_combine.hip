// Weighted combine kernel; the arithmetic is in moe_combine_device.hpp.
#include "moe_combine_device.hpp"

namespace moe {
namespace {

template <bool NT>
__global__ __launch_bounds__(256) void combine_kernel(const uint16_t *__restrict__ y,
                                                      const float *__restrict__ w,
                                                      const int32_t *__restrict__ inv,
                                                      uint16_t *__restrict__ out, int T, int H, int k)
{
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)T * (H / 8)) return;
    combine_chunk<NT>(y, w, inv, out, H, k, idx);
}

}  // namespace

int launch_combine(const moe_config &c, const void *y, const float *w, const int32_t *inv, void *out,
                   hipStream_t s)
{
    const long long work = (long long)c.T * (c.H / 8);
    const unsigned blocks = (unsigned)((work + 255) / 256);
    const bool streamed = combine_streams(c);
    if (streamed)
        hipLaunchKernelGGL(combine_kernel<true>, dim3(blocks), dim3(256), 0, s, static_cast<const uint16_t *>(y), w, inv,
                           static_cast<uint16_t *>(out), c.T, c.H, c.top_k);
    else
        hipLaunchKernelGGL(combine_kernel<false>, dim3(blocks), dim3(256), 0, s, static_cast<const uint16_t *>(y), w, inv,
                           static_cast<uint16_t *>(out), c.T, c.H, c.top_k);
    return check_launch();
}

}  // namespace moe
