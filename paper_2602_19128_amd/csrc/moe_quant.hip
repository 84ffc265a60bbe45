// Activation quantisation for the fp8 expert GEMMs: bf16 rows -> e4m3 payload + one fp32 scale per
// 1x128 block (paper Sec. 4.3, kernel table: the fp8 MoE operator's packing and scaling).
//
// A thread owns 8 consecutive elements (one 16-byte load, one 8-byte store); the 16 threads of a
// quarter wavefront own one 128-wide block and agree on its largest magnitude with four
// cross-lane exchanges.  Rows are a multiple of 128 long, so blocks never straddle rows and the
// tensor is walked as one flat array of blocks.  Both divisions (amax / 448, x / scale) are
// correctly rounded binary32 divisions: the codes are decided in exactly that precision.
#include "moe_internal.hpp"

namespace moe {
namespace {

constexpr float Q_FP8_MAX = 448.f;

__global__ __launch_bounds__(256) void quantize_act_kernel(const uint4 *__restrict__ x, uint2 *__restrict__ q,
                                                           float *__restrict__ scale, long long chunks)
{
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    // chunks is a multiple of 16: the 16 lanes of a block are all inside or all outside
    const bool live = idx < chunks;
    uint4 raw = uint4{0u, 0u, 0u, 0u};
    if (live) raw = x[idx];
    const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
    float v[8];
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = bf16_bits_to_f32(u[i] & 0xffffu);
        v[2 * i + 1] = bf16_bits_to_f32(u[i] >> 16);
        amax = fmaxf(amax, fmaxf(fabsf(v[2 * i]), fabsf(v[2 * i + 1])));
    }
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) amax = fmaxf(amax, __shfl_xor(amax, m, kWave));
    const float sc = amax > 0.f ? __fdiv_rn(amax, Q_FP8_MAX) : 1.f;
    float r[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = fminf(fmaxf(__fdiv_rn(v[i], sc), -Q_FP8_MAX), Q_FP8_MAX);
    int lo = 0, hi = 0;
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(r[0], r[1], lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(r[2], r[3], lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(r[4], r[5], hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(r[6], r[7], hi, true);
    if (live) {
        q[idx] = uint2{(uint32_t)lo, (uint32_t)hi};
        if ((threadIdx.x & 15) == 0) scale[idx >> 4] = sc;
    }
}

}  // namespace

int launch_quantize_act(const moe_config &c, const void *x, void *xq, float *x_scale, hipStream_t s)
{
    const long long chunks = (long long)c.T * (c.H / 8);
    const unsigned blocks = (unsigned)((chunks + 255) / 256);
    hipLaunchKernelGGL(quantize_act_kernel, dim3(blocks), dim3(256), 0, s, static_cast<const uint4 *>(x),
                       static_cast<uint2 *>(xq), x_scale, chunks);
    return check_launch();
}

}  // namespace moe
