// Device code of the weighted combine: out[t,:] = sum_j w[t,j] * y[inv[t*k+j],:].
//
// Each thread owns 8 consecutive hidden elements of one token and walks the token's
// k expert rows in slot order (their loads requested eight at a time), so the fp32 sum
// has one fixed order and needs no atomics; the result is rounded once to bf16
// (nearest-even).  NT: the expert rows are read with non-temporal loads - right when [P,H] is far
// larger than the L2s and was streamed out by the down projection (4096 DeepSeek tokens: 103 ->
// 80 us); wrong when only a share of the experts is local and the few rows that exist are still
// cached (measured 24 -> 29 us on a 32-of-256 share), so the launch picks.
// SPLIT: the expert rows arrive as the two fp32 partial sums of a down projection whose K was cut in
// halves (y = [2][P,H] floats): a row is their sum, first half first, rounded to bf16 as the unsplit
// projection rounds its output, and then enters the weighted sum as above.
#pragma once
#include "moe_internal.hpp"

namespace moe {
namespace {

// One thread's share: 8 consecutive hidden elements of one token; idx numbers the shares token-major
// (idx < T * H / 8).
template <bool NT, bool SPLIT = false>
__device__ __forceinline__ void combine_chunk(const uint16_t *__restrict__ y, const float *__restrict__ w,
                                              const int32_t *__restrict__ inv, uint16_t *__restrict__ out, int H,
                                              int k, long long idx, size_t split_stride = 0)
{
    const int chunks = H / 8;
    const int t = (int)(idx / chunks), h = (int)(idx % chunks) * 8;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    // slots in groups of CB: the rows of a group are requested together, then added in slot order
    constexpr int CB = SPLIT ? 2 : 8;
    for (int j0 = 0; j0 < k; j0 += CB) {
        int row[CB];
        float wt[CB];
        uint4 raw[CB];
#pragma unroll
        for (int u = 0; u < CB; ++u) {
            const bool in = j0 + u < k;
            row[u] = in ? inv[(size_t)t * k + j0 + u] : -1;
            wt[u] = in ? w[(size_t)t * k + j0 + u] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < CB; ++u)
        {
            typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
            u32x4_t v = {0u, 0u, 0u, 0u};
            if constexpr (SPLIT) {
                typedef float f32x4_t __attribute__((ext_vector_type(4)));
                if (row[u] >= 0) {
                    const float *p0 = reinterpret_cast<const float *>(y) + (size_t)row[u] * H + h;
                    const float *p1 = reinterpret_cast<const float *>(reinterpret_cast<const unsigned char *>(y) + split_stride) +
                                      (size_t)row[u] * H + h;
                    const f32x4_t a0 = *reinterpret_cast<const f32x4_t *>(p0), a1 = *reinterpret_cast<const f32x4_t *>(p0 + 4);
                    const f32x4_t b0 = *reinterpret_cast<const f32x4_t *>(p1), b1 = *reinterpret_cast<const f32x4_t *>(p1 + 4);
                    v[0] = pack_bf16x2(a0[0] + b0[0], a0[1] + b0[1]);
                    v[1] = pack_bf16x2(a0[2] + b0[2], a0[3] + b0[3]);
                    v[2] = pack_bf16x2(a1[0] + b1[0], a1[1] + b1[1]);
                    v[3] = pack_bf16x2(a1[2] + b1[2], a1[3] + b1[3]);
                }
            } else if (row[u] >= 0) {
                const u32x4_t *src = reinterpret_cast<const u32x4_t *>(y + (size_t)row[u] * H + h);
                v = NT ? __builtin_nontemporal_load(src) : *src;
            }
            raw[u] = uint4{v[0], v[1], v[2], v[3]};
        }
#pragma unroll
        for (int u = 0; u < CB; ++u) {
            if (row[u] < 0) continue;                      // a pair without a row (its expert is held elsewhere)
            const uint32_t v[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[2 * i] = fmaf(wt[u], bf16_bits_to_f32(v[i] & 0xffffu), acc[2 * i]);
                acc[2 * i + 1] = fmaf(wt[u], bf16_bits_to_f32(v[i] >> 16), acc[2 * i + 1]);
            }
        }
    }
    uint4 o;
    o.x = pack_bf16x2(acc[0], acc[1]);
    o.y = pack_bf16x2(acc[2], acc[3]);
    o.z = pack_bf16x2(acc[4], acc[5]);
    o.w = pack_bf16x2(acc[6], acc[7]);
    *reinterpret_cast<uint4 *>(out + (size_t)t * H + h) = o;
}


// Rows that were streamed out by the down projection and are read exactly once here are better read
// with non-temporal loads (see the header of this file).
inline bool combine_streams(const moe_config &c)
{
    return local_experts(c) == c.E && (size_t)c.T * c.top_k * c.H * 2 > ((size_t)32 << 20);
}

}  // namespace
}  // namespace moe
