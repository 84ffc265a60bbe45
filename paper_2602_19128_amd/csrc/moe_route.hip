// Routing (paper Sec. 4.5 "Routing"): score every expert for every token, keep the top-k.
//
// Few experts (<= 16): router_few_experts_kernel does everything for a token in one wavefront.
// Otherwise two kernels:
//   router_logits_kernel  z = x . router_w^T in fp32, LDS-tiled, split along H so that a
//                         handful of decode tokens still fills the chip; partial sums go
//                         to scratch and are added in a fixed order (deterministic).
//   router_logits_mfma_kernel  the same partial sums on the matrix cores (512 tokens and more):
//                         three bf16 MFMAs per block carry the fp32 weights exactly.
//   router_topk_kernel    one 64-lane wavefront per token: scoring rule, optional
//                         group limiting, then k rounds of a cross-lane arg-max.
#include "moe_route_device.hpp"

namespace moe {
namespace {

template <bool FP8>
__global__ __launch_bounds__(256) void router_logits_kernel(const void *__restrict__ x,
                                                            const float *__restrict__ x_scale,
                                                            const float *__restrict__ router_w,
                                                            float *__restrict__ zpart, int T, int H, int E,
                                                            int k_per_split)
{
    __shared__ LogitsLds lds;
    router_logits_tile<FP8>(x, x_scale, router_w, zpart, T, H, E, k_per_split, blockIdx.x, blockIdx.y, blockIdx.z, lds);
}

// ---- many tokens: logits on the matrix cores ---------------------------------------------------
//
// Each fp32 router weight is split into three bf16 planes, w = hi + mid + lo (each the bf16
// rounding of what the previous ones leave; together they carry the 24-bit mantissa), so that
// x . w = x.hi + x.mid + x.lo with bf16 MFMAs: the hidden states are bf16 (or fp8 payloads, exact
// in bf16), every product is exact in fp32 and the sums accumulate in fp32, which keeps the logits
// at fp32 accuracy - a routing decision is only allowed to differ from an exact evaluation when
// its margin is below 1e-6.  The split happens in registers, on the fragment a wavefront has just
// loaded (a dozen VALU operations per pair of weights, hidden behind the MFMAs): the weights are
// read as fp32, 4 bytes per element instead of the 6 of stored planes, and no separate pass runs.
//
// A workgroup of 8 wavefronts owns TB*16 tokens x 256 experts x one slice of H.  Wavefront w owns
// expert blocks 2w, 2w+1 (16 experts each) against all token blocks; per 32-wide K step the
// workgroup stages the token rows in LDS (double buffered) while every wavefront loads the weights
// of its own experts straight into registers, both several steps ahead.  fp8 inputs: the payload
// is multiplied as is and each 128-wide block's sum is folded in with the token's block scale.
// The partial logits leave through LDS as whole 1 KiB rows.
typedef __attribute__((ext_vector_type(8))) __bf16 rt_bf16x8;
typedef __attribute__((ext_vector_type(4))) float rt_f32x4;

constexpr int RM_BE = 256;                 // experts per workgroup tile
constexpr int RM_BK = 32;                  // hidden elements per K step (one MFMA deep)
constexpr int RM_THREADS = 512;
constexpr int RM_MIN_TOKENS = 512;         // below this the FMA kernel's finer tiles fill the chip better

typedef __attribute__((ext_vector_type(2))) float rt_f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 rt_bf16x2;

// 8 fp8 e4m3 payload bytes -> 8 bf16.  An e4m3 value has 4 significant bits, so its binary32 form
// has a zero low half and keeping the high half is exact: no rounding step is needed.
__device__ inline uint32_t fp8x2_to_bf16x2(uint32_t word, bool high_pair)
{
    const rt_f32x2 f = high_pair ? __builtin_amdgcn_cvt_pk_f32_fp8(word, true) : __builtin_amdgcn_cvt_pk_f32_fp8(word, false);
    return (__float_as_uint(f[0]) >> 16) | (__float_as_uint(f[1]) & 0xffff0000u);
}
__device__ inline uint4 fp8x8_to_bf16x8(uint2 raw)
{
    uint4 o;
    o.x = fp8x2_to_bf16x2(raw.x, false);
    o.y = fp8x2_to_bf16x2(raw.x, true);
    o.z = fp8x2_to_bf16x2(raw.y, false);
    o.w = fp8x2_to_bf16x2(raw.y, true);
    return o;
}

// Two fp32 router weights -> their three bf16 planes (hi, mid, lo: each the bf16 rounding, to nearest
// even, of what the previous ones leave; the remainders are exact in fp32).
__device__ inline void split_pair(float a, float b, uint32_t &hi, uint32_t &mid, uint32_t &lo)
{
    const rt_bf16x2 h = __builtin_convertvector(rt_f32x2{a, b}, rt_bf16x2);
    hi = __builtin_bit_cast(uint32_t, h);
    const float ra = a - __uint_as_float(hi << 16), rb = b - __uint_as_float(hi & 0xffff0000u);
    const rt_bf16x2 m = __builtin_convertvector(rt_f32x2{ra, rb}, rt_bf16x2);
    mid = __builtin_bit_cast(uint32_t, m);
    const float sa = ra - __uint_as_float(mid << 16), sb = rb - __uint_as_float(mid & 0xffff0000u);
    const rt_bf16x2 l = __builtin_convertvector(rt_f32x2{sa, sb}, rt_bf16x2);
    lo = __builtin_bit_cast(uint32_t, l);
}

template <bool FP8, int TB>
__global__ __launch_bounds__(RM_THREADS) void router_logits_mfma_kernel(const void *__restrict__ x,
                                                                        const float *__restrict__ x_scale,
                                                                        const float *__restrict__ router_w,
                                                                        float *__restrict__ zpart, int T, int H, int E,
                                                                        int k_per_split, int splits)
{
    constexpr int BT = TB * 16;                            // tokens per workgroup
    constexpr int X_BYTES = BT * RM_BK * 2;                // one stage of token rows (bf16)
    constexpr int XV = BT * 4 / RM_THREADS;                // 16-byte pieces of x per thread and stage (2 or 1)
    constexpr int AHEAD = FP8 ? 2 : 3;                     // K steps whose loads are in flight (register budget)
    static_assert(XV >= 1 && BT * 4 % RM_THREADS == 0, "token tile must give every thread whole pieces");
    extern __shared__ __align__(16) unsigned char rsm[];   // two stages of token rows; at the end the output tile

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    // Consecutive workgroups go to consecutive XCDs (eight, each with its own L2): the slice of H is
    // the fastest index, so an XCD works on splits/8 (or one) slices of the router weights and keeps
    // them in its L2 while the token tiles stream past.
    const int zs = blockIdx.x % splits, xt = blockIdx.x / splits;
    const int t0 = xt * BT, e0 = blockIdx.y * RM_BE;
    const int kbeg = zs * k_per_split;
    const int kend = min(H, kbeg + k_per_split);
    const int nsteps = (kend - kbeg) / RM_BK;              // H and the split size are multiples of 32

    // Token rows go through LDS (every wavefront needs all of them): piece v of this thread is row
    // (tid + v*512) / 4, 16-byte chunk (tid + v*512) % 4.  The weights of a wavefront's 32 experts
    // are needed by that wavefront alone, so they are loaded straight into the MFMA layout: lane
    // (l16, lq) holds 8 consecutive k of expert l16 of each block.  Both are requested AHEAD steps
    // before use (register sets in rotation).
    auto load_x = [&](int step, uint4 (&xr)[XV]) __attribute__((always_inline)) {
        const int k0 = kbeg + step * RM_BK;
#pragma unroll
        for (int v = 0; v < XV; ++v) {
            const int idx = tid + v * RM_THREADS, row = idx >> 2, ch = idx & 3;
            const int t = min(t0 + row, T - 1);            // rows past the end repeat the last token; never stored
            if constexpr (FP8) {
                const uint2 raw = *reinterpret_cast<const uint2 *>(static_cast<const uint8_t *>(x) + (size_t)t * H + k0 + ch * 8);
                xr[v] = fp8x8_to_bf16x8(raw);
            } else {
                xr[v] = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(x) + (size_t)t * H + k0 + ch * 8);
            }
        }
    };
    auto store_x = [&](int buf, const uint4 (&xr)[XV]) __attribute__((always_inline)) {
        unsigned char *xs = rsm + buf * X_BYTES;
#pragma unroll
        for (int v = 0; v < XV; ++v) *reinterpret_cast<uint4 *>(xs + (tid + v * RM_THREADS) * 16) = xr[v];
    };
    auto load_w = [&](int step, float4 (&wf)[2][2]) __attribute__((always_inline)) {
        const int k = kbeg + step * RM_BK + lq * 8;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int e = min(e0 + (wave * 2 + b) * 16 + l16, E - 1);   // experts past the end: never stored
            const float4 *src = reinterpret_cast<const float4 *>(router_w + (size_t)e * H + k);
            wf[b][0] = src[0];
            wf[b][1] = src[1];
        }
    };

    rt_f32x4 acc[2][TB];
    rt_f32x4 blk[FP8 ? 2 : 1][FP8 ? TB : 1];               // fp8: sum of the current 128-wide scale block
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int m = 0; m < TB; ++m) {
            acc[b][m] = rt_f32x4{0.f, 0.f, 0.f, 0.f};
            if constexpr (FP8) blk[b][m] = rt_f32x4{0.f, 0.f, 0.f, 0.f};
        }

    auto compute_step = [&](int s, const float4 (&wraw)[2][2]) __attribute__((always_inline)) {
        const unsigned char *xs = rsm + (s & 1) * X_BYTES;
        uint4 wr[2][3];                                    // [expert block][plane]: hi, mid, lo
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            split_pair(wraw[b][0].x, wraw[b][0].y, wr[b][0].x, wr[b][1].x, wr[b][2].x);
            split_pair(wraw[b][0].z, wraw[b][0].w, wr[b][0].y, wr[b][1].y, wr[b][2].y);
            split_pair(wraw[b][1].x, wraw[b][1].y, wr[b][0].z, wr[b][1].z, wr[b][2].z);
            split_pair(wraw[b][1].z, wraw[b][1].w, wr[b][0].w, wr[b][1].w, wr[b][2].w);
        }
#pragma unroll
        for (int m = 0; m < TB; ++m) {
            const rt_bf16x8 tf = *reinterpret_cast<const rt_bf16x8 *>(xs + ((m * 16 + l16) * 4 + lq) * 16);
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                rt_f32x4 &dst = FP8 ? blk[b][m] : acc[b][m];
                // smallest plane first: the small contributions meet before the large one is added
                dst = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(rt_bf16x8, wr[b][2]), tf, dst, 0, 0, 0);
                dst = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(rt_bf16x8, wr[b][1]), tf, dst, 0, 0, 0);
                dst = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(rt_bf16x8, wr[b][0]), tf, dst, 0, 0, 0);
            }
        }
        if constexpr (FP8) {
            const int k0 = kbeg + s * RM_BK;
            if ((k0 + RM_BK) % kQBlock == 0 || s + 1 == nsteps) {      // a scale block ends here
#pragma unroll
                for (int m = 0; m < TB; ++m) {
                    const int t = t0 + m * 16 + l16;
                    const float sc = t < T ? x_scale[(size_t)t * (H / kQBlock) + k0 / kQBlock] : 0.f;
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[b][m][v] = fmaf(blk[b][m][v], sc, acc[b][m][v]);
                        blk[b][m] = rt_f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                }
            }
        }
    };

    // Step j uses register set j % AHEAD for its token rows (stored to LDS buffer j & 1 at the end
    // of step j-1) and for its router weights; both sets are refilled for step j + AHEAD as soon as
    // step j has used them.
    uint4 xr0[XV], xr1[XV], xr2[XV];
    float4 w0[2][2], w1[2][2], w2[2][2];
    const int last = max(nsteps - 1, 0);                   // loads past the last step repeat it: no branches
    load_x(0, xr0);
    load_w(0, w0);
    load_x(min(1, last), xr1);
    load_w(min(1, last), w1);
    if constexpr (AHEAD == 3) {
        load_x(min(2, last), xr2);
        load_w(min(2, last), w2);
    }
    store_x(0, xr0);
    __syncthreads();
#define RM_STEP(s_, W_, XCUR_, XNEXT_)                                                        \
    {                                                                                         \
        const int sj = (s_);                                                                  \
        load_x(min(sj + AHEAD, last), XCUR_);        /* XCUR_ held step sj, already in LDS */  \
        compute_step(sj, W_);                                                                 \
        load_w(min(sj + AHEAD, last), W_);                                                    \
        store_x((sj + 1) & 1, XNEXT_);               /* that buffer was last read in step sj-1 */ \
        __syncthreads();                                                                      \
    }
    int s = 0;
    if constexpr (AHEAD == 3) {
        for (; s + 3 <= nsteps; s += 3) {
            RM_STEP(s, w0, xr0, xr1)
            RM_STEP(s + 1, w1, xr1, xr2)
            RM_STEP(s + 2, w2, xr2, xr0)
        }
        if (s < nsteps) RM_STEP(s, w0, xr0, xr1)
        if (s + 1 < nsteps) RM_STEP(s + 1, w1, xr1, xr2)
    } else {
        for (; s + 2 <= nsteps; s += 2) {
            RM_STEP(s, w0, xr0, xr1)
            RM_STEP(s + 1, w1, xr1, xr0)
        }
        if (s < nsteps) RM_STEP(s, w0, xr0, xr1)
    }
#undef RM_STEP

    // Epilogue through LDS, so that the partial logits leave as whole rows: lane (l16, lq) holds, per
    // expert block, experts 4*lq..4*lq+3 of token l16 of each token block; a row of the staged tile
    // is one token's 256 logits (+16 bytes, which spreads the 16 tokens of a write over all banks).
    // The last K step ended with a barrier, so the token stages are free to be overwritten.
    constexpr int OUT_PITCH = RM_BE * 4 + 16;
#pragma unroll
    for (int m = 0; m < TB; ++m)
#pragma unroll
        for (int b = 0; b < 2; ++b)
            *reinterpret_cast<rt_f32x4 *>(rsm + (m * 16 + l16) * OUT_PITCH + ((wave * 2 + b) * 16 + lq * 4) * 4) = acc[b][m];
    __syncthreads();
    float *dst = zpart + (size_t)zs * T * E;
    const int e = e0 + lane * 4;
    const bool vec = (E & 3) == 0 && e + 3 < E;
    for (int r = wave; r < BT; r += RM_THREADS / 64) {
        const int t = t0 + r;
        if (t >= T) break;
        const rt_f32x4 v = *reinterpret_cast<const rt_f32x4 *>(rsm + r * OUT_PITCH + lane * 16);
        float *row = dst + (size_t)t * E + e;
        if (vec) {
            *reinterpret_cast<rt_f32x4 *>(row) = v;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (e + j < E) row[j] = v[j];
        }
    }
}

template <int EPL, int NB>
__global__ __launch_bounds__(256) void router_topk_kernel(const float *__restrict__ zpart,
                                                          const float *__restrict__ bias,
                                                          int32_t *__restrict__ ids, float *__restrict__ w,
                                                          TopkParams p)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int t = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (t >= p.T) return;                                  // whole wave leaves together
    router_topk_token<EPL, NB>(zpart, bias, ids, w, p, t, lane);
}

template <bool FP8, int WPT>
__global__ __launch_bounds__(256) void router_few_experts_kernel(const void *__restrict__ x,
                                                                 const float *__restrict__ x_scale,
                                                                 const float *__restrict__ router_w,
                                                                 const float *__restrict__ bias,
                                                                 int32_t *__restrict__ ids, float *__restrict__ w,
                                                                 TopkParams p, int H)
{
    __shared__ float part_z[4][RT_FEW];
    router_few_tokens<FP8, WPT>(x, x_scale, router_w, bias, ids, w, p, H, blockIdx.x, part_z);
}

}  // namespace

constexpr int RM_OUT_LDS = 8 * 16 * (RM_BE * 4 + 16);    // LDS of the matrix-core logits kernel: the staged output tile
                                                          // (the two token stages fit inside)

// Matrix-core path: token tile height (in 16-row blocks) and H split.
struct MfmaGrid { bool use; int tb, tiles_t, tiles_e, splits, k_per_split; };

MfmaGrid mfma_grid(const moe_config &c)
{
    MfmaGrid g{};
    g.use = c.T >= RM_MIN_TOKENS && c.E > RT_FEW && c.H % RM_BK == 0;
    if (!g.use) return g;
    g.tb = 8;                                              // 128 tokens per workgroup (256 measured 9 % slower: twice the partial logits)
    g.tiles_t = ceil_div(c.T, g.tb * 16);
    g.tiles_e = ceil_div(c.E, RM_BE);
    const int chunks = c.H / RM_BK;
    int want = ceil_div(256, g.tiles_t * g.tiles_e);       // one workgroup per compute unit
    if (want > RT_MAX_SPLIT) want = RT_MAX_SPLIT;
    if (want > chunks) want = chunks;
    if (want < 1) want = 1;
    int per = ceil_div(chunks, want) * RM_BK;
    if (c.dtype == MOE_DTYPE_FP8_E4M3) per = ceil_div(per, kQBlock) * kQBlock;   // splits end on scale-block edges
    g.k_per_split = per;
    g.splits = ceil_div(c.H, per);
    return g;
}

size_t route_workspace_bytes(const moe_config &c)
{
    if (c.E <= RT_FEW) return 256;
    const MfmaGrid m = mfma_grid(c);
    if (m.use)
        return align_up((size_t)m.splits * c.T * c.E * sizeof(float), 256);
    const RouteGrid g = route_grid(c);
    return align_up((size_t)g.splits * c.T * c.E * sizeof(float), 256);
}

int launch_route(const moe_config &c, const void *x, const float *x_scale, const float *router_w,
                 const float *bias, int32_t *ids, float *w, void *ws, hipStream_t s)
{
    TopkParams p{c.T, c.E, c.top_k, c.scoring, c.renormalize, c.n_group, c.topk_group,
                 c.group_score_topn, 1, c.routed_scale};
    if (c.E <= RT_FEW) {
        // few tokens: four wavefronts per token (still at least one workgroup per compute unit's worth of work)
        const bool split = c.T <= 2048 && c.H >= 1024;
        const dim3 fgrid(split ? c.T : ceil_div(c.T, 4));
        if (c.dtype == MOE_DTYPE_FP8_E4M3) {
            if (split)
                hipLaunchKernelGGL((router_few_experts_kernel<true, 4>), fgrid, dim3(256), 0, s, x, x_scale, router_w,
                                   bias, ids, w, p, c.H);
            else
                hipLaunchKernelGGL((router_few_experts_kernel<true, 1>), fgrid, dim3(256), 0, s, x, x_scale, router_w,
                                   bias, ids, w, p, c.H);
        } else {
            if (split)
                hipLaunchKernelGGL((router_few_experts_kernel<false, 4>), fgrid, dim3(256), 0, s, x, x_scale, router_w,
                                   bias, ids, w, p, c.H);
            else
                hipLaunchKernelGGL((router_few_experts_kernel<false, 1>), fgrid, dim3(256), 0, s, x, x_scale, router_w,
                                   bias, ids, w, p, c.H);
        }
        return check_launch();
    }
    float *zpart = static_cast<float *>(ws);
    const MfmaGrid m = mfma_grid(c);
    if (m.use) {
        int rc;
        const dim3 grid(m.tiles_t * m.splits, m.tiles_e, 1);
        if (c.dtype == MOE_DTYPE_FP8_E4M3) {
            auto kern = router_logits_mfma_kernel<true, 8>;
            static DeviceOnce lds_limit_set;
            if ((rc = set_dynamic_lds(lds_limit_set, reinterpret_cast<const void *>(kern), RM_OUT_LDS)) != MOE_OK) return rc;
            hipLaunchKernelGGL(kern, grid, dim3(RM_THREADS), RM_OUT_LDS, s, x, x_scale, router_w, zpart, c.T, c.H, c.E,
                               m.k_per_split, m.splits);
        } else {
            auto kern = router_logits_mfma_kernel<false, 8>;
            static DeviceOnce lds_limit_set;
            if ((rc = set_dynamic_lds(lds_limit_set, reinterpret_cast<const void *>(kern), RM_OUT_LDS)) != MOE_OK) return rc;
            hipLaunchKernelGGL(kern, grid, dim3(RM_THREADS), RM_OUT_LDS, s, x, x_scale, router_w, zpart, c.T, c.H, c.E,
                               m.k_per_split, m.splits);
        }
        rc = check_launch();
        if (rc != MOE_OK) return rc;
        p.splits = m.splits;
    } else {
        const RouteGrid g = route_grid(c);
        const dim3 grid(g.tiles_t, g.tiles_e, g.splits);
        if (c.dtype == MOE_DTYPE_FP8_E4M3)
            hipLaunchKernelGGL(router_logits_kernel<true>, grid, dim3(256), 0, s, x, x_scale, router_w, zpart,
                               c.T, c.H, c.E, g.k_per_split);
        else
            hipLaunchKernelGGL(router_logits_kernel<false>, grid, dim3(256), 0, s, x, x_scale, router_w, zpart,
                               c.T, c.H, c.E, g.k_per_split);
        int rc = check_launch();
        if (rc != MOE_OK) return rc;
        p.splits = g.splits;
    }

    const dim3 tgrid(ceil_div(c.T, 4));
    const int epl = c.E <= 64 ? 1 : c.E <= 128 ? 2 : c.E <= 256 ? 4 : 8;
    const bool many = p.splits > 8;
#define MOE_LAUNCH_TOPK(EPL_)                                                                                       \
    if (many) hipLaunchKernelGGL((router_topk_kernel<EPL_, RT_MAX_SPLIT>), tgrid, dim3(256), 0, s, zpart, bias, ids, w, p); \
    else hipLaunchKernelGGL((router_topk_kernel<EPL_, 8>), tgrid, dim3(256), 0, s, zpart, bias, ids, w, p);
    switch (epl) {
    case 1: MOE_LAUNCH_TOPK(1) break;
    case 2: MOE_LAUNCH_TOPK(2) break;
    case 4: MOE_LAUNCH_TOPK(4) break;
    default: MOE_LAUNCH_TOPK(8) break;
    }
#undef MOE_LAUNCH_TOPK
    return check_launch();
}

}  // namespace moe
