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
#include "moe_internal.hpp"

namespace moe {
namespace {

constexpr int RT_TM = 64;     // tokens per workgroup tile
constexpr int RT_TN = 64;     // experts per workgroup tile
constexpr int RT_BK = 32;     // hidden elements per LDS stage
constexpr int RT_PAD = 4;
constexpr int RT_MAX_SPLIT = 32;

struct RouteGrid { int tiles_t, tiles_e, splits, k_per_split; };

RouteGrid route_grid(const moe_config &c)
{
    RouteGrid g;
    g.tiles_t = ceil_div(c.T, RT_TM);
    g.tiles_e = ceil_div(c.E, RT_TN);
    const int chunks = ceil_div(c.H, RT_BK);
    int want = ceil_div(512, g.tiles_t * g.tiles_e);          // aim at >= 2 workgroups per CU
    if (want > RT_MAX_SPLIT) want = RT_MAX_SPLIT;
    if (want > chunks) want = chunks;
    if (want < 1) want = 1;
    g.k_per_split = ceil_div(chunks, want) * RT_BK;
    g.splits = ceil_div(c.H, g.k_per_split);
    return g;
}

// 8 consecutive hidden values of one token as fp32 (zero outside the tensor).
template <bool FP8>
__device__ inline void load_x8(const void *x, const float *x_scale, int T, int H, int t, int h, float v[8])
{
    if (t >= T || h >= H) {
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = 0.f;
        return;
    }
    if constexpr (FP8) {
        const uint2 raw = *reinterpret_cast<const uint2 *>(static_cast<const uint8_t *>(x) + (size_t)t * H + h);
        const float sc = x_scale[(size_t)t * (H / kQBlock) + h / kQBlock];
        v[0] = __builtin_amdgcn_cvt_f32_fp8(raw.x, 0) * sc;
        v[1] = __builtin_amdgcn_cvt_f32_fp8(raw.x, 1) * sc;
        v[2] = __builtin_amdgcn_cvt_f32_fp8(raw.x, 2) * sc;
        v[3] = __builtin_amdgcn_cvt_f32_fp8(raw.x, 3) * sc;
        v[4] = __builtin_amdgcn_cvt_f32_fp8(raw.y, 0) * sc;
        v[5] = __builtin_amdgcn_cvt_f32_fp8(raw.y, 1) * sc;
        v[6] = __builtin_amdgcn_cvt_f32_fp8(raw.y, 2) * sc;
        v[7] = __builtin_amdgcn_cvt_f32_fp8(raw.y, 3) * sc;
    } else {
        const uint4 raw = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(x) + (size_t)t * H + h);
        v[0] = bf16_bits_to_f32(raw.x & 0xffffu); v[1] = bf16_bits_to_f32(raw.x >> 16);
        v[2] = bf16_bits_to_f32(raw.y & 0xffffu); v[3] = bf16_bits_to_f32(raw.y >> 16);
        v[4] = bf16_bits_to_f32(raw.z & 0xffffu); v[5] = bf16_bits_to_f32(raw.z >> 16);
        v[6] = bf16_bits_to_f32(raw.w & 0xffffu); v[7] = bf16_bits_to_f32(raw.w >> 16);
    }
}

template <bool FP8>
__global__ __launch_bounds__(256) void router_logits_kernel(const void *__restrict__ x,
                                                            const float *__restrict__ x_scale,
                                                            const float *__restrict__ router_w,
                                                            float *__restrict__ zpart, int T, int H, int E,
                                                            int k_per_split)
{
    __shared__ float As[RT_BK][RT_TM + RT_PAD];
    __shared__ float Bs[RT_BK][RT_TN + RT_PAD];
    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * RT_TM, e0 = blockIdx.y * RT_TN;
    const int kbeg = blockIdx.z * k_per_split;
    const int kend = min(H, kbeg + k_per_split);
    const int lrow = tid >> 2, lk = (tid & 3) * 8;       // loader coordinates
    const int ty = tid >> 4, tx = tid & 15;              // 4x4 outputs per thread

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = kbeg; k0 < kend; k0 += RT_BK) {
        float xv[8], wv[8];
        load_x8<FP8>(x, x_scale, T, H, t0 + lrow, k0 + lk, xv);
        if (e0 + lrow < E && k0 + lk < H) {
            const float4 *src = reinterpret_cast<const float4 *>(router_w + (size_t)(e0 + lrow) * H + k0 + lk);
            const float4 a = src[0], b = src[1];
            wv[0] = a.x; wv[1] = a.y; wv[2] = a.z; wv[3] = a.w;
            wv[4] = b.x; wv[5] = b.y; wv[6] = b.z; wv[7] = b.w;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) wv[j] = 0.f;
        }
        __syncthreads();                                  // previous stage fully consumed
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            As[lk + j][lrow] = xv[j];
            Bs[lk + j][lrow] = wv[j];
        }
        __syncthreads();
        // two-level summation: a short chain per stage, added to the running total
        float part[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) part[i][j] = 0.f;
#pragma unroll
        for (int k = 0; k < RT_BK; ++k) {
            const float4 a = *reinterpret_cast<const float4 *>(&As[k][ty * 4]);
            const float4 b = *reinterpret_cast<const float4 *>(&Bs[k][tx * 4]);
            const float av[4] = {a.x, a.y, a.z, a.w};
            const float bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) part[i][j] = fmaf(av[i], bv[j], part[i][j]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] += part[i][j];
    }

    float *dst = zpart + (size_t)blockIdx.z * T * E;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = t0 + ty * 4 + i;
        if (t >= T) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = e0 + tx * 4 + j;
            if (e < E) dst[(size_t)t * E + e] = acc[i][j];
        }
    }
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

// ---- cross-lane helpers -------------------------------------------------------

// Monotone map fp32 -> uint32 (larger float <=> larger integer).
__device__ inline uint32_t orderable(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// (key, expert) packed so that an unsigned max picks the larger key, then the lower index.
__device__ inline unsigned long long pack_key(float c, int e)
{
    return ((unsigned long long)orderable(c) << 32) | (unsigned long long)(0xffffffffu - (uint32_t)e);
}

// Partner exchange of an all-reduce butterfly over the 64 lanes, step by step (STEP = 0..5 joins
// groups of 2^STEP lanes into groups of twice the size).  Inside a row of 16 lanes the value
// comes through DPP, which costs no more than the ALU operation it feeds: swaps inside a quad for
// steps 0 and 1, then the mirror images of 8 and of 16 lanes (after the earlier steps all lanes of
// a group hold the same value, so any lane of the other group serves).  Step 4 crosses rows with
// a swizzle, step 5 crosses the two halves of the wavefront with a lane permute; only those two
// go through the LDS crossbar.
template <int STEP>
__device__ __forceinline__ uint32_t butterfly_partner(uint32_t v)
{
    static_assert(STEP >= 0 && STEP <= 5, "64 lanes");
    if constexpr (STEP == 0) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false);    // quad_perm [1,0,3,2]
    else if constexpr (STEP == 1) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
    else if constexpr (STEP == 2) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, false);  // row_half_mirror
    else if constexpr (STEP == 3) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, false);  // row_mirror
    else if constexpr (STEP == 4) return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F);                     // lane ^ 16
    else return (uint32_t)__shfl_xor((int)v, 32, kWave);
}

template <int STEP>
__device__ __forceinline__ unsigned long long butterfly_max_u64(unsigned long long v)
{
    const uint32_t lo = butterfly_partner<STEP>((uint32_t)v);
    const uint32_t hi = butterfly_partner<STEP>((uint32_t)(v >> 32));
    const unsigned long long o = ((unsigned long long)hi << 32) | lo;
    return o > v ? o : v;
}

// max over aligned segments of `width` lanes (width = power of two <= 64; the same on every lane)
__device__ inline unsigned long long seg_max_u64(unsigned long long v, int width)
{
    if (width > 1) v = butterfly_max_u64<0>(v);
    if (width > 2) v = butterfly_max_u64<1>(v);
    if (width > 4) v = butterfly_max_u64<2>(v);
    if (width > 8) v = butterfly_max_u64<3>(v);
    if (width > 16) v = butterfly_max_u64<4>(v);
    if (width > 32) v = butterfly_max_u64<5>(v);
    return v;
}

__device__ inline float wave_max_f32(float v)
{
    v = fmaxf(v, __uint_as_float(butterfly_partner<0>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(butterfly_partner<1>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(butterfly_partner<2>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(butterfly_partner<3>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(butterfly_partner<4>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(butterfly_partner<5>(__float_as_uint(v))));
    return v;
}

// Every lane adds the same two operands at every step, so all lanes end with the same value.
__device__ inline float wave_sum_f32(float v)
{
    v += __uint_as_float(butterfly_partner<0>(__float_as_uint(v)));
    v += __uint_as_float(butterfly_partner<1>(__float_as_uint(v)));
    v += __uint_as_float(butterfly_partner<2>(__float_as_uint(v)));
    v += __uint_as_float(butterfly_partner<3>(__float_as_uint(v)));
    v += __uint_as_float(butterfly_partner<4>(__float_as_uint(v)));
    v += __uint_as_float(butterfly_partner<5>(__float_as_uint(v)));
    return v;
}

struct TopkParams {
    int T, E, top_k, scoring, renormalize, n_group, topk_group, group_score_topn, splits;
    float routed_scale;
};

// Scoring rule, optional group limiting and top-k of one token by one wavefront.  Lane l owns
// experts l*EPL .. l*EPL+EPL-1 (contiguous, so a group of experts is a run of lanes); z holds
// their logits.
template <int EPL>
__device__ __forceinline__ void route_token(const float (&z)[EPL], int lane, int t, const float *__restrict__ bias,
                                            int32_t *__restrict__ ids, float *__restrict__ w, const TopkParams &p)
{
    const int E = p.E;
    float s[EPL];
    unsigned long long key[EPL];
    if (p.scoring == MOE_SCORE_SOFTMAX) {
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < EPL; ++i) if (lane * EPL + i < E) m = fmaxf(m, z[i]);
        m = wave_max_f32(m);
        float den = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            s[i] = (lane * EPL + i < E) ? expf(z[i] - m) : 0.f;
            den += s[i];
        }
        den = wave_sum_f32(den);
#pragma unroll
        for (int i = 0; i < EPL; ++i) s[i] = s[i] / den;
    } else {
#pragma unroll
        for (int i = 0; i < EPL; ++i) s[i] = 1.f / (1.f + expf(-z[i]));
    }
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const int e = lane * EPL + i;
        const float c = s[i] + ((bias != nullptr && e < E) ? bias[e] : 0.f);
        key[i] = (e < E) ? pack_key(c, e) : 0ull;          // 0 = not a candidate
    }

    // ---- group limiting ----------------------------------------------------
    if (p.n_group > 1) {
        const int gsz = E / p.n_group;
        const int lpg = gsz / EPL;                         // lanes per group (power of two)
        const int my_group = lane / lpg;
        unsigned long long left[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) left[i] = key[i];
        float gscore = 0.f;
        for (int n = 0; n < p.group_score_topn; ++n) {
            unsigned long long best = 0ull;
#pragma unroll
            for (int i = 0; i < EPL; ++i) best = left[i] > best ? left[i] : best;
            best = seg_max_u64(best, lpg);
#pragma unroll
            for (int i = 0; i < EPL; ++i) if (left[i] == best) left[i] = 0ull;
            // undo the order-preserving map to get the key value back
            const uint32_t ob = (uint32_t)(best >> 32);
            const uint32_t fb = (ob & 0x80000000u) ? (ob & 0x7fffffffu) : ~ob;
            gscore += (best != 0ull) ? __uint_as_float(fb) : 0.f;
        }
        int rank = 0;
        for (int g = 0; g < p.n_group; ++g) {
            const float og = __shfl(gscore, g * lpg, kWave);
            rank += (og > gscore) || (og == gscore && g < my_group);
        }
        const bool kept = my_group < p.n_group && rank < p.topk_group;
#pragma unroll
        for (int i = 0; i < EPL; ++i) if (!kept) key[i] = 0ull;
    }

    // ---- k rounds of wave-wide arg-max ----------------------------------------
    int my_id = 0;
    float my_s = 0.f;
    for (int j = 0; j < p.top_k; ++j) {
        unsigned long long best = 0ull;
#pragma unroll
        for (int i = 0; i < EPL; ++i) best = key[i] > best ? key[i] : best;
        best = seg_max_u64(best, kWave);
        int e = (int)(0xffffffffu - (uint32_t)best);
        e = e < 0 ? 0 : (e >= E ? E - 1 : e);              // keeps ids in range whatever the inputs
        float sel = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i)
            if (lane * EPL + i == e) { sel = s[i]; key[i] = 0ull; }
        sel = __shfl(sel, e / EPL, kWave);
        if (lane == j) { my_id = e; my_s = sel; }
    }
    float sum = 0.f;
    for (int j = 0; j < p.top_k; ++j) sum += __shfl(my_s, j, kWave);   // slot order
    if (lane < p.top_k) {
        float wt = my_s;
        if (p.renormalize) wt = wt / sum;
        wt *= p.routed_scale;
        ids[(size_t)t * p.top_k + lane] = my_id;
        w[(size_t)t * p.top_k + lane] = wt;
    }
}

// One wavefront per token: adds the partial logits of the H splits, then routes the token.
// NB = splits whose partial logits are requested together (8, or 32 when H was cut into more than
// 8 slices - few tokens, so registers are not what limits the kernel, the latency of one round of
// loads after another is: 64 decode tokens 17 -> 9 us).
template <int EPL, int NB>
__global__ __launch_bounds__(256) void router_topk_kernel(const float *__restrict__ zpart,
                                                          const float *__restrict__ bias,
                                                          int32_t *__restrict__ ids, float *__restrict__ w,
                                                          TopkParams p)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int t = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (t >= p.T) return;                                  // whole wave leaves together
    const int E = p.E;
    float z[EPL];
    // partial logits of the H splits, added in split order; the loads of NB splits are issued
    // together so that their latencies overlap
#pragma unroll
    for (int i = 0; i < EPL; ++i) z[i] = 0.f;
    // Every load is unconditional (split and expert indices are clamped, what lies outside is
    // zeroed afterwards): a load under a branch would be waited for before the next one is issued.
    const bool whole = E % EPL == 0;                       // a lane's experts are all inside or all outside: one wide load
    for (int sp0 = 0; sp0 < p.splits; sp0 += NB) {
        float part[NB][EPL];
        if (whole) {
            typedef float wide_t __attribute__((ext_vector_type(EPL < 4 ? EPL : 4)));
            constexpr int WN = EPL < 4 ? EPL : 4;
            const int e_lane = min(lane * EPL, E - EPL);
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int sp = min(sp0 + u, p.splits - 1);
                const wide_t *src = reinterpret_cast<const wide_t *>(zpart + ((size_t)sp * p.T + t) * E + e_lane);
#pragma unroll
                for (int q = 0; q < EPL / WN; ++q) {
                    const wide_t v = src[q];
#pragma unroll
                    for (int i = 0; i < WN; ++i) part[u][q * WN + i] = v[i];
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int sp = min(sp0 + u, p.splits - 1);
                const float *src = zpart + ((size_t)sp * p.T + t) * E;
#pragma unroll
                for (int i = 0; i < EPL; ++i) part[u][i] = src[min(lane * EPL + i, E - 1)];
            }
        }
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
            for (int i = 0; i < EPL; ++i)
                if (sp0 + u >= p.splits || lane * EPL + i >= E) part[u][i] = 0.f;
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
            for (int i = 0; i < EPL; ++i) z[i] += part[u][i];
    }

    route_token<EPL>(z, lane, t, bias, ids, w, p);
}

// Few experts (E <= RT_FEW): logits and routing of a token in one wavefront, one launch.  The
// lanes split H (8 consecutive elements per lane and pass); every lane keeps one running sum per
// expert, a butterfly adds them across the wavefront in a fixed order.
constexpr int RT_FEW = 16;

// WPT wavefronts share a token (each takes a contiguous part of H, the parts are added in wavefront
// order): with few tokens one wavefront per token leaves most of the chip idle and is bound by the
// latency of its own loads.
template <bool FP8, int WPT>
__global__ __launch_bounds__(256) void router_few_experts_kernel(const void *__restrict__ x,
                                                                 const float *__restrict__ x_scale,
                                                                 const float *__restrict__ router_w,
                                                                 const float *__restrict__ bias,
                                                                 int32_t *__restrict__ ids, float *__restrict__ w,
                                                                 TopkParams p, int H)
{
    constexpr int TPB = 4 / WPT;                           // tokens per workgroup of four wavefronts
    __shared__ float part_z[4][RT_FEW];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x / kWave;
    const int t = blockIdx.x * TPB + wv / WPT;
    const int sub = wv % WPT;                              // which part of H this wavefront sums
    const bool live = t < p.T;
    if (WPT == 1 && !live) return;                         // whole wave leaves together (no barrier below)
    const int E = p.E;
    // parts are whole 128-element scale blocks (H is a multiple of 64; of 128 for fp8)
    const int hpart = ((H / WPT + 127) / 128) * 128;
    const int hbeg = min(H, sub * hpart), hend = min(H, hbeg + hpart);
    float acc[RT_FEW];
#pragma unroll
    for (int e = 0; e < RT_FEW; ++e) acc[e] = 0.f;
    // four passes per iteration so that the loads of all of them are in flight together
    for (int h0 = hbeg + lane * 8; live && h0 < hend; h0 += 4 * kWave * 8) {
        float xv[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int h = h0 + u * kWave * 8;              // beyond this wavefront's part: zeros (h >= H gives zeros)
            load_x8<FP8>(x, x_scale, p.T, H, t, h < hend ? h : H, xv[u]);
        }
#pragma unroll
        for (int e = 0; e < RT_FEW; ++e) {
            if (e < E) {
                float4 a[4], b[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int h = h0 + u * kWave * 8;
                    if (h < hend) {
                        const float4 *src = reinterpret_cast<const float4 *>(router_w + (size_t)e * H + h);
                        a[u] = src[0]; b[u] = src[1];
                    } else {
                        a[u] = b[u] = float4{0.f, 0.f, 0.f, 0.f};
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    float part = xv[u][0] * a[u].x;        // short chain per pass, added to the running sum
                    part = fmaf(xv[u][1], a[u].y, part); part = fmaf(xv[u][2], a[u].z, part);
                    part = fmaf(xv[u][3], a[u].w, part); part = fmaf(xv[u][4], b[u].x, part);
                    part = fmaf(xv[u][5], b[u].y, part); part = fmaf(xv[u][6], b[u].z, part);
                    part = fmaf(xv[u][7], b[u].w, part);
                    acc[e] += part;
                }
            }
        }
    }
    float z[1] = {0.f};
#pragma unroll
    for (int e = 0; e < RT_FEW; ++e) {
        if (e < E) {
            const float total = wave_sum_f32(acc[e]);
            if (lane == e) z[0] = total;
        }
    }
    if constexpr (WPT > 1) {
        if (lane < RT_FEW) part_z[wv][lane] = z[0];
        __syncthreads();
        if (sub != 0 || !live) return;
        if (lane < RT_FEW) {
            float total = part_z[wv][lane];
#pragma unroll
            for (int j = 1; j < WPT; ++j) total += part_z[wv + j][lane];
            z[0] = total;
        }
    }
    route_token<1>(z, lane, t, bias, ids, w, p);
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
