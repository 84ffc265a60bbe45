// Device code of the router shared by the stand-alone routing kernels and the single-launch
// forward (paper Sec. 4.5 "Routing"): the LDS-tiled fp32 logits tile, the scoring rule with optional
// group limiting and the cross-lane top-k of one token by one wavefront, and the one-wavefront
// logits + routing of layers with few experts.
#pragma once
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

// One (64 tokens x 64 experts x one slice of H) tile of the partial logits by a workgroup of 256
// threads: z = x . router_w^T in fp32, LDS-tiled.  As / Bs are the workgroup's two LDS stages.
struct LogitsLds { float As[RT_BK][RT_TM + RT_PAD]; float Bs[RT_BK][RT_TN + RT_PAD]; };

template <bool FP8>
__device__ __forceinline__ void router_logits_tile(const void *__restrict__ x, const float *__restrict__ x_scale,
                                                   const float *__restrict__ router_w, float *__restrict__ zpart,
                                                   int T, int H, int E, int k_per_split, int tile_t, int tile_e,
                                                   int split, LogitsLds &lds)
{
    float (&As)[RT_BK][RT_TM + RT_PAD] = lds.As;
    float (&Bs)[RT_BK][RT_TN + RT_PAD] = lds.Bs;
    const int tid = threadIdx.x;
    const int t0 = tile_t * RT_TM, e0 = tile_e * RT_TN;
    const int kbeg = split * k_per_split;
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

    float *dst = zpart + (size_t)split * T * E;
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
__device__ __forceinline__ void router_topk_token(const float *__restrict__ zpart, const float *__restrict__ bias,
                                                  int32_t *__restrict__ ids, float *__restrict__ w,
                                                  const TopkParams &p, int t, int lane)
{
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
// `block` numbers groups of 4 / WPT tokens; part_z is the workgroup's LDS scratch (with WPT > 1 the
// caller must put a workgroup barrier between two calls).
template <bool FP8, int WPT>
__device__ __forceinline__ void router_few_tokens(const void *__restrict__ x, const float *__restrict__ x_scale,
                                                  const float *__restrict__ router_w, const float *__restrict__ bias,
                                                  int32_t *__restrict__ ids, float *__restrict__ w,
                                                  const TopkParams &p, int H, int block, float (&part_z)[4][RT_FEW])
{
    constexpr int TPB = 4 / WPT;                           // tokens per workgroup of four wavefronts
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x / kWave;
    const int t = block * TPB + wv / WPT;
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

// How a problem is routed: which of the paths above, and the H split of the two-kernel paths.
inline bool route_few(const moe_config &c) { return c.E <= RT_FEW; }
inline bool route_few_split(const moe_config &c) { return c.T <= 2048 && c.H >= 1024; }   // four wavefronts per token
inline int route_epl(const moe_config &c) { return c.E <= 64 ? 1 : c.E <= 128 ? 2 : c.E <= 256 ? 4 : 8; }

inline TopkParams topk_params(const moe_config &c, int splits)
{
    return TopkParams{c.T, c.E, c.top_k, c.scoring, c.renormalize, c.n_group, c.topk_group, c.group_score_topn,
                      splits, c.routed_scale};
}

}  // namespace
}  // namespace moe
