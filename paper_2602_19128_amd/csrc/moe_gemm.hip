// Grouped expert GEMMs on the bf16 matrix cores (paper Sec. 4.5 "Expert FFN
// computation": tensor-core tiles, loads of the next block overlapping the compute of the
// current one, experts without tokens skipped).
//
// Both GEMMs are C[m,n] = sum_k A[m,k] * W[e,n,k] with few rows m per expert (a few to a
// few hundred) against large weight matrices, so the weights must stream from HBM exactly
// once and at full rate.  The kernel is built around that:
//
//  * A workgroup of 8 wavefronts owns ALL rows of one expert tile (up to 16*MB_MAX) times a
//    slab of weight rows; wavefront w owns two blocks of 16 weight rows (gate + matching up
//    rows, or 32 consecutive down-projection rows).  Nothing is shared between wavefronts on
//    the weight side, so weights go HBM -> VGPR directly in the MFMA operand layout (lane l
//    holds 16 bytes of weight row l%16), prefetched D K-steps ahead through D+1 rotating
//    register sets.  No LDS round trip and no barrier stands between HBM and the matrix core.
//  * The token rows (x gathered through the sorted pair list, or act) are shared by all
//    wavefronts: they are copied global -> LDS directly (global_load_lds), D stages ahead in a
//    ring of D+1 stages, and read as the second MFMA operand.  Physical 16-byte chunk pc of
//    LDS row r holds logical chunk pc ^ (r & 7) (applied on the global-address side of the
//    copy) which keeps the fragment reads spread over the banks.
//  * v_mfma_f32_16x16x32_bf16 with the weights as the row operand: the accumulator of lane l
//    holds 4 consecutive output columns of token l%16, so the epilogue applies
//    act = silu(g) * u in registers and stores 8 bytes per lane.
//  * One s_barrier per K step (64 elements) orders the LDS ring; outstanding-load counts are
//    waited for explicitly so that a barrier never drains the weight prefetch queue.
//  * Row blocks beyond the tile's real row count are skipped (the K loop is instantiated per
//    row-block count), so an expert with 140 tokens costs 9 blocks of 16, not 256 rows.
//
// Workgroups are numbered so that each XCD (own L2) gets a contiguous range of the
// (expert tile, column slab) work: the token rows of an expert stay in one L2.
#include "moe_internal.hpp"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int GM_BK = 64;                 // k elements per step (one 128-byte LDS row per token row)
constexpr int GM_WAVES = 8;
constexpr int GM_THREADS = GM_WAVES * kWave;
constexpr int GM_XCDS = 8;
constexpr int GM_B_LOADS = 4;             // weight loads per lane per step: 2 blocks x 2 halves of the step

#define MOE_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define MOE_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define MOE_WAIT_VMCNT(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")
// 16-byte global load issued exactly here.  The compiler does not track its completion: the value
// may only be read after an explicit s_waitcnt followed by a MOE_TIE_SET that names the register
// (an empty asm that makes every later reader data-dependent on a point after the wait, so no
// reader can be scheduled above it).
#define MOE_LOAD16(reg, ptr, off) \
    asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(reg) : "v"(ptr), "n"(off) : "memory")
#define MOE_TIE_SET(r0, r1, r2, r3) asm volatile("" : "+v"(r0), "+v"(r1), "+v"(r2), "+v"(r3)::"memory")

__device__ __forceinline__ int lds_off(int row, int chunk)   // byte offset of logical 16-byte chunk of a row
{
    return row * 128 + ((chunk ^ (row & 7)) << 4);
}

struct GemmArgs {
    const uint16_t *A;            // gate/up: x [T,K]; down: act [P,K]
    const uint16_t *W;            // [E, w_rows, K]
    const int32_t *sorted_pair;   // gate/up only
    uint16_t *out;                // gate/up: act [P,n_out]; down: y [P,n_out]
    int K, n_out, top_k;
};

// Everything after the (tile, column slab) decision, instantiated per active row-block count NB.
template <int MB_MAX, int D, bool SWIGLU, int NB>
__device__ __forceinline__ void gemm_tile(const GemmArgs &g, const moe_tile &tile, int ct, unsigned char *smem)
{
    constexpr int S = D + 1;                                  // register sets == LDS stages
    constexpr int STAGE_BYTES = MB_MAX * 16 * 128;
    constexpr int A_PASS_MAX = (MB_MAX * 2 + GM_WAVES - 1) / GM_WAVES;   // 8-row copy passes per wavefront
    constexpr int SLAB = SWIGLU ? 16 : 32;                    // output columns per wavefront

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, lets the compiler keep it scalar
    const int l16 = lane & 15, lq = lane >> 4;
    const int rows = tile.rows;
    const int K = g.K, n_out = g.n_out;
    const int nk = K / GM_BK;

    // ---- weight row pointers (two 16-row blocks per wavefront) ----------------
    const int col0 = ct * (SLAB * GM_WAVES) + wave * SLAB;    // first output column of this wavefront
    const int w_rows = SWIGLU ? 2 * n_out : n_out;
    int wrow0, wrow1;
    if constexpr (SWIGLU) {
        const int c = min(col0 + l16, n_out - 1);             // clamp: columns past the end are never stored
        wrow0 = c;                                            // gate row
        wrow1 = n_out + c;                                    // matching up row
    } else {
        wrow0 = min(col0 + l16, n_out - 1);
        wrow1 = min(col0 + 16 + l16, n_out - 1);
    }
    const uint16_t *wbase = g.W + (size_t)tile.expert * w_rows * K + lq * 8;
    const uint16_t *wp0 = wbase + (size_t)wrow0 * K;
    const uint16_t *wp1 = wbase + (size_t)wrow1 * K;

    // ---- token row pointers for the global -> LDS copies -----------------------
    // copy pass p moves LDS rows 8p..8p+7 (lane l: row 8p + l/8, physical chunk l%8)
    const int rows16 = NB * 16;
    int a_cnt = 0;
    const uint16_t *a_ptr[A_PASS_MAX];
    int a_dst[A_PASS_MAX];
#pragma unroll
    for (int i = 0; i < A_PASS_MAX; ++i) {
        const int p = wave + GM_WAVES * i;
        if (8 * p < rows16) ++a_cnt;
        int r = 8 * p + (lane >> 3);
        r = r < rows ? r : rows - 1;                          // padded rows repeat the last row; never stored
        size_t src;
        if constexpr (SWIGLU) src = (size_t)(g.sorted_pair[tile.row0 + r] / g.top_k);
        else src = (size_t)(tile.row0 + r);
        a_ptr[i] = g.A + src * K + (((lane & 7) ^ (lane >> 3)) << 3);
        a_dst[i] = p * 1024;
    }

    f32x4 acc[NB][2];
#pragma unroll
    for (int m = 0; m < NB; ++m)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[m][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 wq[S][2][2];                                        // [set][block][half of the K step]

    // issue the loads of K step `s` (clamped to the last step: the tail prefetches are dummies)
#define MOE_ISSUE(s, set)                                                                              \
    {                                                                                                  \
        const int k0_ = min((s), nk - 1) * GM_BK;                                                      \
        unsigned char *dst_ = smem + ((s) % S) * STAGE_BYTES;                                          \
        _Pragma("unroll") for (int i = 0; i < A_PASS_MAX; ++i)                                         \
            if (i < a_cnt)                                                                             \
                __builtin_amdgcn_global_load_lds(MOE_GLOBAL_PTR(a_ptr[i] + k0_), MOE_LDS_PTR(dst_ + a_dst[i]), 16, 0, 0); \
        MOE_LOAD16(wq[set][0][0], wp0 + k0_, 0);                                                       \
        MOE_LOAD16(wq[set][0][1], wp0 + k0_, 64);                                                      \
        MOE_LOAD16(wq[set][1][0], wp1 + k0_, 0);                                                       \
        MOE_LOAD16(wq[set][1][1], wp1 + k0_, 64);                                                      \
    }

    // prologue: D steps in flight
#pragma unroll
    for (int d = 0; d < D; ++d) MOE_ISSUE(d, d)

    for (int s0 = 0; s0 < nk; s0 += S) {
#pragma unroll
        for (int j = 0; j < S; ++j) {
            const int s = s0 + j;
            // Loads of step s (issued D slots ago) must have landed; the D-1 newer slots may stay
            // in flight.  Every slot of this wavefront is GM_B_LOADS + a_cnt loads, returned in order.
switch (a_cnt) {
            case 0: MOE_WAIT_VMCNT((D - 1) * (GM_B_LOADS + 0)); break;
            case 1: MOE_WAIT_VMCNT((D - 1) * (GM_B_LOADS + 1)); break;
            case 2: MOE_WAIT_VMCNT((D - 1) * (GM_B_LOADS + 2)); break;
            case 3: MOE_WAIT_VMCNT((D - 1) * (GM_B_LOADS + 3)); break;
            default: MOE_WAIT_VMCNT((D - 1) * (GM_B_LOADS + 4)); break;
            }
            MOE_TIE_SET(wq[j][0][0], wq[j][0][1], wq[j][1][0], wq[j][1][1]);
            asm volatile("s_barrier" ::: "memory");           // stage s complete for everyone; stage s-1 free
            MOE_ISSUE(s + D, (j + D) % S)
            __builtin_amdgcn_sched_barrier(0);
            if (s < nk) {
                const unsigned char *sa = smem + (s % S) * STAGE_BYTES;
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const bf16x8 w0 = __builtin_bit_cast(bf16x8, wq[j][0][kk]);
                    const bf16x8 w1 = __builtin_bit_cast(bf16x8, wq[j][1][kk]);
#pragma unroll
                    for (int m = 0; m < NB; ++m) {
                        const bf16x8 t = *reinterpret_cast<const bf16x8 *>(sa + lds_off(m * 16 + l16, kk * 4 + lq));
                        acc[m][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w0, t, acc[m][0], 0, 0, 0);
                        acc[m][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w1, t, acc[m][1], 0, 0, 0);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    MOE_WAIT_VMCNT(0);                                        // dummy tail prefetches must not outlive the LDS ring
#undef MOE_ISSUE

    // ---- epilogue: lane l holds, for token l%16 of each row block, output columns 4*(l/16)..+3
    // of each of its two weight blocks
#pragma unroll
    for (int m = 0; m < NB; ++m) {
        const int r = m * 16 + l16;
        if (r >= rows) continue;
        uint16_t *orow = g.out + (size_t)(tile.row0 + r) * n_out;
        if constexpr (SWIGLU) {
            const int c = col0 + lq * 4;
            if (c < n_out) {
                float a[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float gt = acc[m][0][v], up = acc[m][1][v];
                    a[v] = gt / (1.f + __expf(-gt)) * up;
                }
                uint2 o;
                o.x = pack_bf16x2(a[0], a[1]);
                o.y = pack_bf16x2(a[2], a[3]);
                *reinterpret_cast<uint2 *>(orow + c) = o;
            }
        } else {
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int c = col0 + b * 16 + lq * 4;
                if (c < n_out) {
                    uint2 o;
                    o.x = pack_bf16x2(acc[m][b][0], acc[m][b][1]);
                    o.y = pack_bf16x2(acc[m][b][2], acc[m][b][3]);
                    *reinterpret_cast<uint2 *>(orow + c) = o;
                }
            }
        }
    }
}

template <int MB_MAX, int D, bool SWIGLU, int NB>
__device__ __forceinline__ void dispatch_blocks(int nb, const GemmArgs &g, const moe_tile &tile, int ct,
                                                unsigned char *smem)
{
    if constexpr (NB > MB_MAX) {
        return;
    } else {
        // row-block counts are rounded up to even above 4 to bound the number of instantiations
        constexpr int NEXT = NB < 4 ? NB + 1 : NB + 2;
        if (nb <= NB) gemm_tile<MB_MAX, D, SWIGLU, NB>(g, tile, ct, smem);
        else dispatch_blocks<MB_MAX, D, SWIGLU, NEXT>(nb, g, tile, ct, smem);
    }
}

template <int MB_MAX, int D, bool SWIGLU>
__global__ __launch_bounds__(GM_THREADS) void grouped_gemm_bf16_kernel(GemmArgs g, const moe_tile *__restrict__ tiles,
                                                                       const int32_t *__restrict__ ntiles,
                                                                       int col_tiles)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int total = *ntiles * col_tiles;
    const int per_xcd = ceil_div(total, GM_XCDS);
    const int slot = blockIdx.x / GM_XCDS;
    if (slot >= per_xcd) return;
    const int work = (blockIdx.x % GM_XCDS) * per_xcd + slot;
    if (work >= total) return;
    const moe_tile head = tiles[work / col_tiles];
    const int local = work - head.first * col_tiles;           // index inside this expert's work
    const int ct = local / head.count;                         // column slab
    const moe_tile tile = tiles[head.first + local % head.count];
    const int nb = ceil_div(tile.rows, 16);
    dispatch_blocks<MB_MAX, D, SWIGLU, 1>(nb, g, tile, ct, smem);
}

template <int MB_MAX, int D, bool SWIGLU>
int launch_variant(const GemmArgs &g, const moe_tile *tiles, const int32_t *ntiles, int max_tiles, hipStream_t s)
{
    constexpr int cols_per_wg = (SWIGLU ? 16 : 32) * GM_WAVES;
    const int col_tiles = ceil_div(g.n_out, cols_per_wg);
    const int blocks = ceil_div(max_tiles * col_tiles, GM_XCDS) * GM_XCDS;
    const size_t lds = (size_t)(D + 1) * MB_MAX * 16 * 128;
    auto kern = grouped_gemm_bf16_kernel<MB_MAX, D, SWIGLU>;
    static bool attr_done = false;          // raise the dynamic-LDS limit once per variant
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { set_last_hip_error(e); return MOE_ERR_HIP; }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(GM_THREADS), lds, s, g, tiles, ntiles, col_tiles);
    return check_launch();
}

template <bool SWIGLU>
int launch_by_tile_rows(int tile_rows, const GemmArgs &g, const moe_tile *tiles, const int32_t *ntiles,
                        int max_tiles, hipStream_t s)
{
    switch (tile_rows) {
    case 256: return launch_variant<16, 3, SWIGLU>(g, tiles, ntiles, max_tiles, s);
    case 128: return launch_variant<8, 3, SWIGLU>(g, tiles, ntiles, max_tiles, s);
    case 64:  return launch_variant<4, 3, SWIGLU>(g, tiles, ntiles, max_tiles, s);
    case 32:  return launch_variant<2, 3, SWIGLU>(g, tiles, ntiles, max_tiles, s);
    case 16:  return launch_variant<1, 3, SWIGLU>(g, tiles, ntiles, max_tiles, s);
    default:  return MOE_ERR_UNSUPPORTED;
    }
}

}  // namespace

int launch_gemm_swiglu(const moe_config &c, int tile_rows, int max_tiles, const void *x,
                       const float *, const void *w1, const float *, const int32_t *sorted_pair,
                       const moe_tile *tiles, const int32_t *ntiles, void *act, float *, hipStream_t s)
{
    if (c.dtype != MOE_DTYPE_BF16) return MOE_ERR_UNSUPPORTED;
    GemmArgs g{static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(w1), sorted_pair,
               static_cast<uint16_t *>(act), c.H, c.I, c.top_k};
    return launch_by_tile_rows<true>(tile_rows, g, tiles, ntiles, max_tiles, s);
}

int launch_gemm_down(const moe_config &c, int tile_rows, int max_tiles, const void *act, const float *,
                     const void *w2, const float *, const moe_tile *tiles, const int32_t *ntiles, void *y,
                     hipStream_t s)
{
    if (c.dtype != MOE_DTYPE_BF16) return MOE_ERR_UNSUPPORTED;
    GemmArgs g{static_cast<const uint16_t *>(act), static_cast<const uint16_t *>(w2), nullptr,
               static_cast<uint16_t *>(y), c.I, c.H, c.top_k};
    return launch_by_tile_rows<false>(tile_rows, g, tiles, ntiles, max_tiles, s);
}

}  // namespace moe
