// Grouped expert GEMMs on the bf16 matrix cores (paper Sec. 4.5 "Expert FFN
// computation": tensor-core tiles with double buffering, empty experts skipped).
//
// Both GEMMs are C[m,n] = sum_k A[m,k] * W[e,n,k] with A rows and W rows contiguous
// along k, so both operands are fetched as 16-byte pieces of a row.  A workgroup of
// four wavefronts owns one row tile of one expert times BN weight rows.  Each K
// step of 64 elements is one 128-byte LDS row per tile row.  Global memory is copied
// straight into LDS (global_load_lds, 16 bytes per lane, no register staging): the
// copy of step kt+1 is issued before the MFMAs of step kt and only waited for at the
// barrier that ends the step, so HBM latency hides behind the matrix cores.
//
// LDS layout: the hardware places lane l of a direct load at base + 16*l, so a
// wavefront fills 8 consecutive 128-byte rows.  To keep the 16-byte MFMA fragment
// reads conflict-free, physical chunk pc of row r holds logical chunk pc ^ (r & 7);
// the permutation is applied on the global-address side of the copy.
//
//   gate/up GEMM: A rows are gathered from x through the sorted pair list; a wavefront
//                 holds matching gate and up columns in the same lanes, so
//                 act = silu(g) * u is applied to the accumulators in registers.
//   down GEMM   : A = act rows (already contiguous per expert).
//
// Workgroups are numbered so that each XCD (own L2) gets a contiguous range of the
// (expert, column tile) work: all row tiles that need one weight tile run next to
// each other on one XCD and the weight tile is fetched from HBM once.
#include "moe_internal.hpp"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int GM_BK = 64;                 // k elements per LDS stage (one 128-byte row)
constexpr int GM_THREADS = 256;
constexpr int GM_XCDS = 8;

#define MOE_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define MOE_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

__device__ inline int lds_off(int row, int chunk)      // byte offset of logical 16-byte chunk `chunk` of `row`
{
    return row * 128 + ((chunk ^ (row & 7)) << 4);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool SWIGLU>
__global__ __launch_bounds__(GM_THREADS) void grouped_gemm_bf16_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, const int32_t *__restrict__ sorted_pair,
    const moe_tile *__restrict__ tiles, const int32_t *__restrict__ ntiles, uint16_t *__restrict__ out,
    int K, int n_out, int top_k, int col_tiles)
{
    static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;      // wavefront tile
    constexpr int MI = WTM / 32, NI = WTN / 32;                // 32x32 MFMA blocks per wavefront
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wavefront tile is made of 32x32 blocks");
    static_assert(!SWIGLU || NI % 2 == 0, "gate and up halves live in one wavefront");
    constexpr int A_PASS = BM / 32, B_PASS = BN / 32;          // one pass = 32 rows = 4 wavefronts x 8 rows
    constexpr int STAGE_BYTES = (BM + BN) * 128;

    extern __shared__ __align__(16) unsigned char smem[];

    // ---- which (row tile, column tile) ------------------------------------
    const int total = *ntiles * col_tiles;
    const int per_xcd = ceil_div(total, GM_XCDS);
    const int slot = blockIdx.x / GM_XCDS;
    if (slot >= per_xcd) return;
    const int work = (blockIdx.x % GM_XCDS) * per_xcd + slot;
    if (work >= total) return;
    const moe_tile head = tiles[work / col_tiles];
    const int local = work - head.first * col_tiles;           // index inside this expert's work
    const int ct = local / head.count;                         // column tile
    const moe_tile tile = tiles[head.first + local % head.count];
    const int rows = tile.rows;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int lrow = tid >> 3;                                 // loader: row inside a 32-row pass
    const int lchunk = (tid & 7) ^ (lrow & 7);                 // logical chunk that lands on this lane's LDS slot

    // ---- global row pointers of the loader ---------------------------------
    const int w_rows = SWIGLU ? 2 * n_out : n_out;
    const uint16_t *wbase = W + (size_t)tile.expert * w_rows * K;
    const uint16_t *a_ptr[A_PASS];
    const uint16_t *b_ptr[B_PASS];
#pragma unroll
    for (int i = 0; i < A_PASS; ++i) {
        int r = lrow + 32 * i;
        r = r < rows ? r : rows - 1;                           // clamp: result of padded rows is never stored
        size_t src;
        if constexpr (SWIGLU) src = (size_t)(sorted_pair[tile.row0 + r] / top_k);
        else src = (size_t)(tile.row0 + r);
        a_ptr[i] = A + src * K + lchunk * 8;
    }
#pragma unroll
    for (int i = 0; i < B_PASS; ++i) {
        const int r = lrow + 32 * i;                           // LDS row of the weight tile
        int n;
        if constexpr (SWIGLU) {
            // wavefront wn owns act columns ct*BN/2 + wn*WTN/2 + [0,WTN/2): first its gate rows, then its up rows
            const int w_of_r = r / WTN, in_w = r % WTN;
            const int col = ct * (BN / 2) + w_of_r * (WTN / 2) + (in_w % (WTN / 2));
            n = (in_w < WTN / 2) ? col : n_out + col;
            if (col >= n_out) n = 0;
        } else {
            n = ct * BN + r;
            if (n >= n_out) n = 0;
        }
        b_ptr[i] = wbase + (size_t)n * K + lchunk * 8;
    }

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = K / GM_BK;
    // LDS destination of this wavefront inside a 32-row pass (the hardware adds 16 * lane)
    unsigned char *const wave_dst = smem + wave * 1024;

#define MOE_COPY_STAGE(k0, buf)                                                                         \
    {                                                                                                   \
        unsigned char *da_ = wave_dst + (buf) * STAGE_BYTES;                                            \
        unsigned char *db_ = da_ + BM * 128;                                                            \
        _Pragma("unroll") for (int i = 0; i < A_PASS; ++i)                                              \
            __builtin_amdgcn_global_load_lds(MOE_GLOBAL_PTR(a_ptr[i] + (k0)), MOE_LDS_PTR(da_ + i * 4096), 16, 0, 0); \
        _Pragma("unroll") for (int i = 0; i < B_PASS; ++i)                                              \
            __builtin_amdgcn_global_load_lds(MOE_GLOBAL_PTR(b_ptr[i] + (k0)), MOE_LDS_PTR(db_ + i * 4096), 16, 0, 0); \
    }
#define MOE_COMPUTE_STAGE(buf)                                                                          \
    {                                                                                                   \
        const unsigned char *sa_ = smem + (buf) * STAGE_BYTES + (wm * WTM) * 128;                       \
        const unsigned char *sb_ = smem + (buf) * STAGE_BYTES + BM * 128 + (wn * WTN) * 128;            \
        _Pragma("unroll") for (int kk = 0; kk < GM_BK / 16; ++kk) {                                     \
            const int chunk = kk * 2 + (lane >> 5);                                                     \
            bf16x8 af[MI], bfr[NI];                                                                     \
            _Pragma("unroll") for (int i = 0; i < MI; ++i)                                              \
                af[i] = *reinterpret_cast<const bf16x8 *>(sa_ + lds_off(i * 32 + (lane & 31), chunk));  \
            _Pragma("unroll") for (int j = 0; j < NI; ++j)                                              \
                bfr[j] = *reinterpret_cast<const bf16x8 *>(sb_ + lds_off(j * 32 + (lane & 31), chunk)); \
            _Pragma("unroll") for (int i = 0; i < MI; ++i)                                              \
                _Pragma("unroll") for (int j = 0; j < NI; ++j)                                          \
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0); \
        }                                                                                               \
    }

    // K loop.  __syncthreads() waits for this wavefront's outstanding copies (it carries a
    // workgroup-scope fence) and then for the other wavefronts, so after it every copy into
    // the next buffer has landed and every read of the current buffer is done.
    MOE_COPY_STAGE(0, 0)
    __syncthreads();
    for (int kt = 0; kt + 1 < nk; ++kt) {
        MOE_COPY_STAGE((kt + 1) * GM_BK, (kt + 1) & 1)
        MOE_COMPUTE_STAGE(kt & 1)
        __syncthreads();
    }
    MOE_COMPUTE_STAGE((nk - 1) & 1)
#undef MOE_COPY_STAGE
#undef MOE_COMPUTE_STAGE

    // ---- epilogue: accumulator element v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32
    const int lcol = lane & 31, lrow4 = (lane >> 5) * 4;
    if constexpr (SWIGLU) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI / 2; ++j) {
                const int col = ct * (BN / 2) + wn * (WTN / 2) + j * 32 + lcol;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = wm * WTM + i * 32 + (v >> 2) * 8 + lrow4 + (v & 3);
                    if (r < rows && col < n_out) {
                        const float g = acc[i][j][v], u = acc[i][j + NI / 2][v];
                        const float a = g / (1.f + __expf(-g)) * u;
                        out[(size_t)(tile.row0 + r) * n_out + col] = (uint16_t)f32_to_bf16_bits(a);
                    }
                }
            }
    } else {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int col = ct * BN + wn * WTN + j * 32 + lcol;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = wm * WTM + i * 32 + (v >> 2) * 8 + lrow4 + (v & 3);
                    if (r < rows && col < n_out)
                        out[(size_t)(tile.row0 + r) * n_out + col] = (uint16_t)f32_to_bf16_bits(acc[i][j][v]);
                }
            }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool SWIGLU>
int launch_variant(const uint16_t *A, const uint16_t *W, const int32_t *sorted_pair, const moe_tile *tiles,
                   const int32_t *ntiles, uint16_t *out, int K, int n_out, int top_k, int max_tiles,
                   hipStream_t s)
{
    constexpr int cols_per_tile = SWIGLU ? BN / 2 : BN;
    const int col_tiles = ceil_div(n_out, cols_per_tile);
    const int blocks = ceil_div(max_tiles * col_tiles, GM_XCDS) * GM_XCDS;
    const size_t lds = 2 * (size_t)(BM + BN) * 128;
    auto kern = grouped_gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, SWIGLU>;
    static bool attr_done = false;          // raise the dynamic-LDS limit once per variant
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { set_last_hip_error(e); return MOE_ERR_HIP; }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(GM_THREADS), lds, s, A, W, sorted_pair, tiles, ntiles, out, K,
                       n_out, top_k, col_tiles);
    return check_launch();
}

template <bool SWIGLU>
int launch_by_tile_rows(int tile_rows, const uint16_t *A, const uint16_t *W, const int32_t *sorted_pair,
                        const moe_tile *tiles, const int32_t *ntiles, uint16_t *out, int K, int n_out,
                        int top_k, int max_tiles, hipStream_t s)
{
    switch (tile_rows) {
    case 128: return launch_variant<128, 128, 2, 2, SWIGLU>(A, W, sorted_pair, tiles, ntiles, out, K, n_out, top_k, max_tiles, s);
    case 64:  return launch_variant<64, 128, 2, 2, SWIGLU>(A, W, sorted_pair, tiles, ntiles, out, K, n_out, top_k, max_tiles, s);
    case 32:  return launch_variant<32, 256, 1, 4, SWIGLU>(A, W, sorted_pair, tiles, ntiles, out, K, n_out, top_k, max_tiles, s);
    default:  return MOE_ERR_UNSUPPORTED;
    }
}

}  // namespace

int launch_gemm_swiglu(const moe_config &c, int tile_rows, int max_tiles, const void *x,
                       const float *, const void *w1, const float *, const int32_t *sorted_pair,
                       const moe_tile *tiles, const int32_t *ntiles, void *act, float *, hipStream_t s)
{
    if (c.dtype != MOE_DTYPE_BF16) return MOE_ERR_UNSUPPORTED;
    return launch_by_tile_rows<true>(tile_rows, static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(w1),
                                     sorted_pair, tiles, ntiles, static_cast<uint16_t *>(act), c.H, c.I, c.top_k,
                                     max_tiles, s);
}

int launch_gemm_down(const moe_config &c, int tile_rows, int max_tiles, const void *act, const float *,
                     const void *w2, const float *, const moe_tile *tiles, const int32_t *ntiles, void *y,
                     hipStream_t s)
{
    if (c.dtype != MOE_DTYPE_BF16) return MOE_ERR_UNSUPPORTED;
    return launch_by_tile_rows<false>(tile_rows, static_cast<const uint16_t *>(act), static_cast<const uint16_t *>(w2),
                                      nullptr, tiles, ntiles, static_cast<uint16_t *>(y), c.I, c.H, c.top_k,
                                      max_tiles, s);
}

}  // namespace moe
