// Streaming-read probe: what this chip reads from HBM with the access pattern of the grouped GEMMs'
// weight stream, and nothing else going on.  A stand-alone program (not part of the library):
//
//     python -m paper_2602_19128_amd.build --probe && paper_2602_19128_amd/probe/stream_probe
//
// It is the yardstick the GEMM kernels are held against: the figures it prints bound any weight
// stream whatever the kernel does (the nominal 8 TB/s are not reachable by reads).
//
// Every workgroup has 8 wavefronts; a wavefront owns 32 rows of `stride` bytes and walks them 128
// bytes at a time, four instructions of 8 rows x 128 B per step (the grouped GEMM's weight copy), or
// reads 1 KiB contiguous per instruction.  DEPTH steps are in flight per wavefront.  Loads go
// straight to LDS (as in the kernels) or into registers.  Variants: non-temporal or cacheable loads,
// one or two workgroups per compute unit, a grid smaller than the chip (the rate one compute unit
// reaches when the chip is not saturated), and some workgroups reading what a neighbour on the same
// XCD reads at the same time (second row tiles of one expert).
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define CK(x)                                                                                   \
    do {                                                                                        \
        hipError_t e_ = (x);                                                                    \
        if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } \
    } while (0)

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// One 1 KiB load of a wavefront: to LDS byte address `lds_dst` (LDS true) or into `reg`.
template <bool LDS>
__device__ __forceinline__ void load16(const unsigned char *p, uint32_t lds_dst, u32x4 &reg, int nt)
{
    if (LDS) {
        if (nt) asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds_dst), "v"(p) : "memory", "m0");
        else asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_dst), "v"(p) : "memory", "m0");
    } else {
        if (nt) asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(reg) : "v"(p) : "memory");
        else asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(reg) : "v"(p) : "memory");
    }
}

// total: bytes of the buffer that are read (a multiple of 32 * stride is used); stride: bytes per row, a
// multiple of 128 * DEPTH; dup: 0, or N = of every N workgroups of an XCD (blockIdx % 8) the second reads
// what the first reads.
template <bool LDS, bool ROWS, int DEPTH, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void stream_kernel(const unsigned char *__restrict__ src, size_t total, int stride,
                                                            int nt, int dup, unsigned *sink)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int bid = blockIdx.x, nb = gridDim.x;
    if (dup > 0) {
        const int x = bid % 8, j = bid / 8, per = nb / 8;
        const int grp = j / dup, pos = j % dup;
        bid = (grp * (dup - 1) + (pos == 0 ? 0 : pos - 1)) * 8 + x;      // stream number: positions 0 and 1 share one
        nb = (per / dup) * (dup - 1) * 8;
    }
    const size_t gw = (size_t)bid * WAVES + wave, nw = (size_t)nb * WAVES;
    const size_t item_bytes = (size_t)32 * stride;
    const int steps = stride / 128;
    const size_t items = total / item_bytes;
    const uint32_t ring = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)(lds) + wave * DEPTH * 4096);
    u32x4 v[DEPTH][4];
    unsigned acc = 0;
    for (size_t it = gw; it < items; it += nw) {
        const unsigned char *base = src + it * item_bytes;
        auto issue = [&](int s, int slot) __attribute__((always_inline)) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned char *p = ROWS ? base + (size_t)(q * 8 + (lane >> 3)) * stride + (size_t)s * 128 + (lane & 7) * 16
                                              : base + ((size_t)s * 4 + q) * 1024 + lane * 16;
                load16<LDS>(p, ring + slot * 4096 + q * 1024, v[slot][q], nt);
            }
        };
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) issue(s, s);
        for (int s0 = 0; s0 < steps; s0 += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {                  // step s0 + d sits in slot d (steps % DEPTH == 0)
                wait_vmcnt<4 * (DEPTH - 1)>();
                if (!LDS) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) { asm volatile("" : "+v"(v[d][q])); acc ^= v[d][q].x; }
                }
                if (s0 + d + DEPTH < steps) issue(s0 + d + DEPTH, d);
                else wait_vmcnt<0>();                          // the end of an item: no bookkeeping of a shrinking queue
            }
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;                     // keeps the register loads alive
}

static int g_cus = 256;

template <bool LDS, bool ROWS, int DEPTH>
void run(const char *what, const unsigned char *buf, size_t total, int stride, int nt, int wgs_per_cu, int cus, int dup, unsigned *sink)
{
    constexpr int WAVES = 8;
    auto k = stream_kernel<LDS, ROWS, DEPTH, WAVES>;
    const size_t lds = LDS ? (size_t)WAVES * DEPTH * 4096 : 0;
    CK(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    const int grid = cus * wgs_per_cu;
    float best = 1e30f;
    for (int rep = 0; rep < 4; ++rep) {                        // the first launch warms up
        CK(hipEventRecord(a));
        hipLaunchKernelGGL(k, dim3(grid), dim3(WAVES * 64), lds, 0, buf, total, stride, nt, dup, sink);
        CK(hipGetLastError());
        CK(hipEventRecord(b));
        CK(hipEventSynchronize(b));
        float ms;
        CK(hipEventElapsedTime(&ms, a, b));
        if (rep && ms < best) best = ms;
    }
    const double bytes = (double)(total / ((size_t)32 * stride)) * 32 * stride;   // each byte once (shared streams counted once)
    printf("| %s | %d | %s | %d | %d of %d | %s | %.0f | %.2f | %.1f |\n", what, stride, nt ? "non-temporal" : "cacheable", wgs_per_cu, cus, g_cus,
           dup ? (dup == 2 ? "1 in 2" : dup == 4 ? "1 in 4" : "1 in 8") : "-", best * 1e3, bytes / best / 1e9, bytes / best / 1e6 / cus);
    fflush(stdout);
    CK(hipEventDestroy(a));
    CK(hipEventDestroy(b));
}

int main()
{
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    g_cus = prop.multiProcessorCount;
    const size_t total = (size_t)12 << 30;
    unsigned char *buf;
    unsigned *sink;
    CK(hipMalloc(&buf, total));
    CK(hipMalloc(&sink, 64));
    CK(hipMemset(buf, 1, total));
    CK(hipDeviceSynchronize());
    const int S = 14336, cu = g_cus;                           // 7168 bf16: the gate/up weight rows of the DeepSeek-shaped configs
    printf("device: %s, %d compute units; %zu GiB read per launch, 8 wavefronts per workgroup, 4 KiB per wavefront and step\n\n", prop.name, cu,
           total >> 30);
    printf("| loads | row stride B | policy | workgroups per CU | CUs busy | shared streams | us | TB/s (unique bytes) | GB/s per CU |\n|---|---|---|---|---|---|---|---|---|\n");
    run<true, true, 2>("to LDS, 8 rows x 128 B, 2 steps deep", buf, total, S, 1, 1, cu, 0, sink);
    run<true, true, 4>("to LDS, 8 rows x 128 B, 4 steps deep", buf, total, S, 1, 1, cu, 0, sink);
    run<false, true, 2>("to registers, 8 rows x 128 B, 2 steps deep", buf, total, S, 1, 1, cu, 0, sink);
    run<false, true, 4>("to registers, 8 rows x 128 B, 4 steps deep", buf, total, S, 1, 1, cu, 0, sink);
    run<true, true, 2>("to LDS, 8 rows x 128 B, 2 steps deep", buf, total, S, 1, 2, cu, 0, sink);
    run<true, false, 2>("to LDS, 1 KiB contiguous, 2 steps deep", buf, total, S, 1, 1, cu, 0, sink);
    run<false, false, 4>("to registers, 1 KiB contiguous, 4 steps deep", buf, total, S, 1, 2, cu, 0, sink);
    run<true, true, 2>("to LDS, 8 rows x 128 B, 2 steps deep", buf, total, S, 0, 1, cu, 0, sink);
    run<false, false, 4>("to registers, 1 KiB contiguous, 4 steps deep", buf, total, S, 0, 2, cu, 0, sink);
    run<true, true, 2>("to LDS, 8 rows x 128 B, 2 steps deep", buf, total, 4096, 1, 1, cu, 0, sink);
    run<true, true, 4>("to LDS, 8 rows x 128 B, 4 steps deep", buf, total, 4096, 1, 1, cu, 0, sink);
    run<true, true, 2>("to LDS, 8 rows x 128 B, 2 steps deep", buf, total / 8, S, 1, 1, cu / 8, 0, sink);
    run<true, true, 4>("to LDS, 8 rows x 128 B, 4 steps deep", buf, total / 8, S, 1, 1, cu / 8, 0, sink);
    run<true, true, 2>("to LDS, 8 rows x 128 B, 2 steps deep", buf, total / 2, S, 1, 1, cu / 2, 0, sink);
    run<true, true, 2>("to LDS, 8 rows x 128 B, 2 steps deep", buf, total, S, 1, 1, cu, 8, sink);
    run<true, true, 2>("to LDS, 8 rows x 128 B, 2 steps deep", buf, total, S, 1, 1, cu, 4, sink);
    run<true, true, 2>("to LDS, 8 rows x 128 B, 2 steps deep", buf, total, S, 1, 1, cu, 2, sink);
    run<true, true, 2>("to LDS, 8 rows x 128 B, 2 steps deep", buf, total, S, 0, 1, cu, 4, sink);
    CK(hipFree(buf));
    CK(hipFree(sink));
    return 0;
}
