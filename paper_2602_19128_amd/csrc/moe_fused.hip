// Single-launch forward for the latency-bound regime (paper Sec. 4.5, "Expert FFN computation":
// the paper contrasts one persistent kernel with a pipeline of several launches; for layers whose
// whole forward is a few microseconds of work the launches themselves are most of the time).
//
// One persistent kernel runs the steps of the layer as phases, every workgroup taking a share of
// each phase, with a grid-wide barrier where a phase needs the previous one complete:
//
//   route      the same device code as the stand-alone routing kernels (few experts: one or four
//              wavefronts per token do logits and top-k; otherwise LDS-tiled partial logits, a
//              barrier, then one wavefront per token)
//   barrier
//   sort-scatter   every workgroup builds the whole permutation, tile list and schedule in its own
//              LDS and writes it out (all workgroups write the same values), so no barrier is
//              needed before the GEMMs
//   gate/up GEMM   the schedule is walked exactly as the stand-alone kernel walks it (static
//              assignment of items to workgroups by their index: no work-queue counter)
//   barrier
//   down GEMM
//   barrier
//   combine
//
// Every phase is the device code of the multi-launch path, instantiated for the kernel shapes that
// path picks for the same problem, so the results are the same bits.
//
// Only every eighth workgroup of the launch takes part (workgroups are handed to the XCDs in turn), so
// a launch normally sits on one XCD, at most 32 workgroups, and its barriers stay inside one L2.
// The barriers use a few counters in static device memory (zero between launches: the last
// workgroup to leave a launch clears them).  A wait is bounded (about two seconds of the constant
// 100 MHz clock): a workgroup that gives up counts a time-out, goes on, still arrives at every later
// barrier and still leaves, so the counters return to zero and the kernel always drains; results of
// such a launch are undefined and moe_single_launch_timeouts() reports it.  All workgroups of a
// launch are resident at once (the grid never exceeds the number of compute units, and one
// workgroup of this kernel always fits a free compute unit).  Launches of this kernel share the
// counters, so two of them must not overlap on one device; launches on one stream never do.
#include "moe_combine_device.hpp"
#include "moe_gemm_kernel.hpp"
#include "moe_permute_device.hpp"
#include "moe_route_device.hpp"

namespace moe {
namespace {

constexpr int FZ_THREADS = 256;
constexpr int FZ_WAVES = FZ_THREADS / kWave;
constexpr int FZ_BARRIERS = 4;
constexpr unsigned long long FZ_WAIT_TICKS = 200000000ull;    // bounded wait: ~2 s of the 100 MHz wall clock
constexpr int FZ_MAX_PAIRS = 1024;                            // every workgroup sorts all pairs itself
constexpr int FZ_MAX_EXPERTS = FZ_THREADS;                    // the sort-scatter gives one thread to every local expert

// Barrier counters, each on a cache line of its own.
struct alignas(128) SyncWord { unsigned v; unsigned pad[31]; };
struct GridSync {
    SyncWord arrived[FZ_BARRIERS];     // workgroups that reached barrier b of the running launch
    SyncWord departed;                 // workgroups that finished the running launch
    SyncWord xcc_mask;                 // bit x: a workgroup of the running launch runs on XCD x
    SyncWord timeouts;                 // waits that were given up since the library was loaded
};
static __device__ GridSync g_sync;     // all zero between launches (except timeouts)

enum RouteMode { ROUTE_FEW = 0, ROUTE_FEW_SPLIT = 1, ROUTE_TILED = 2 };

struct FusedArgs {
    // routing
    const void *x;
    const float *router_w, *bias;
    float *zpart;
    int32_t *ids;
    float *w;
    TopkParams tp;
    RouteGrid rg;
    int route_mode, epl, H;
    // sort-scatter
    int P, EL, e_first, tile_rows, max_tiles;
    int32_t *offsets, *sorted_pair, *inv;
    moe_tile *tiles;
    int32_t *sched;
    // expert GEMMs
    GemmArgs g1, g2;
    int col_tiles1, col_tiles2, whole_ranges;
    // combine
    uint16_t *out;
    int T, out_H, top_k;
};

__device__ __forceinline__ unsigned xcc_id()
{
    unsigned v;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID, 0, 4)" : "=s"(v));
    return v;
}

// Read-modify-write that returns the value the L2 held and is complete when it returns (a plain
// load could be served by the compute unit's own cache; an atomic without a result may still be on
// its way when the next one is issued).  bits = 0 reads the word.
__device__ __forceinline__ unsigned or_in_l2(unsigned *p, unsigned bits)
{
    unsigned old;
    asm volatile("global_atomic_or %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)" : "=v"(old) : "v"(p), "v"(bits) : "memory");
    return old;
}

// All workgroups of the launch meet here.  Writes made before the barrier by any thread of any
// workgroup are visible after it to every thread of every workgroup.
//
// The workgroup barrier in front completes every wavefront's stores: they are in this XCD's L2
// then.  Thread 0 arrives and polls with atomics, then drops what the compute unit's cache (and the
// L2, of other XCDs' data) holds, once for the whole workgroup.  When the workgroups run on
// several XCDs, thread 0 first writes its L2's dirty lines back (`spread`); when they all share one
// XCD - the normal case, see the kernel - they share its L2 and nothing has to be written back.
// Whether they do is established by the first barrier of a launch, which every workgroup enters
// after publishing the id of its XCD.  (Measured: cache operations per thread instead of per
// workgroup 30 us per barrier; per workgroup with the workgroups spread over eight XCDs about 5 us;
// on one XCD without the write-back 1..2 us including the wait for the slowest workgroup.)
struct GridBarrier {
    unsigned nblocks;
    bool spread;                        // workgroups on more than one XCD; only thread 0's copy is used

    __device__ __forceinline__ void meet(int b, bool first)
    {
        __syncthreads();
        if (threadIdx.x == 0) {
            if (first) (void)or_in_l2(&g_sync.xcc_mask.v, 1u << xcc_id());   // done before this workgroup arrives
            if (spread) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __hip_atomic_fetch_add(&g_sync.arrived[b].v, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            unsigned long long t0 = 0;
            for (unsigned polls = 0; or_in_l2(&g_sync.arrived[b].v, 0u) < nblocks; ++polls) {
                __builtin_amdgcn_s_sleep(1);
                if ((polls & 63u) == 63u) {                   // look at the clock now and then
                    const unsigned long long now = wall_clock64();
                    if (t0 == 0) t0 = now;
                    if (now - t0 > FZ_WAIT_TICKS) {           // give up: count it, go on, keep arriving
                        __hip_atomic_fetch_add(&g_sync.timeouts.v, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            if (first) {                                      // every arrival published its bit before arriving
                const unsigned mask = or_in_l2(&g_sync.xcc_mask.v, 0u);
                spread = (mask & (mask - 1u)) != 0u;
            }
        }
        __syncthreads();
    }

    // Last thing a workgroup does: the last one out leaves the counters zeroed for the next launch.
    __device__ __forceinline__ void depart()
    {
        __syncthreads();
        if (threadIdx.x == 0) {
            const unsigned before = __hip_atomic_fetch_add(&g_sync.departed.v, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (before == nblocks - 1) {                      // everyone else has passed every barrier and left
                for (int b = 0; b < FZ_BARRIERS; ++b)
                    __hip_atomic_store(&g_sync.arrived[b].v, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&g_sync.xcc_mask.v, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&g_sync.departed.v, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
};

template <int EPL>
__device__ __forceinline__ void topk_phase(const FusedArgs &a, int block, int nblocks)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    for (int t = block * FZ_WAVES + wave; t < a.tp.T; t += nblocks * FZ_WAVES) {
        if (a.tp.splits > 8) router_topk_token<EPL, RT_MAX_SPLIT>(a.zpart, a.bias, a.ids, a.w, a.tp, t, lane);
        else router_topk_token<EPL, 8>(a.zpart, a.bias, a.ids, a.w, a.tp, t, lane);
    }
}

// MB_MAX: row blocks of the tallest tile.
template <int MB_MAX>
__global__ __launch_bounds__(FZ_THREADS) void fused_forward_kernel(FusedArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    // Workgroups are handed to the XCDs in turn; only every eighth one takes part, so that the
    // launch normally sits on one XCD and its barriers stay inside that XCD's L2.
    if (blockIdx.x % MOE_WORK_RANGES != 0) return;
    const int block = (int)blockIdx.x / MOE_WORK_RANGES, nblocks = (int)gridDim.x / MOE_WORK_RANGES;
    GridBarrier sync{(unsigned)nblocks, true};              // (spread until the first barrier has shown otherwise)
    int bar = 0;

    // ---- routing ---------------------------------------------------------------------------------
    if (a.route_mode == ROUTE_TILED) {
        LogitsLds &lds = *reinterpret_cast<LogitsLds *>(smem);
        const int per_split = a.rg.tiles_t * a.rg.tiles_e;
        for (int i = block; i < per_split * a.rg.splits; i += nblocks) {
            const int split = i / per_split, r = i % per_split;
            router_logits_tile<false>(a.x, nullptr, a.router_w, a.zpart, a.tp.T, a.H, a.tp.E, a.rg.k_per_split,
                                      r % a.rg.tiles_t, r / a.rg.tiles_t, split, lds);
        }
        sync.meet(bar, bar == 0), ++bar;                      // the partial logits of every H slice are there
        switch (a.epl) {
        case 1: topk_phase<1>(a, block, nblocks); break;
        case 2: topk_phase<2>(a, block, nblocks); break;
        default: topk_phase<4>(a, block, nblocks); break;
        }
    } else {
        float (&part_z)[4][RT_FEW] = *reinterpret_cast<float (*)[4][RT_FEW]>(smem);
        if (a.route_mode == ROUTE_FEW_SPLIT) {
            for (int b = block; b < a.tp.T; b += nblocks) {
                router_few_tokens<false, 4>(a.x, nullptr, a.router_w, a.bias, a.ids, a.w, a.tp, a.H, b, part_z);
                __syncthreads();                              // part_z is reused by the next token
            }
        } else {
            for (int b = block; b < ceil_div(a.tp.T, 4); b += nblocks)
                router_few_tokens<false, 1>(a.x, nullptr, a.router_w, a.bias, a.ids, a.w, a.tp, a.H, b, part_z);
        }
    }
    sync.meet(bar, bar == 0), ++bar;                          // every token is routed

    // ---- sort-scatter ------------------------------------------------------------------------------
    permute_block<FZ_THREADS>(a.ids, a.P, a.EL, a.e_first, a.tile_rows, a.max_tiles, a.offsets, a.sorted_pair,
                              a.inv, a.tiles, a.sched, reinterpret_cast<int *>(smem), 0, 1);
    {
        // this workgroup reads back what it has just written: its stores are complete after the
        // workgroup barrier, and one invalidate keeps the compute unit's cache from answering with older lines
        __syncthreads();
        if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        __syncthreads();
        // ---- expert GEMMs and combine --------------------------------------------------------------
        using SH1 = typename ShapesFor<MB_MAX, true, false>::Narrow;
        using SH2 = typename ShapesFor<MB_MAX, false, false>::Narrow;
        gemm_items<SH1>(a.g1, a.tiles, a.sched, a.col_tiles1, a.whole_ranges, 32, block, nblocks, smem);
        sync.meet(bar, false), ++bar;                         // act is complete
        gemm_items<SH2>(a.g2, a.tiles, a.sched, a.col_tiles2, a.whole_ranges, 32, block, nblocks, smem);
        sync.meet(bar, false), ++bar;                         // y is complete
        const long long shares = (long long)a.T * (a.out_H / 8);
        for (long long idx = (long long)block * FZ_THREADS + threadIdx.x; idx < shares; idx += (long long)nblocks * FZ_THREADS)
            combine_chunk<false>(reinterpret_cast<const uint16_t *>(a.g2.out), a.w, a.inv, a.out, a.out_H, a.top_k, idx);
    }
    sync.depart();
}

template <int MB_MAX>
constexpr int full_lds_bytes()
{
    using SH1 = typename ShapesFor<MB_MAX, true, false>::Narrow;
    using SH2 = typename ShapesFor<MB_MAX, false, false>::Narrow;
    constexpr int gemm = SH1::LDS_BYTES > SH2::LDS_BYTES ? SH1::LDS_BYTES : SH2::LDS_BYTES;
    return gemm;
}

std::atomic<int> g_enabled{0};

int compute_units()
{
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

template <int MB_MAX>
int launch_variant(const FusedArgs &a, int blocks, int lds, hipStream_t s)
{
    auto kern = fused_forward_kernel<MB_MAX>;
    static DeviceOnce lds_limit_set;
    const int rc = set_dynamic_lds(lds_limit_set, reinterpret_cast<const void *>(kern), lds);
    if (rc != MOE_OK) return rc;
    hipLaunchKernelGGL(kern, dim3(blocks * MOE_WORK_RANGES), dim3(FZ_THREADS), lds, s, a);   // one in eight takes part
    return check_launch();
}

}  // namespace

void set_single_launch(int enable) { g_enabled.store(enable ? 1 : 0, std::memory_order_relaxed); }

int single_launch_timeouts(unsigned *out)
{
    GridSync host;
    hipError_t e = hipMemcpyFromSymbol(&host, HIP_SYMBOL(g_sync), sizeof(host), 0, hipMemcpyDeviceToHost);
    if (e != hipSuccess) { set_last_hip_error(e); return MOE_ERR_HIP; }
    *out = host.timeouts.v;
    return MOE_OK;
}

// Whether moe_forward runs this problem as one launch (a property of the problem statement and of
// the switch above; see include/moe.h).
int single_launch_mode(const moe_config &c, int tile_rows)
{
    if (!g_enabled.load(std::memory_order_relaxed)) return MOE_SINGLE_LAUNCH_NONE;
    const long P = (long)c.T * c.top_k;
    if (c.T <= 0 || P > FZ_MAX_PAIRS || local_experts(c) > FZ_MAX_EXPERTS || c.E > 256) return MOE_SINGLE_LAUNCH_NONE;
    if (c.dtype != MOE_DTYPE_BF16 || c.quantize_x) return MOE_SINGLE_LAUNCH_NONE;
    if (!route_few(c) && c.T >= 512) return MOE_SINGLE_LAUNCH_NONE;          // (the matrix-core router's territory)
    const int mb = tile_rows / 16, est = expected_tiles(c);
    const bool small = tile_rows <= 64 && gemm_width(mb, true, false, c.I, est) == GEMM_NARROW &&
                       gemm_width(mb, false, false, c.H, est) == GEMM_NARROW;
    return small ? MOE_SINGLE_LAUNCH_ALL : MOE_SINGLE_LAUNCH_NONE;
}

int launch_fused(const moe_config &c, int tile_rows, int max_tiles, const void *x, const float *router_w,
                 const float *bias, void *route_ws, int32_t *ids, float *w, int32_t *offsets, int32_t *sorted_pair,
                 int32_t *inv, moe_tile *tiles, int32_t *sched, const void *w1, const void *w2, void *act, void *y,
                 void *out, hipStream_t s)
{
    const int cus = compute_units();
    if (cus < 8 * MOE_WORK_RANGES) return MOE_ERR_UNSUPPORTED;   // (the caller falls back to the pipeline)
    FusedArgs a{};
    a.x = x; a.router_w = router_w; a.bias = bias;
    a.zpart = static_cast<float *>(route_ws);
    a.ids = ids; a.w = w;
    a.H = c.H;
    a.epl = route_epl(c);
    int route_blocks;
    if (route_few(c)) {
        a.route_mode = route_few_split(c) ? ROUTE_FEW_SPLIT : ROUTE_FEW;
        a.tp = topk_params(c, 1);
        route_blocks = route_few_split(c) ? c.T : ceil_div(c.T, 4);
    } else {
        a.route_mode = ROUTE_TILED;
        a.rg = route_grid(c);
        a.tp = topk_params(c, a.rg.splits);
        route_blocks = a.rg.tiles_t * a.rg.tiles_e * a.rg.splits;
        if (route_blocks < ceil_div(c.T, FZ_WAVES)) route_blocks = ceil_div(c.T, FZ_WAVES);
    }
    a.P = c.T * c.top_k; a.EL = local_experts(c); a.e_first = c.local_expert_offset;
    a.tile_rows = tile_rows; a.max_tiles = max_tiles;
    a.offsets = offsets; a.sorted_pair = sorted_pair; a.inv = inv; a.tiles = tiles; a.sched = sched;
    a.T = c.T; a.out_H = c.H; a.top_k = c.top_k;
    a.out = static_cast<uint16_t *>(out);
    const int lds_front = (int)sizeof(LogitsLds) > (int)(sizeof(int) * permute_lds_ints(FZ_THREADS, a.EL))
                              ? (int)sizeof(LogitsLds) : (int)(sizeof(int) * permute_lds_ints(FZ_THREADS, a.EL));
    a.g1 = gateup_args(c, x, nullptr, w1, nullptr, sorted_pair, act, nullptr);
    a.g2 = down_args(c, act, nullptr, w2, nullptr, y, 1);   // (tiles of at most 64 rows: K is never split here)
    a.whole_ranges = expected_tiles(c) <= 8 * MOE_WORK_RANGES ? 1 : 0;
    const int mb = tile_rows / 16;
    const int cols1 = 16 * 4, cols2 = 32 * 4;                 // columns per narrow workgroup (gate/up, down)
    a.col_tiles1 = ceil_div(c.I, cols1);
    a.col_tiles2 = ceil_div(c.H, cols2);
    long need = route_blocks;
    const long items1 = (long)max_tiles * a.col_tiles1, items2 = (long)max_tiles * a.col_tiles2;
    if (items1 > need) need = items1;
    if (items2 > need) need = items2;
    const long comb = ((long)c.T * (c.H / 8) + FZ_THREADS - 1) / FZ_THREADS;
    if (comb > need) need = comb;
    // workgroups that take part: a multiple of eight (the GEMM schedule has eight parts), at most
    // the compute units of one XCD
    int blocks = (int)((need + 7) / 8 * 8);
    const int cap = cus / MOE_WORK_RANGES / 8 * 8;
    if (blocks > cap) blocks = cap;
    if (blocks < 8) blocks = 8;
    switch (mb) {
    case 1: return launch_variant<1>(a, blocks, full_lds_bytes<1>() > lds_front ? full_lds_bytes<1>() : lds_front, s);
    case 2: return launch_variant<2>(a, blocks, full_lds_bytes<2>() > lds_front ? full_lds_bytes<2>() : lds_front, s);
    case 4: return launch_variant<4>(a, blocks, full_lds_bytes<4>() > lds_front ? full_lds_bytes<4>() : lds_front, s);
    default: return MOE_ERR_UNSUPPORTED;
    }
}

}  // namespace moe
