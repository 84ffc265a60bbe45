// Device code of the sort-scatter (paper Sec. 4.5: tokens reordered by expert into contiguous memory).
//
// A stable counting sort of the P (token, slot) pairs by expert id.  The pairs are cut into
// slices of PM_SLICE, one workgroup of 16 wavefronts each, and the workgroups never talk to each
// other: every workgroup counts ALL pairs in LDS (how many of each expert lie before its slice,
// inside it per wavefront, and after it), which gives it the expert offsets and the first row
// of each of its wavefronts; then each wavefront walks its contiguous part of the slice in
// order and ranks equal experts inside a 64-pair batch with ballots.  Counting everything in
// every workgroup costs a few microseconds; placing the pairs is the expensive part (it is bound
// by the instruction rate of a compute unit) and is what the slices divide.  Workgroup 0 also
// writes the offsets and cuts every non-empty expert segment into row tiles for the grouped
// GEMMs; experts without tokens get no tile and therefore cost nothing downstream.
//
// The tile list is also the GEMMs' schedule.  A tile's cost grows with its rows, and a launch
// ends when its last tile ends, so experts are ranked by row count (largest first) and dealt in
// snake order (0..7, 7..0, ...) to eight work ranges, one per XCD: every range starts with its
// tallest tiles and the eight ranges carry about the same load.  All tiles of an expert stay in
// one range (its workgroups share the expert's token rows, and the weights of an expert with
// several tiles, through that XCD's L2).
#pragma once
#include "moe_internal.hpp"

namespace moe {
namespace {

constexpr int PM_BATCH = 8;             // 64-pair batches whose ids are loaded together
constexpr int PM_SLICE = 1024;          // pairs placed by one workgroup (one 64-pair batch per wavefront)
constexpr int PM_MAX_WGS = 64;

// Inclusive scan of n <= kMaxExperts ints held in LDS (Hillis-Steele, all threads sync).
__device__ inline void block_inclusive_scan(int *a, int *b, int n, int tid)
{
    int *src = a, *dst = b;
    for (int off = 1; off < n; off <<= 1) {
        if (tid < n) dst[tid] = src[tid] + (tid >= off ? src[tid - off] : 0);
        __syncthreads();
        int *tmp = src; src = dst; dst = tmp;
    }
    if (src != a) {
        if (tid < n) a[tid] = src[tid];
        __syncthreads();
    }
}

// E is the number of experts that own a segment (the local ones); a pair's segment is
// ids[p] - e_first, and pairs outside [0, E) after that shift are dropped.
// The body is written for a workgroup of THREADS threads that is "block" number `block` of `nblocks`
// independent ones; `lds` must hold permute_lds_ints(THREADS, E) ints.
inline __host__ __device__ size_t permute_lds_ints(int threads, int E)
{
    const size_t eq = (size_t)ceil_div(E, MOE_WORK_RANGES) * MOE_WORK_RANGES;
    return (size_t)(threads / kWave) * E + 7 * (size_t)E + 1 + 2 * eq;
}

template <int THREADS>
__device__ __forceinline__ void permute_block(const int32_t *__restrict__ ids, int P, int E, int e_first, int tile_rows,
                                              int max_tiles, int32_t *__restrict__ offsets,
                                              int32_t *__restrict__ sorted_pair, int32_t *__restrict__ inv,
                                              moe_tile *__restrict__ tiles, int32_t *__restrict__ sched, int *lds,
                                              int block, int nblocks)
{
    constexpr int WAVES = THREADS / kWave;
        int *wcount = lds;                         // [WAVES][E]  per-wavefront counts -> write cursors
    int *scan_a = wcount + WAVES * E;       // [E]
    int *scan_b = scan_a + E;                  // [E]
    int *first_row = scan_b + E;               // [E+1] exclusive offsets
    const int RQ = ceil_div(E, MOE_WORK_RANGES); // schedule positions per work range
    const int EQ = RQ * MOE_WORK_RANGES;
    int *rows_of = first_row + E + 1;          // [E]  rows per expert, for the ranking
    int *rank_of = rows_of + E;                // [E]  experts that come earlier in the ranking
    int *before = rank_of + E;                 // [E]  pairs of each expert in earlier slices
    int *after = before + E;                   // [E]  ... in later slices
    int *sch_a = after + E;                    // [EQ] tiles at each schedule position (range-major)
    int *sch_b = sch_a + EQ;                   // [EQ]

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    // this workgroup's slice, and this wavefront's part of it (whole 64-pair batches)
    const int slice = ceil_div(ceil_div(P, nblocks), WAVES * kWave) * WAVES * kWave;
    const int s_beg = min(P, block * slice), s_end = min(P, s_beg + slice);
    const int per_wave = slice / WAVES;
    const int p_beg = min(s_end, s_beg + wave * per_wave), p_end = min(s_end, p_beg + per_wave);
    const bool lead = block == 0;         // the workgroup that writes offsets, tiles and schedule

    for (int i = tid; i < WAVES * E; i += THREADS) wcount[i] = 0;
    if (tid < E) { before[tid] = 0; after[tid] = 0; }
    __syncthreads();

    // pass 1: count every pair once (integer LDS adds: order-independent).  The ids of PM_BATCH
    // strides are requested together so that their latencies overlap.
    for (int base = 0; base < P; base += PM_BATCH * THREADS) {
        int ev[PM_BATCH];
#pragma unroll
        for (int j = 0; j < PM_BATCH; ++j) {
            const int p = base + j * THREADS + tid;
            const int e = ids[min(p, P - 1)] - e_first;      // unconditional: a load under a branch is waited for at once
            ev[j] = (p < P) ? e : -1;
        }
#pragma unroll
        for (int j = 0; j < PM_BATCH; ++j) {
            const int p = base + j * THREADS + tid;
            if (ev[j] >= 0 && ev[j] < E) {
                int *bin = p < s_beg ? before : p >= s_end ? after : wcount + ((p - s_beg) / per_wave) * E;
                atomicAdd(&bin[ev[j]], 1);
            }
        }
    }
    __syncthreads();

    // rows per expert -> exclusive offsets -> first row of each wavefront of this slice
    int total = 0;
    if (tid < E) {
        total = before[tid] + after[tid];
        for (int wv = 0; wv < WAVES; ++wv) total += wcount[wv * E + tid];
        scan_a[tid] = total;
    }
    __syncthreads();
    block_inclusive_scan(scan_a, scan_b, E, tid);
    if (tid < E) {
        const int excl = scan_a[tid] - total;
        first_row[tid] = excl;
        if (lead) offsets[tid] = excl;
        int run = excl + before[tid];          // turn counts into per-wavefront write cursors
        for (int wv = 0; wv < WAVES; ++wv) {
            const int c = wcount[wv * E + tid];
            wcount[wv * E + tid] = run;
            run += c;
        }
        if (tid == E - 1) { first_row[E] = scan_a[tid]; if (lead) offsets[E] = scan_a[tid]; }
    }
    __syncthreads();

    if (lead) {
    // tile list: expert e gets ceil(rows_e / tile_rows) records.  Schedule position of an expert:
    // rank by rows (descending, ties by index), dealt in snake order to the work ranges.
    const int my_tiles = (tid < E) ? ceil_div(total, tile_rows) : 0;
    if (tid < E) { rows_of[tid] = total; rank_of[tid] = 0; }
    for (int i = tid; i < EQ; i += THREADS) sch_a[i] = 0;
    __syncthreads();
    // rank of expert e = experts with more rows (or as many and a lower index); the comparisons of
    // one expert are spread over THREADS / E threads
    {
        const int parts = max(1, THREADS / E);
        const int seg = ceil_div(E, parts);
        const int e = tid % E, part = tid / E;
        if (part < parts) {
            const int mine = rows_of[e];
            const int lo = part * seg, hi = min(E, lo + seg);
            int before = 0;
#pragma unroll 8
            for (int e2 = lo; e2 < hi; ++e2) {
                const int r2 = rows_of[e2];
                before += (r2 > mine || (r2 == mine && e2 < e)) ? 1 : 0;
            }
            if (before) atomicAdd(&rank_of[e], before);
        }
    }
    __syncthreads();
    int q = 0;
    if (tid < E) {
        const int rank = rank_of[tid];
        const int round = rank / MOE_WORK_RANGES, pos = rank % MOE_WORK_RANGES;
        const int range = (round & 1) ? MOE_WORK_RANGES - 1 - pos : pos;
        q = range * RQ + round;
        sch_a[q] = my_tiles;
    }
    __syncthreads();
    block_inclusive_scan(sch_a, sch_b, EQ, tid);
    if (tid < E) {
        const int first = sch_a[q] - my_tiles;
        // an expert with more rows than a tile is cut into equal parts (rounded up to whole MFMA
        // row blocks): the grouped GEMMs' step time grows with the rows of a tile
        const int part = my_tiles > 0 ? ceil_div(ceil_div(total, my_tiles), 16) * 16 : 0;
        for (int i = 0; i < my_tiles && first + i < max_tiles; ++i) {
            moe_tile rec;
            rec.expert = tid;
            rec.row0 = first_row[tid] + i * part;
            rec.rows = max(0, min(part, total - i * part));
            rec.first = first;
            rec.count = my_tiles;
            rec.pad0 = rec.pad1 = rec.pad2 = 0;
            tiles[first + i] = rec;
        }
    }
    if (tid <= MOE_WORK_RANGES) {              // [0] records written, [1 + r] first record of range r (r = 8: the end)
        const int upto = tid * RQ;             // schedule positions before range `tid`
        const int at = upto > 0 ? sch_a[upto - 1] : 0;
        sched[1 + tid] = min(at, max_tiles);
        if (tid == MOE_WORK_RANGES) sched[0] = min(at, max_tiles);
    }
    }   // lead

    // pass 2: stable placement.  Batches of 64 consecutive pairs; inside a batch a pair's
    // rank among equal experts is the number of lower lanes holding the same expert.
    volatile int *cursor = wcount + wave * E;
    const int ebits = 32 - __clz(max(E - 1, 1));
    for (int base0 = p_beg; base0 < p_end; base0 += PM_BATCH * kWave) {
        int ev[PM_BATCH];
#pragma unroll
        for (int j = 0; j < PM_BATCH; ++j) {
            const int p = base0 + j * kWave + lane;
            const int e = ids[min(p, P - 1)] - e_first;
            ev[j] = (p < p_end) ? e : -1;
        }
#pragma unroll
        for (int j = 0; j < PM_BATCH; ++j) {
            const int base = base0 + j * kWave;
            if (base >= p_end) break;                          // wave-uniform
            const int p = base + lane;
            const int e = ev[j];
            const bool valid = e >= 0 && e < E;
            unsigned long long same = __ballot(valid);
            for (int b = 0; b < ebits; ++b) {
                const unsigned long long m = __ballot((e >> b) & 1);
                same &= ((e >> b) & 1) ? m : ~m;
            }
            const unsigned long long lower = (1ull << lane) - 1ull;
            const int at = cursor[valid ? e : 0];          // every lane of an expert reads its cursor ...
            __builtin_amdgcn_wave_barrier();               // ... before the first of them advances it
            if (valid) {
                const int rank = __popcll(same & lower);
                const int row = at + rank;
                sorted_pair[row] = p;
                inv[p] = row;
                if (rank == 0) cursor[e] = at + __popcll(same);
            } else if (p < p_end) {
                inv[p] = -1;
            }
            // the next batch reads the cursors this one advanced: keep the wavefront's LDS accesses in order
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}


}  // namespace
}  // namespace moe
