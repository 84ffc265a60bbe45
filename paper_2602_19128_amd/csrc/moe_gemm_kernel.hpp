// Grouped expert GEMMs on the matrix cores, bf16 and block-scaled fp8 (paper Sec. 4.5 "Expert
// FFN computation": tensor-core tiles, loads of the next block overlapping the compute of the
// current one, experts without tokens skipped; the kernel table of Sec. 4.3 names fp8 packing and
// scaling as the challenge of this operator).
//
// Both GEMMs are C[m,n] = sum_k A[m,k] * W[e,n,k] with few rows m per expert (a few to a
// few hundred) against large weight matrices, so the weights must stream from HBM exactly
// once and at full rate.  The kernel is built around that:
//
//  * A workgroup of NW wavefronts owns ALL rows of one expert tile (up to 16*MB_MAX) times a
//    slab of weight rows; wavefront w owns two blocks of 16 weight rows (gate + matching up
//    rows, or 32 consecutive down-projection rows; 64 rows for the down projection of low tiles).
//  * Every global read is a direct global -> LDS copy (global_load_lds, 16 bytes per lane) whose
//    64 lanes cover 8 rows x 128 contiguous bytes: whole cache lines per instruction.  (Loading
//    weights straight into the MFMA register layout would touch 16 rows x 64 bytes per
//    instruction, half lines, which measures ~20% slower on this memory system.)  Weights land
//    in a ring private to the owning wavefront (no barrier on the weight path, DW steps ahead;
//    a slot is refilled as soon as its fragments sit in registers, so the ring holds exactly the
//    DW stages in flight); the token rows (x gathered through the sorted pair list, or act) are
//    shared by all wavefronts and land in a second ring DA steps ahead.  Physical 16-byte chunk pc
//    of LDS row r holds logical chunk pc ^ (r & 7) (applied on the global-address side of the
//    copy), which keeps the 16-byte MFMA fragment reads free of bank conflicts.
//  * One K step is 128 bytes of every row: 64 bf16 elements (two v_mfma_f32_16x16x32_bf16) or
//    128 fp8 elements (one v_mfma_f32_16x16x128_f8f6f4, exactly one 128-wide scale block).  The
//    weights are the row operand, so the accumulator of lane l holds 4 consecutive output
//    columns of token l%16: the epilogue applies act = silu(g) * u in registers and stores whole
//    8-byte (bf16) or 4-byte (fp8) pieces.
//  * Inside a step the token fragments are software-pipelined: fragment q+PF is requested from
//    LDS while the MFMAs of fragment q run (the order is pinned with scheduling barriers).
//  * fp8: each K step's product is formed in a fresh accumulator and folded into the running
//    fp32 sum with (activation scale of the token's 1x128 block) x (weight scale of the 128x128
//    block).  Activation scales ride along with the token rows in the LDS ring; a wavefront's
//    weight scales for the whole K range sit in one or two registers and are broadcast by lane
//    index.  The gate/up epilogue re-quantises act per 1x128 block (scale = amax/448) - a
//    workgroup of 8 wavefronts covers exactly one such block per row.
//  * One s_barrier per K step orders the token ring; outstanding-copy counts are waited for
//    explicitly (s_waitcnt vmcnt(n)) so that a barrier never drains the copy queue.
//  * Row blocks beyond the tile's real row count are skipped (the K loop is instantiated per
//    row-block count), so an expert with 140 tokens costs 9-10 blocks of 16, not 256 rows.
//  * Workgroups start their K loops at different columns when the row stride is a multiple of
//    4 KiB (see k_groups_for).
//
// The tile list arrives as a schedule of eight work ranges, tallest tiles first (moe_permute);
// workgroups are numbered so that each XCD (own L2) works through one range: the token rows of
// an expert stay in one L2, and the tiles that take longest start first.
#pragma once
#include "moe_internal.hpp"

namespace moe {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;

constexpr int GM_XCDS = MOE_WORK_RANGES;  // one work range of the schedule per XCD
constexpr int GM_CUS = 256;
constexpr float GM_FP8_MAX = 448.f;
constexpr int GM_PF = 4;                 // token fragments requested ahead of the MFMAs that use them (bf16)
constexpr int GM_PF_FP8 = 2;             // the same for fp8 (a fragment is twice as large)
                 // cache policy bit "non-temporal" of a copy

#define MOE_WAIT_VMCNT(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")

// Direct global -> LDS copies, one instruction per wavefront: lane l moves 16 (or 4) bytes from its
// own global address to LDS byte address lds_base + 16*l (4*l).  Written as inline assembly so that
// the compiler's wait-count bookkeeping of the ordinary LDS reads stays exact (it otherwise falls
// back to full waits whenever such a copy is pending); the copies are tracked by hand with
// MOE_WAIT_VMCNT.  lds_base must be wavefront-uniform.
__device__ __forceinline__ uint32_t lds_addr_of(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)(p);
}
// m0 (the LDS base of such a copy) is named as clobbered so that the compiler never carries a value of
// its own in m0 across these statements; clang notes that it does not save reserved registers, which
// is what is wanted here.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
template <bool NT>
__device__ __forceinline__ void copy16_to_lds(const void *g, uint32_t lds_base)
{
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds_base), "v"(g) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(g) : "memory", "m0");
}
__device__ __forceinline__ void copy4_to_lds(const void *g, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_base), "v"(g) : "memory", "m0");
}
#pragma clang diagnostic pop

// s_waitcnt vmcnt(n) for a wavefront-uniform run-time n (the instruction takes an immediate).
__device__ __forceinline__ void wait_vmcnt_upto(int n)
{
    switch (n) {
#define MOE_WAIT_CASE(k) case k: MOE_WAIT_VMCNT(k); break;
        MOE_WAIT_CASE(0) MOE_WAIT_CASE(1) MOE_WAIT_CASE(2) MOE_WAIT_CASE(3) MOE_WAIT_CASE(4) MOE_WAIT_CASE(5)
        MOE_WAIT_CASE(6) MOE_WAIT_CASE(7) MOE_WAIT_CASE(8) MOE_WAIT_CASE(9) MOE_WAIT_CASE(10) MOE_WAIT_CASE(11)
        MOE_WAIT_CASE(12) MOE_WAIT_CASE(13) MOE_WAIT_CASE(14) MOE_WAIT_CASE(15) MOE_WAIT_CASE(16) MOE_WAIT_CASE(17)
        MOE_WAIT_CASE(18) MOE_WAIT_CASE(19) MOE_WAIT_CASE(20) MOE_WAIT_CASE(21) MOE_WAIT_CASE(22) MOE_WAIT_CASE(23)
        MOE_WAIT_CASE(24) MOE_WAIT_CASE(25) MOE_WAIT_CASE(26) MOE_WAIT_CASE(27) MOE_WAIT_CASE(28) MOE_WAIT_CASE(29)
        MOE_WAIT_CASE(30)
#undef MOE_WAIT_CASE
    default: MOE_WAIT_VMCNT(0); break;                        // waiting for more than needed is always safe
    }
}

__device__ __forceinline__ int lds_off(int row, int chunk)   // byte offset of logical 16-byte chunk of a row
{
    return row * 128 + ((chunk ^ (row & 7)) << 4);
}


// Compile-time shape of one kernel variant.
//   MB_MAX  row blocks (of 16) a tile may have        NW  wavefronts per workgroup
//   DA      token-row stages in flight                DW  weight stages in flight (DW >= DA)
//   SPLITK  down projection whose K is cut in halves (see down_k_split): an item is (tile, column slab, half
//           of K) and leaves an fp32 partial sum
template <int MB_MAX_, int NW_, int DA_, int DW_, bool SWIGLU_, bool FP8_, int BPW_ = 2, bool SPLITK_ = false>
struct Shape {
    static constexpr int MB_MAX = MB_MAX_, NW = NW_, DA = DA_, DW = DW_;
    static constexpr bool SWIGLU = SWIGLU_, FP8 = FP8_, SPLITK = SPLITK_;
    static_assert(!SPLITK || (!SWIGLU && !FP8), "K is split for the bf16 down projection only");
    static constexpr int BPW = BPW_;                          // 16-row weight blocks per wavefront (gate/up: one gate + one up block)
    static_assert(!SWIGLU || BPW == 2, "gate/up: one gate and one up block per wavefront");
    static constexpr int THREADS = NW * kWave;
    static constexpr int W_COPIES = 2 * BPW;                  // weight copies per wavefront per step, 8 rows each
    static constexpr int W_STAGE = 16 * BPW * 128;            // bytes of one wavefront's weight stage
    static constexpr int SLAB = SWIGLU ? 16 : 16 * BPW;       // output columns per wavefront
    static constexpr int COLS = SLAB * NW;                    // output columns per workgroup
    static constexpr int STAGE_BYTES = MB_MAX * 16 * 128;     // one token-row stage
    static constexpr int A_RING_BYTES = (DA + 1) * STAGE_BYTES;
    static constexpr int W_RING_BYTES = DW * NW * W_STAGE;
    // one fp32 activation scale per token row, copied 64 rows (one wavefront) at a time
    static constexpr int SC_STAGE_BYTES = FP8 ? ((MB_MAX * 16 + 63) / 64) * 256 : 0;
    static constexpr int LDS_BYTES = A_RING_BYTES + W_RING_BYTES + (DA + 1) * SC_STAGE_BYTES;
    static_assert(DW >= DA && DA >= 1, "weights are copied at least as far ahead as token rows");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of one compute unit");
    // half-width items (see gemm_tile): wide workgroups only; the fp8 gate/up epilogue needs whole 128-column blocks
    static constexpr bool HALF_ITEMS = NW >= 8 && !(FP8 && SWIGLU) && !SPLITK;
    static_assert(!(FP8 && SWIGLU) || COLS == kQBlock, "fp8 gate/up: a workgroup re-quantises one 1x128 block per row");
};

// One item of a launch's work: a row tile, a column slab of it (half: 0 the whole slab, 1 / 2 its
// first / second half) and the item's number in the launch (which fixes its K rotation).
struct Item {
    moe_tile tile;
    int ct, half, work;
};

// Everything after the (tile, column slab) decision, instantiated per active row-block count NB.
// A workgroup may work through several items in a row.  `next` (if has_next) is the item it takes
// after this one: when both are whole-slab items and the staged output tile of this one leaves the
// weight ring alone, the first weight stages of `next` are requested before this item's epilogue,
// so that the latency of their trip from HBM passes while the output is written; the call then
// returns true and the next call is told so (`prefetched`: its weight copies of stages 0..DW-1
// are already under way).
template <class SH, int NB, bool HALF>
__device__ __forceinline__ bool gemm_tile(const GemmArgs &g, const Item item, const Item next, const bool has_next,
                                          const bool prefetched, unsigned char *smem)
{
    const moe_tile &tile = item.tile;
    // (split K: the items of one column slab are its halves of K, first half first)
    const int ct = SH::SPLITK ? item.ct >> 1 : item.ct, kh = SH::SPLITK ? item.ct & 1 : 0;
    const int half = item.half, work = item.work;
    constexpr int NW = SH::NW, DA = SH::DA, DW = SH::DW;
    constexpr bool SWIGLU = SH::SWIGLU, FP8 = SH::FP8;
    constexpr int ES = FP8 ? 1 : 2;                           // bytes per element
    constexpr int SA = DA + 1;                                // token-row stages
    constexpr int SW = DW;                                    // weight stages (a slot is refilled as soon as its fragments are in registers)
    constexpr int STAGE_BYTES = SH::STAGE_BYTES;
    constexpr int A_PASS_MAX = (NB * 2 + NW - 1) / NW;        // 8-row copy passes per wavefront
    constexpr int SLAB = SH::SLAB;
    constexpr int BPW = SH::BPW, GM_W_COPIES = SH::W_COPIES, GM_W_STAGE = SH::W_STAGE;
    static_assert(GM_W_COPIES + (DA - 1) * (GM_W_COPIES + A_PASS_MAX + 1) <= 30, "wait_vmcnt_upto covers up to 30 copies in flight");

    // The thread index goes through an empty asm statement, so that everything derived from it is
    // computed here, per item: otherwise the compiler hoists the per-lane addresses of every
    // row-block variant out of the kernel's item loop and keeps them all in registers at once.
    int tid_opaque = threadIdx.x;
    asm volatile("" : "+v"(tid_opaque));
    const int tid = tid_opaque, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, lets the compiler keep it scalar
    const int l16 = lane & 15, lq = lane >> 4;
    const int crow = lane >> 3;                               // copy: row inside an 8-row pass
    const int cbyte = ((lane & 7) ^ crow) << 4;               // copy: byte offset of the logical chunk for this lane's slot
    const int rows = tile.rows;
    // Weights are read once and marked non-temporal so they do not push the shared token rows out
    // of L2.  Exception (measured): an expert with several row tiles, whose workgroups run side by
    // side and share each weight line through L2 - in the down projection from two tiles on, in the
    // gate/up projection from three on (hot experts and the compute-bound regime: -3..5 %; with two
    // tiles the cacheable weight stream costs the token rows more than the sharing saves: +1..4 %).
    const bool share_weights = tile.count > (SWIGLU ? 2 : 1);
    const int n_out = g.n_out;
    const size_t row_bytes = (size_t)g.K * ES;
    const int nk = (int)(row_bytes / GM_STEP_BYTES) / (SH::SPLITK ? 2 : 1);   // K steps of this item
    const size_t kbase = (size_t)kh * nk * GM_STEP_BYTES;     // byte offset of its first step in a row
    // Workgroups that run side by side start their K loops at different columns (and wrap around):
    // with every workgroup at the same column, rows whose stride is a multiple of a large power of
    // two keep hitting the same memory channels.  The sum over K is the same set of terms.
    const int koff = (int)((long)(work % g.k_groups) * nk / g.k_groups);
    auto k_rot = [&](int s_) __attribute__((always_inline)) { const int r_ = s_ + koff; return r_ >= nk ? r_ - nk : r_; };

    // ---- weight row pointers: copy q (0..3) moves rows 8q..8q+7 of this wavefront's 32 rows
    // (rows 0..15 = first block, 16..31 = second block)
    // half = 0: the whole column slab.  half = 1 / 2: its first / second half only, computed by the
    // first half of the wavefronts (the others still copy token rows and keep the barriers); such
    // items fill the compute units that the last round of a launch would leave idle, and with
    // half the fragment traffic through LDS their K steps are shorter.
    const bool active = !HALF || wave < NW / 2;               // (HALF is instantiated separately: whole slabs keep their code)
    const int half_col = (HALF && half == 2) ? SH::COLS / 2 : 0;
    const int col0 = ct * SH::COLS + half_col + (HALF ? wave % (NW / 2) : wave) * SLAB;   // first output column of this wavefront
    const int wc = active ? GM_W_COPIES : 0;                  // weight copies this wavefront issues per step
    const int w_rows = SWIGLU ? 2 * n_out : n_out;
    // pointers of this wavefront's weight copies for the slab starting at output column c0 of expert e
    auto weight_ptrs = [&](int e, int c0, const unsigned char *(&ptr)[GM_W_COPIES]) __attribute__((always_inline)) {
        const unsigned char *wbase = g.W + (size_t)e * w_rows * row_bytes + kbase + cbyte;
#pragma unroll
        for (int q = 0; q < GM_W_COPIES; ++q) {
            const int in_blk = (q & 1) * 8 + crow;            // row inside the 16-row block
            int wrow;
            if constexpr (SWIGLU) {
                const int c = min(c0 + in_blk, n_out - 1);    // clamp: columns past the end are never stored
                wrow = (q < 2) ? c : n_out + c;               // gate row / matching up row
            } else {
                wrow = min(c0 + q * 8 + crow, n_out - 1);
            }
            ptr[q] = wbase + (size_t)wrow * row_bytes;
        }
    };
    const unsigned char *w_ptr[GM_W_COPIES];
    weight_ptrs(tile.expert, col0, w_ptr);
    unsigned char *const w_ring = smem + SH::A_RING_BYTES + wave * (SW * GM_W_STAGE);
    unsigned char *const sc_ring = smem + SH::A_RING_BYTES + SH::W_RING_BYTES;
    const uint32_t smem_lds = __builtin_amdgcn_readfirstlane(lds_addr_of(smem));
    const uint32_t w_lds = __builtin_amdgcn_readfirstlane(lds_addr_of(w_ring));
    const uint32_t sc_lds = __builtin_amdgcn_readfirstlane(lds_addr_of(sc_ring));

    // fp8: this wavefront's weight scales for every K step, lane l holds step l (and l + 64)
    float wsc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
    if constexpr (FP8) {
        const int cc = min(col0, n_out - 1);
        const int blk0 = cc / kQBlock;
        const int blk1 = SWIGLU ? (n_out + cc) / kQBlock : blk0;
        const float *ws = g.w_scale + (size_t)tile.expert * (w_rows / kQBlock) * nk;
        if (lane < nk) { wsc[0][0] = ws[(size_t)blk0 * nk + lane]; wsc[1][0] = ws[(size_t)blk1 * nk + lane]; }
        if (lane + 64 < nk) { wsc[0][1] = ws[(size_t)blk0 * nk + lane + 64]; wsc[1][1] = ws[(size_t)blk1 * nk + lane + 64]; }
    }

    // ---- token row pointers: copy pass p moves LDS rows 8p..8p+7 -----------------
    int a_cnt = 0;                                            // copies per slot beyond the weight copies
    const unsigned char *a_ptr[A_PASS_MAX];
    int a_dst[A_PASS_MAX];
#pragma unroll
    for (int i = 0; i < A_PASS_MAX; ++i) {
        const int p = wave + NW * i;
        if (8 * p < NB * 16) ++a_cnt;
        int r = 8 * p + crow;
        r = r < rows ? r : rows - 1;                          // padded rows repeat the last row; never stored
        size_t src;
        if constexpr (SWIGLU) src = (size_t)(g.sorted_pair[tile.row0 + r] / g.top_k);
        else src = (size_t)(tile.row0 + r);
        a_ptr[i] = g.A + src * row_bytes + kbase + cbyte;
        a_dst[i] = p * 1024;
    }
    // fp8: wavefront j also copies the activation scales of rows 64j..64j+63 (4 bytes per lane)
    const float *sc_ptr = nullptr;
    bool sc_copy = false;
    if constexpr (FP8) {
        sc_copy = wave * 64 < NB * 16;
        if (sc_copy) ++a_cnt;
        int r = wave * 64 + lane;
        r = r < rows ? r : rows - 1;
        size_t src;
        if constexpr (SWIGLU) src = (size_t)(g.sorted_pair[tile.row0 + r] / g.top_k);
        else src = (size_t)(tile.row0 + r);
        sc_ptr = g.a_scale + src * nk;
    }

    f32x4 acc[NB][BPW];
#pragma unroll
    for (int m = 0; m < NB; ++m)
#pragma unroll
        for (int b = 0; b < BPW; ++b) acc[m][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Copies of K step `s` (callers issue them only for s < nk).
#define MOE_COPY_TOKENS(s)                                                                             \
    {                                                                                                  \
        const int ks_ = k_rot(s);                                                                      \
        const int k0_ = ks_ * GM_STEP_BYTES;                                                           \
        const uint32_t dst_ = smem_lds + ((s) % SA) * STAGE_BYTES;                                     \
        _Pragma("unroll") for (int i = 0; i < A_PASS_MAX; ++i)                                         \
            if (i < a_cnt - (sc_copy ? 1 : 0))                                                         \
                copy16_to_lds<false>(a_ptr[i] + k0_, dst_ + a_dst[i]);                                 \
        if constexpr (FP8) {                                                                           \
            if (sc_copy)                                                                               \
                copy4_to_lds(sc_ptr + ks_, sc_lds + ((s) % SA) * SH::SC_STAGE_BYTES + wave * 256);     \
        }                                                                                              \
    }
#define MOE_COPY_WEIGHTS_OF(s, ptr_, koff_, share_)                                                   \
    {                                                                                                  \
        const int r_ = (s) + (koff_);                                                                  \
        const int k0_ = (r_ >= nk ? r_ - nk : r_) * GM_STEP_BYTES;                                     \
        const uint32_t dst_ = w_lds + ((s) % SW) * GM_W_STAGE;                                         \
        if (share_) {                                                                                  \
            _Pragma("unroll") for (int q = 0; q < GM_W_COPIES; ++q)                                    \
                copy16_to_lds<false>(ptr_[q] + k0_, dst_ + q * 1024);                                  \
        } else {                                                                                       \
            _Pragma("unroll") for (int q = 0; q < GM_W_COPIES; ++q)                                    \
                copy16_to_lds<true>(ptr_[q] + k0_, dst_ + q * 1024);                                   \
        }                                                                                              \
    }
#define MOE_COPY_WEIGHTS(s) MOE_COPY_WEIGHTS_OF(s, w_ptr, koff, share_weights)

    // Issue slot t (t = -DW .. nk-1) holds [token copy of step t+DA, weight copy of step t+DW].
    // prologue: slots -DW .. -1
    // (prefetched: the weight copies of these slots were issued by the previous item of this workgroup,
    // ahead of all the token copies below)
#pragma unroll
    for (int t = -DW; t < 0; ++t) {
        if (t + DA >= 0 && t + DA < nk) MOE_COPY_TOKENS(t + DA)
        if (!prefetched && active && t + DW < nk) MOE_COPY_WEIGHTS(t + DW)
    }

    for (int s = 0; s < nk; ++s) {
        // Step s needs its token copy (slot s-DA) and its weight copy (slot s-DW, older or same)
        // landed.  Copies complete in order, so it is enough to let only what was issued after the
        // younger of the two stay in flight: the weight copy sharing the slot of that token copy
        // (when the weights run further ahead than the token rows) and the DA-1 slots after it.
        // Near the end of K some of those copies do not exist; they are not counted.
        int in_flight = (DW > DA && s - DA + DW < nk) ? wc : 0;
#pragma unroll
        for (int t = 1 - DA; t < 0; ++t)
            in_flight += (s + t + DA < nk ? a_cnt : 0) + (s + t + DW < nk ? wc : 0);
        // (a prefetched item issued its weight copies first and its token copies last, behind the
        // stores of the previous epilogue: its first step simply waits for all of them)
        if (prefetched && s == 0) MOE_WAIT_VMCNT(0);
        else wait_vmcnt_upto(in_flight);
        asm volatile("s_barrier" ::: "memory");               // token stage s complete for everyone; stage s-1 free
        if (s + DA < nk) MOE_COPY_TOKENS(s + DA)
        __builtin_amdgcn_sched_barrier(0);
        const unsigned char *sa = smem + (s % SA) * STAGE_BYTES;
        const unsigned char *sw = w_ring + (s % SW) * GM_W_STAGE;
        if (active) {
        if constexpr (FP8) {
            // one MFMA spans the whole step: lane (l16, lq) holds bytes 32*lq .. 32*lq+31 of its row
            const float *ssc = reinterpret_cast<const float *>(sc_ring + (s % SA) * SH::SC_STAGE_BYTES);
            const int sr = k_rot(s);
            const int sl = sr & 63;
            const float sw0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(
                __builtin_bit_cast(int, sr < 64 ? wsc[0][0] : wsc[0][1]), sl));
            const float sw1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(
                __builtin_bit_cast(int, sr < 64 ? wsc[1][0] : wsc[1][1]), sl));
            constexpr int PF = NB < GM_PF_FP8 ? NB : GM_PF_FP8;
            i32x8 wq[BPW];
#pragma unroll
            for (int b = 0; b < BPW; ++b) {
                const u32x4 lo = *reinterpret_cast<const u32x4 *>(sw + lds_off(b * 16 + l16, 2 * lq));
                const u32x4 hi = *reinterpret_cast<const u32x4 *>(sw + lds_off(b * 16 + l16, 2 * lq + 1));
                wq[b] = i32x8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
            }
            __builtin_amdgcn_sched_barrier(0);
            u32x4 tlo[PF], thi[PF];
            float tsx[PF];
#define MOE_LOAD_TOK8(slot, m_)                                                                        \
            {                                                                                          \
                tlo[slot] = *reinterpret_cast<const u32x4 *>(sa + lds_off((m_) * 16 + l16, 2 * lq));     \
                thi[slot] = *reinterpret_cast<const u32x4 *>(sa + lds_off((m_) * 16 + l16, 2 * lq + 1)); \
                tsx[slot] = ssc[(m_) * 16 + l16];                                                      \
            }
#pragma unroll
            for (int q = 0; q < PF; ++q) MOE_LOAD_TOK8(q, q)
            __builtin_amdgcn_sched_barrier(0);
            f32x4 pp[BPW][2];
            float fs[BPW][2];
#pragma unroll
            for (int m = 0; m <= NB; ++m) {
                if (m < NB) {
                    const u32x4 lo = tlo[m % PF], hi = thi[m % PF];
                    const i32x8 t = i32x8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
                    const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
                    // e4m3 x e4m3, hardware block scales set to 1.0 (E8M0 0x7f): the fp32 scales are applied below
#pragma unroll
                    for (int b = 0; b < BPW; ++b) {
                        pp[b][m & 1] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(wq[b], t, zero, 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
                        fs[b][m & 1] = tsx[m % PF] * ((SWIGLU && b == 1) ? sw1 : sw0);
                    }
                    if (m + PF < NB) MOE_LOAD_TOK8(m % PF, m + PF)
                }
                if (m > 0) {
                    const int pm = m - 1;
#pragma unroll
                    for (int b = 0; b < BPW; ++b)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[pm][b][v] = fmaf(pp[b][pm & 1][v], fs[b][pm & 1], acc[pm][b][v]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (m == 0) {
                    // the MFMAs above waited for the weight fragments (LDS reads return in order and the
                    // token fragment was requested after them): the weight slot may be refilled
                    if (s + DW < nk) MOE_COPY_WEIGHTS(s + DW)
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#undef MOE_LOAD_TOK8
        } else {
            // Software pipeline over the 2*NB token fragments of this step: fragment q+PF is read
            // from LDS while the MFMAs of fragment q run.
            constexpr int NQ = 2 * NB;
            constexpr int PF = NQ < GM_PF ? NQ : GM_PF;
            bf16x8 wf[2][BPW], tf[PF];
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
                for (int b = 0; b < BPW; ++b)
                    wf[kk][b] = *reinterpret_cast<const bf16x8 *>(sw + lds_off(b * 16 + l16, kk * 4 + lq));
            }
            __builtin_amdgcn_sched_barrier(0);
#define MOE_LOAD_TOK(q_) (*reinterpret_cast<const bf16x8 *>(sa + lds_off(((q_) % NB) * 16 + l16, ((q_) / NB) * 4 + lq)))
#pragma unroll
            for (int q = 0; q < PF; ++q) tf[q] = MOE_LOAD_TOK(q);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int kk = q / NB, m = q % NB;
#pragma unroll
                for (int b = 0; b < BPW; ++b)
                    acc[m][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[kk][b], tf[q % PF], acc[m][b], 0, 0, 0);
                if (q + PF < NQ) tf[q % PF] = MOE_LOAD_TOK(q + PF);
                __builtin_amdgcn_sched_barrier(0);
                if (q == 0) {
                    // the MFMAs above waited for all four weight fragments (LDS reads return in order and
                    // the token fragment was requested after them): the weight slot may be refilled
                    if (s + DW < nk) MOE_COPY_WEIGHTS(s + DW)
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#undef MOE_LOAD_TOK
        }
        }   // active
        __builtin_amdgcn_sched_barrier(0);
    }
    // Every copy of this item has landed (the last step waited for its own, and nothing was issued
    // after those).  The output tile is staged over the token ring; when it stays clear of the
    // weight ring, this wavefront's first weight stages of the next item go out now.
    constexpr int STAGED_BYTES = ((SWIGLU && FP8) ? NW * NB * 16 * 4 : 0) + NB * 16 * SH::COLS * ((SWIGLU && FP8) ? 1 : 2);
    bool gave_next = false;
    if constexpr (!HALF && !SH::SPLITK && STAGED_BYTES <= SH::A_RING_BYTES) {
        if (has_next && next.half == 0) {
            const unsigned char *nw_ptr[GM_W_COPIES];
            weight_ptrs(next.tile.expert, next.ct * SH::COLS + wave * SLAB, nw_ptr);
            const int nkoff = (int)((long)(next.work % g.k_groups) * nk / g.k_groups);
            const bool nshare = next.tile.count > (SWIGLU ? 2 : 1);
#pragma unroll
            for (int t = 0; t < DW; ++t)
                if (t < nk) MOE_COPY_WEIGHTS_OF(t, nw_ptr, nkoff, nshare)
            gave_next = true;
        }
    }
    if (!gave_next) MOE_WAIT_VMCNT(0);                        // nothing is in flight any more; cheap insurance for the LDS reuse below
#undef MOE_COPY_TOKENS
#undef MOE_COPY_WEIGHTS
#undef MOE_COPY_WEIGHTS_OF

    if constexpr (SH::SPLITK) {
        // ---- epilogue of a K half: the fp32 accumulators leave as they are, to this half's partial-sum
        // array.  Staged through LDS like the bf16 tile below (a lane holds 4 consecutive columns of 16
        // rows: written straight from registers a store would touch 16 rows x 16 bytes); a 1 KiB row per
        // token does not fit for a whole tall tile, so the tile leaves in parts of NBP row blocks.
        constexpr int ROW_B = SH::COLS * 4;
        constexpr int CPR = ROW_B / 16;
        constexpr int PARTS = (NB * 16 * ROW_B + SH::LDS_BYTES - 1) / SH::LDS_BYTES;
        constexpr int NBP = (NB + PARTS - 1) / PARTS;
        static_assert(NBP * 16 * ROW_B <= SH::LDS_BYTES, "a part of the output tile must fit the LDS of the rings");
        auto stage_at = [&](int r, int byte) __attribute__((always_inline)) {
            return smem + r * ROW_B + ((((byte >> 4) ^ ((r & (CPR / 2 - 1)) << 1))) << 4) + (byte & 15);
        };
        unsigned char *const part_out = g.out + (size_t)kh * g.split_stride;
        const size_t out_pitch = (size_t)n_out * 4;
#pragma unroll
        for (int part = 0; part < PARTS; ++part) {
            const int m0 = part * NBP;                        // first row block of this part
            __syncthreads();                                  // the rings (or the previous part) are done with
#pragma unroll
            for (int m = m0; m < m0 + NBP && m < NB; ++m) {
                const int r = (m - m0) * 16 + l16;
#pragma unroll
                for (int b = 0; b < BPW; ++b)
                    *reinterpret_cast<f32x4 *>(stage_at(r, (wave * SLAB + b * 16 + lq * 4) * 4)) = acc[m][b];
            }
            __syncthreads();
            const int part_rows = min(rows - m0 * 16, NBP * 16);
            for (int c = tid; c < part_rows * CPR; c += SH::THREADS) {
                const int r = c / CPR, ch = c % CPR;
                const int col = ct * SH::COLS + ch * 4;       // n_out is a multiple of 16 elements: chunks are all in or all out
                if (col < n_out) {
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(stage_at(r, ch * 16));
                    u32x4 *dst = reinterpret_cast<u32x4 *>(part_out + (size_t)(tile.row0 + m0 * 16 + r) * out_pitch + (size_t)col * 4);
                    if (g.nt_out) __builtin_nontemporal_store(v, dst);
                    else *dst = v;
                }
            }
        }
        return false;
    } else {

    // ---- epilogue: lane l holds, for token l%16 of each row block, output columns 4*(l/16)..+3
    // of each of its two weight blocks.  Written straight from that layout a store instruction
    // would touch 16 rows x 32 bytes; such partial-line writes cost the down projection a fifth
    // of its time.  So the workgroup stages its rows x COLS output tile in LDS (the rings are
    // free now) and writes it out row-major, 16 bytes per lane, whole 128-byte lines.
    constexpr int OUT_ES = (SWIGLU && FP8) ? 1 : 2;           // bytes per output element
    constexpr int ROW_B = SH::COLS * OUT_ES;                  // bytes of one staged row
    constexpr int CPR = ROW_B / 16;                           // 16-byte chunks per staged row
    constexpr int RED_BYTES = (SWIGLU && FP8) ? NW * NB * 16 * 4 : 0;
    static_assert(RED_BYTES + NB * 16 * ROW_B <= SH::LDS_BYTES, "output tile must fit the LDS of the rings");
    unsigned char *const stage = smem + RED_BYTES;
    // chunk ch of staged row r sits at chunk ch ^ swz(r): spreads the 16 rows of one store over the banks
    auto stage_at = [&](int r, int byte) __attribute__((always_inline)) {
        return stage + r * ROW_B + ((((byte >> 4) ^ ((r & (CPR / 2 - 1)) << 1))) << 4) + (byte & 15);
    };
    __syncthreads();                                          // every wavefront is done with the rings
    const int scol = (HALF ? wave % (NW / 2) : wave) * SLAB;   // this wavefront's first column inside the staged tile
    if constexpr (SWIGLU && FP8) {
        // act = silu(g)*u, then per-row amax over the workgroup's 128 columns -> scale = amax/448
        float a[NB][4];
        float *red = reinterpret_cast<float *>(smem);         // [NW][NB*16]
#pragma unroll
        for (int m = 0; m < NB; ++m) {
            float mx = 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float gt = acc[m][0][v], up = acc[m][1][v];
                a[m][v] = (col0 + lq * 4 + v < n_out) ? gt / (1.f + __expf(-gt)) * up : 0.f;
                mx = fmaxf(mx, fabsf(a[m][v]));
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            if (lq == 0) red[wave * (NB * 16) + m * 16 + l16] = mx;
        }
        __syncthreads();
#pragma unroll
        for (int m = 0; m < NB; ++m) {
            const int r = m * 16 + l16;
            float amax = 0.f;
#pragma unroll
            for (int wv = 0; wv < NW; ++wv) amax = fmaxf(amax, red[wv * (NB * 16) + r]);
            const float scale = amax > 0.f ? amax / GM_FP8_MAX : 1.f;
            const float inv = 1.f / scale;
            float q[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) q[v] = fminf(fmaxf(a[m][v] * inv, -GM_FP8_MAX), GM_FP8_MAX);
            int packed = 0;
            packed = __builtin_amdgcn_cvt_pk_fp8_f32(q[0], q[1], packed, false);
            packed = __builtin_amdgcn_cvt_pk_fp8_f32(q[2], q[3], packed, true);
            *reinterpret_cast<int *>(stage_at(r, (scol + lq * 4) * OUT_ES)) = packed;
            if (r < rows && wave == 0 && lq == 0) g.out_scale[(size_t)(tile.row0 + r) * (n_out / kQBlock) + ct] = scale;
        }
    } else if (active) {
#pragma unroll
        for (int m = 0; m < NB; ++m) {
            const int r = m * 16 + l16;
            if constexpr (SWIGLU) {
                float a[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float gt = acc[m][0][v], up = acc[m][1][v];
                    a[v] = gt / (1.f + __expf(-gt)) * up;
                }
                uint2 o;
                o.x = pack_bf16x2(a[0], a[1]);
                o.y = pack_bf16x2(a[2], a[3]);
                *reinterpret_cast<uint2 *>(stage_at(r, (scol + lq * 4) * OUT_ES)) = o;
            } else {
#pragma unroll
                for (int b = 0; b < BPW; ++b) {
                    uint2 o;
                    o.x = pack_bf16x2(acc[m][b][0], acc[m][b][1]);
                    o.y = pack_bf16x2(acc[m][b][2], acc[m][b][3]);
                    *reinterpret_cast<uint2 *>(stage_at(r, (scol + b * 16 + lq * 4) * OUT_ES)) = o;
                }
            }
        }
    }
    __syncthreads();
    // row-major write-out: consecutive lanes hold consecutive 16-byte chunks of a row
    const size_t out_pitch = (size_t)n_out * OUT_ES;
    const int cpr = HALF ? CPR / 2 : CPR;                     // chunks of a row that were computed
    for (int c = tid; c < rows * cpr; c += SH::THREADS) {
        const int r = c / cpr, ch = c % cpr;
        const int col = ct * SH::COLS + half_col + ch * (16 / OUT_ES);   // n_out is a multiple of 16 elements: chunks are all in or all out
        if (col < n_out) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(stage_at(r, ch * 16));
            u32x4 *dst = reinterpret_cast<u32x4 *>(g.out + (size_t)(tile.row0 + r) * out_pitch + (size_t)col * OUT_ES);
            if (g.nt_out) __builtin_nontemporal_store(v, dst);
            else *dst = v;
        }
    }
    return gave_next;
    }   // not SPLITK
}

template <class SH, int NB>
__device__ __forceinline__ bool dispatch_blocks(int nb, const GemmArgs &g, const Item item, const Item next,
                                                const bool has_next, const bool prefetched, unsigned char *smem)
{
    if constexpr (NB > SH::MB_MAX) {
        return false;
    } else {
        constexpr int NEXT = NB + 1;
        if (nb <= NB) {
            if constexpr (SH::HALF_ITEMS) {
                if (item.half) return gemm_tile<SH, NB, true>(g, item, next, has_next, prefetched, smem);
                return gemm_tile<SH, NB, false>(g, item, next, has_next, prefetched, smem);
            } else {
                return gemm_tile<SH, NB, false>(g, item, next, has_next, prefetched, smem);
            }
        } else {
            return dispatch_blocks<SH, NEXT>(nb, g, item, next, has_next, prefetched, smem);
        }
    }
}

// The schedule (see moe_permute) lists the tiles range by range, tallest first; XCD r (the
// workgroups with blockIdx % 8 == r, which share an L2) works through part r of the resulting item
// sequence (tile-major, one item per column slab), so the workgroups running side by side there
// are on neighbouring column slabs of the same expert tile and share its token rows through that L2.
//   whole_ranges = 1: part r is work range r, whole tiles only.  With few tiles per XCD this
//     keeps each XCD on as few tiles at a time as possible (their token rows compete with the
//     weight stream for its L2; measured +20 % on a 32-expert share when parts cut through tiles).
//   whole_ranges = 0: the sequence is cut into eight equal parts, which coincide with the ranges
//     up to a tile or two at their ends.  Every tile streams the same weight bytes, so with many
//     tiles per XCD equal item counts are what lets the XCDs finish together.
// The launch normally has one workgroup per item; the loop only matters when a part holds more
// work than its share of the grid.
// Workgroup `block` of `nblocks` (a multiple of MOE_WORK_RANGES) works through its share of the
// schedule; the stand-alone kernel below and the single-launch forward both run this loop.
// Where a workgroup does take several items (the single-launch forward, whose grid is small), every item
// but its first has its first weight stages requested before the epilogue of its predecessor (see
// gemm_tile).  Shrinking the stand-alone launch to make every workgroup loop was measured and is not
// done: with 2 / 4 / 8 items per workgroup the gate/up GEMM of a 4096-token DeepSeek-shaped prefill took
// +2 / +8 / +21 % (the hardware's hand-out of fresh workgroups balances tiles of unequal height, a fixed
// share per workgroup does not), with or without the prefetch.
template <class SH>
__device__ __forceinline__ void gemm_items(const GemmArgs &g, const moe_tile *tiles, const int32_t *sched,
                                           int col_tiles, int whole_ranges, int round_slots, int block,
                                           int nblocks, unsigned char *smem)
{
    const int part = block % MOE_WORK_RANGES;
    int first, items;
    if (whole_ranges) {
        first = sched[1 + part] * col_tiles;
        items = sched[2 + part] * col_tiles - first;
    } else {
        const int total = sched[0] * col_tiles;
        const int per = ceil_div(total, MOE_WORK_RANGES);
        first = part * per;
        items = min(per, total - first);
    }
    const int stride = nblocks / MOE_WORK_RANGES;
    // Order inside a long part: alternating between its front and its back in chunks of col_tiles
    // items (tall tile, short tile, tall, ...) instead of tallest-first.  Tall tiles spend their
    // time on LDS and the matrix cores, short ones on the weight stream, and a mix of both running
    // side by side is faster than all tall tiles together: gate/up GEMM -4..5 % on the DeepSeek-shaped
    // prefills; the down GEMM -12 % when the tallest tiles are full height (hot experts), but +5 % when
    // every tile is low, where tallest-first only shortens the tail - so it alternates only when the
    // tallest tile of the list (its first record) has more than 128 rows.
    const bool zigzag = !whole_ranges && (SH::SWIGLU || tiles[0].rows > 128);
    const int nchunks = ceil_div(items, col_tiles);
    // A last round that would fill at most half of the XCD's workgroup slots is handed out as
    // half-width items, two per column slab.
    const int rest = items % round_slots;
    const int halved = (SH::HALF_ITEMS && whole_ranges && rest > 0 && 2 * rest <= round_slots) ? rest : 0;
    const int slots = zigzag ? nchunks * col_tiles : items + halved;
    // the item in slot `slot` of this part (false: the slot is past the end, or a hole of the last, short chunk)
    auto item_at = [&](int slot, Item &it) __attribute__((always_inline)) -> bool {
        if (slot >= slots) return false;
        int pos = slot;
        if (zigzag) {
            const int c = slot / col_tiles;
            const int pc = (c & 1) ? nchunks - 1 - (c >> 1) : (c >> 1);
            pos = pc * col_tiles + slot % col_tiles;
            if (pos >= items) return false;
        }
        it.half = 0;
        if (pos >= items - halved) {                           // (never together with zigzag)
            const int h = pos - (items - halved);
            pos = items - halved + (h >> 1);
            it.half = 1 + (h & 1);
        }
        it.work = first + pos;
        const moe_tile head = tiles[it.work / col_tiles];
        const int local = it.work - head.first * col_tiles;    // index inside this expert's work
        it.ct = local / head.count;                            // column slab
        it.tile = tiles[head.first + local % head.count];
        return true;
    };
    // The workgroup takes slots b, b + stride, b + 2 stride, ... (neighbouring workgroups are on
    // neighbouring slots at any time, so the column slabs of a tile still run side by side and share
    // its token rows through L2; a workgroup that took consecutive slots instead measured +10..15 %).
    Item cur{}, nxt{};
    int slot = block / MOE_WORK_RANGES;
    bool have = item_at(slot, cur), prefetched = false;
    while (slot < slots) {
        const bool have_next = item_at(slot + stride, nxt);
        if (have) {
            const int nb = ceil_div(cur.tile.rows, 16);
            prefetched = dispatch_blocks<SH, 1>(nb, g, cur, nxt, have_next, prefetched, smem);
            __syncthreads();                                   // the output tile has left LDS
        } else {
            prefetched = false;
        }
        cur = nxt;
        have = have_next;
        slot += stride;
    }
}

template <class SH>
__global__ __launch_bounds__(SH::THREADS) void grouped_gemm_kernel(GemmArgs g, const moe_tile *__restrict__ tiles,
                                                                   const int32_t *__restrict__ sched, int col_tiles,
                                                                   int whole_ranges, int round_slots)
{
    extern __shared__ __align__(16) unsigned char smem[];
    gemm_items<SH>(g, tiles, sched, col_tiles, whole_ranges, round_slots, (int)blockIdx.x, (int)gridDim.x, smem);
}

template <class SH>
int launch_shape(const GemmArgs &g, const moe_tile *tiles, const int32_t *sched, int max_tiles, int est_tiles,
                 hipStream_t s)
{
    const int col_tiles = ceil_div(g.n_out, SH::COLS) * (SH::SPLITK ? 2 : 1);   // split K: two items per column slab
    auto kern = grouped_gemm_kernel<SH>;
    // workgroups one XCD runs at once: LDS (160 KiB) and wavefront slots (32) of a compute unit decide it
    int per_cu = (160 * 1024) / SH::LDS_BYTES;
    if (per_cu > 32 / SH::NW) per_cu = 32 / SH::NW;
    const int round_slots = (GM_CUS / GM_XCDS) * (per_cu < 1 ? 1 : per_cu);
    static DeviceOnce lds_limit_set;                          // the dynamic-LDS limit, once per device
    const int rc = set_dynamic_lds(lds_limit_set, reinterpret_cast<const void *>(kern), SH::LDS_BYTES);
    if (rc != MOE_OK) return rc;
    // a part holds about an eighth of the tiles; the slack (a tile's slabs, and the half-width items
    // of a last round) keeps the loop in the kernel at one trip
    const int part_slots = (ceil_div(max_tiles, GM_XCDS) + 1) * col_tiles + (SH::HALF_ITEMS ? round_slots / 2 : 0);
    const int blocks = part_slots * GM_XCDS;
    const int whole_ranges = est_tiles <= 8 * GM_XCDS ? 1 : 0;   // at most eight tiles per XCD
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(SH::THREADS), SH::LDS_BYTES, s, g, tiles, sched, col_tiles, whole_ranges,
                       round_slots);
    return check_launch();
}

// The workgroup widths (see gemm_width) as kernel shapes.
template <int MB_MAX, bool SWIGLU, bool FP8>
struct ShapesFor {
    static constexpr int DA = MB_MAX >= 16 ? 1 : 2;           // 16 row blocks: 32 KiB per token stage
    static constexpr int DW = 2;
    using Wide = Shape<MB_MAX, 8, DA, DW, SWIGLU, FP8>;
    using Narrow = Shape<MB_MAX, 4, DA, 3, SWIGLU, FP8>;
    using Wide4 = Shape<MB_MAX, 8, DA, DW, SWIGLU, FP8, SWIGLU ? 2 : 4>;
    using WideSplit = Shape<MB_MAX, 8, DA, DW, false, false, 2, true>;
};

template <int MB_MAX, bool SWIGLU, bool FP8>
int launch_for_rows(const GemmArgs &g, const moe_tile *tiles, const int32_t *sched, int max_tiles, int est_tiles,
                    hipStream_t s)
{
    using SF = ShapesFor<MB_MAX, SWIGLU, FP8>;
    if (g.k_split > 1) {                                      // (down_k_split asks for it only where this holds)
        if constexpr (!SWIGLU && !FP8 && MB_MAX >= 8)
            return launch_shape<typename SF::WideSplit>(g, tiles, sched, max_tiles, est_tiles, s);
        return MOE_ERR_UNSUPPORTED;
    }
    switch (gemm_width(MB_MAX, SWIGLU, FP8, g.n_out, est_tiles)) {
    case GEMM_WIDE4:
        if constexpr (!SWIGLU && (MB_MAX == 2 || MB_MAX == 4))
            return launch_shape<typename SF::Wide4>(g, tiles, sched, max_tiles, est_tiles, s);
        return MOE_ERR_UNSUPPORTED;
    case GEMM_NARROW:
        if constexpr (!(FP8 && SWIGLU))
            return launch_shape<typename SF::Narrow>(g, tiles, sched, max_tiles, est_tiles, s);
        return MOE_ERR_UNSUPPORTED;
    default:
        return launch_shape<typename SF::Wide>(g, tiles, sched, max_tiles, est_tiles, s);
    }
}

template <bool SWIGLU, bool FP8>
int launch_by_tile_rows(int tile_rows, const GemmArgs &g, const moe_tile *tiles, const int32_t *sched,
                        int max_tiles, int est_tiles, hipStream_t s)
{
    switch (tile_rows) {
    case 256: return launch_for_rows<16, SWIGLU, FP8>(g, tiles, sched, max_tiles, est_tiles, s);
    case 128: return launch_for_rows<8, SWIGLU, FP8>(g, tiles, sched, max_tiles, est_tiles, s);
    case 64:  return launch_for_rows<4, SWIGLU, FP8>(g, tiles, sched, max_tiles, est_tiles, s);
    case 32:  return launch_for_rows<2, SWIGLU, FP8>(g, tiles, sched, max_tiles, est_tiles, s);
    case 16:  return launch_for_rows<1, SWIGLU, FP8>(g, tiles, sched, max_tiles, est_tiles, s);
    default:  return MOE_ERR_UNSUPPORTED;
    }
}

}  // namespace
}  // namespace moe
