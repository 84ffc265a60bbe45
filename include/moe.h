/*
 * Fused Mixture-of-Experts layer forward for AMD Instinct MI355X (gfx950).
 *
 * The operator is the MoE layer the paper analyses in Sec. 4.5 ("Kernel
 * Analysis: FP8 MoE Kernel"): every token scores all experts and keeps the top-k;
 * the chosen experts run a gate and an up projection combined through SiLU, then a
 * down projection.  The pipeline follows the one the paper credits for the fast
 * kernel (Sec. 4.5, "Expert FFN computation"): (1) routing, (2) a sort-scatter
 * that places each expert's tokens contiguously, (3) tensor-core expert GEMMs,
 * with experts that received no token skipped; a weighted sum over the k experts
 * of a token finishes the layer.
 *
 * Conventions for every entry point
 *   - C ABI, plain pointers and sizes.  Unless marked HOST, a pointer is a DEVICE
 *     pointer owned by the caller; tensors are contiguous, row-major, with the
 *     shape written beside them, and 16-byte aligned.
 *   - `stream` is the caller's hipStream_t (passed as void*; NULL = default
 *     stream).  Calls only enqueue work: no allocation, no free, no host
 *     synchronisation, no device-to-host copy happens inside the library.
 *   - Same inputs give bit-identical outputs (no floating-point atomics anywhere).
 *   - Return value: MOE_OK or a negative error code; nothing is enqueued when an
 *     argument check fails.
 *   - Threads: any number of host threads may call in at the same time (the only
 *     shared host state is a once-per-device kernel set-up that tolerates it); the
 *     error of moe_last_hip_error() is per thread.  Calls that share a workspace or
 *     an output must not overlap on the device: put them on one stream.
 *   - Shapes: H and I multiples of 64 (128 for fp8, and at most 16384 there),
 *     E <= 512, top_k <= min(E,64).
 *     Group-limited routing needs E % n_group == 0, a power-of-two number of
 *     lanes per group (see moe_route) and top_k <= topk_group * E / n_group.
 *   - Notation: T tokens, H hidden size, I expert intermediate size, E experts,
 *     k = top_k, P = T*k (token, slot) pairs, pair id p = t*k + j.
 *   - Local-expert mode (the share of the layer one device holds under expert
 *     parallelism; the paper's Sec. 4.5 workload is 32 local experts of 256):
 *     the router still scores all E experts, but only experts
 *     [local_expert_offset, local_expert_offset + num_local_experts) have weights
 *     here.  Pairs routed elsewhere are dropped by the sort-scatter and contribute
 *     nothing to `out`, which is then this device's partial sum of the layer.
 *     EL below is num_local_experts, or E when that field is 0.
 *   - Quantise-on-the-path mode (cfg->quantize_x = 1, fp8 layers): the hidden states
 *     arrive as bf16 and the per-token 1x128 block quantisation that an fp8 expert GEMM
 *     needs (the "fp8 packing and scaling" that the paper's kernel table in Sec. 4.3
 *     names as this operator's difficulty) is a step of the layer instead of the
 *     caller's job.
 */
#ifndef MOE_H
#define MOE_H

#include <stddef.h>
#include <stdint.h>

/* The library is built with hidden symbol visibility; the entry points below are its whole
 * exported surface. */
#define MOE_API __attribute__((visibility("default")))

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MOE_OK = 0,
    MOE_ERR_INVALID = -1,       /* null pointer / inconsistent argument */
    MOE_ERR_UNSUPPORTED = -2,   /* shape or dtype combination the kernels do not cover */
    MOE_ERR_WORKSPACE = -3,     /* workspace too small */
    MOE_ERR_HIP = -4            /* a launch failed; see moe_last_hip_error() */
};

enum { MOE_SCORE_SOFTMAX = 0, MOE_SCORE_SIGMOID = 1 };
enum { MOE_DTYPE_BF16 = 0, MOE_DTYPE_FP8_E4M3 = 1 };

/* Problem statement of one layer call (plain data, passed from HOST memory). */
typedef struct moe_config {
    int32_t T, H, I, E, top_k;
    int32_t scoring;            /* MOE_SCORE_SOFTMAX: s = softmax(z), choice key c = s
                                   MOE_SCORE_SIGMOID: s = sigmoid(z), c = s + bias      */
    int32_t renormalize;        /* divide the k weights by their sum */
    int32_t n_group;            /* <= 1: no group limiting.  Otherwise experts form n_group
                                   contiguous blocks, a block scores the sum of its
                                   group_score_topn largest keys, and only experts of the
                                   topk_group best blocks may be chosen */
    int32_t topk_group;
    int32_t group_score_topn;
    int32_t dtype;              /* payload type of x, w1, w2 (and of the act buffer) */
    float   routed_scale;       /* final factor on the k weights */
    int32_t local_expert_offset;/* first expert whose weights this call holds */
    int32_t num_local_experts;  /* how many it holds; 0 = all E (then the offset must be 0) */
    int32_t quantize_x;         /* 1 (dtype fp8 only): x arrives as bf16 and the layer quantises it
                                   to e4m3 per 1x128 block itself (moe_quantize_act); the router
                                   scores the bf16 values.  Only moe_forward, moe_route and the
                                   size queries look at this field */
} moe_config;

/* Row count of one tile of the grouped GEMMs for this problem (the height the
 * tile list produced by moe_permute is cut to), and the capacity, in tiles, the
 * caller must give the tile list. */
MOE_API int32_t moe_tile_rows(const moe_config *cfg);
MOE_API int32_t moe_max_tiles(const moe_config *cfg);

/* One tile-list record: rows [row0, row0+rows) of the expert-sorted order all
 * belong to `expert`; `first` is the index of that expert's first record and
 * `count` how many records the expert has (they are consecutive). */
typedef struct moe_tile {
    int32_t expert, row0, rows, first, count, pad0, pad1, pad2;
} moe_tile;

/* The tile list doubles as the schedule of the grouped GEMMs.  It is cut into
 * MOE_WORK_RANGES consecutive ranges (one per XCD of the device); moe_permute
 * describes them in an int32 array of MOE_SCHED_INTS entries:
 *   sched[0]      records written
 *   sched[1 + r]  index of the first record of range r, r = 0..MOE_WORK_RANGES
 *                 (the last entry is the end: equal to sched[0])
 * Experts are ranked by their row count, largest first (equal counts: lower index
 * first), and dealt to the ranges in snake order (0..7, 7..0, ...), so every range
 * lists its tallest tiles first and the ranges carry similar loads.  The grouped
 * GEMMs give range r to XCD r when a range is a few tiles, and otherwise cut the
 * list into eight parts of equal tile-slab count (the ranges, up to a tile or two
 * at their ends). */
enum { MOE_WORK_RANGES = 8, MOE_SCHED_INTS = 16 };

/* Launch shape of a grouped GEMM for this problem (a property of the problem statement alone;
 * which = 0: gate/up, 1: down), for tests and tuning:
 *   plan[0] tile rows (= moe_tile_rows)      plan[1] wavefronts per workgroup
 *   plan[2] 16-row weight blocks per wavefront   plan[3] output columns per workgroup
 *   plan[4] 1: XCD r works through work range r (whole tiles); 0: eight parts of equal item count
 *   plan[5] 1: a last round that fills at most half an XCD is handed out as half-width items
 *   plan[6] down projection inside moe_forward: 1, or 2 = K is cut in halves with items of their own
 *           (few experts with tall tiles and a long K, bf16): the halves' fp32 partial sums take the
 *           place of y in the workspace and the combine adds them, first half first, before it rounds a
 *           row to bf16.  moe_grouped_gemm_down itself always reduces over the whole of K (plan[1..5]
 *           with which = 1 describe what moe_forward launches), so for such a problem the two differ in
 *           the order of the fp32 sum, both inside the stated tolerance.
 * Returns MOE_OK or the error code of the problem statement. */
enum { MOE_GEMM_PLAN_INTS = 8 };
MOE_API int moe_gemm_plan(const moe_config *cfg, int which, int32_t *plan /* HOST, MOE_GEMM_PLAN_INTS */);

/* Bytes of device scratch moe_route / moe_forward need for this problem. */
MOE_API size_t moe_route_workspace_size(const moe_config *cfg);
MOE_API size_t moe_workspace_size(const moe_config *cfg);

/*
 * Routing (paper Sec. 4.5 "Routing": score all experts per token, keep the top-k).
 * Logits z[t,e] = sum_h x[t,h] * router_w[e,h] in fp32, then the scoring rule of
 * cfg; one wavefront per token selects the k experts with cross-lane exchanges.
 *   x         [T,H] bf16, or fp8 e4m3 with x_scale [T,H/128] fp32 (else x_scale NULL);
 *             with cfg->quantize_x the router is handed the bf16 tensor whatever cfg->dtype says
 *   router_w  [E,H] fp32;  bias [E] fp32 or NULL (added to the choice key only)
 *   ids_out   [T,k] int32, experts in descending key order, equal keys -> lower index
 *   w_out     [T,k] fp32, w = s[id] (/ sum over the k if renormalize) * routed_scale
 *   workspace device scratch of at least moe_route_workspace_size(cfg) bytes
 * Non-finite inputs give unspecified but in-range ids.
 */
MOE_API int moe_route(const moe_config *cfg, const void *x, const float *x_scale, const float *router_w,
              const float *bias, int32_t *ids_out, float *w_out,
              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Activation quantisation for the fp8 expert GEMMs (paper Sec. 4.3, kernel table: the fp8
 * MoE operator's "packing and scaling"; DeepSeek-V3 style 1x128 activation blocks):
 *   scale[t,b] = max |x[t, 128b .. 128b+127]| / 448      (1 when the block is all zero)
 *   q[t,c]     = e4m3( x[t,c] / scale[t,c/128] )         round to nearest even, |.| <= 448
 * with both divisions in IEEE binary32, so the result is the same bits on every run and machine.
 *   x [T,H] bf16 -> xq_out [T,H] fp8 e4m3 (OCP e4m3fn), x_scale_out [T,H/128] fp32; H % 128 == 0.
 * cfg->dtype and cfg->quantize_x are not consulted; T and H are.
 */
MOE_API int moe_quantize_act(const moe_config *cfg, const void *x, void *xq_out, float *x_scale_out, void *stream);

/*
 * Sort-scatter (paper Sec. 4.5: reorder tokens by expert into contiguous memory).
 * A stable counting sort of the P pairs by expert id:
 *   ids          [P] int32 (= the [T,k] routing result); an id outside the local expert
 *                range drops the pair
 *   offsets_out  [EL+1] int32, first sorted row of each local expert; offsets[EL] = kept pairs
 *   sorted_pair_out [P] int32, pair stored at each sorted row (ascending p inside an expert)
 *   inv_out      [P] int32, sorted row of each pair (-1 for a dropped pair)
 *   tiles_out    [moe_max_tiles(cfg)] records of at most moe_tile_rows(cfg) rows (an expert with
 *                more rows is cut into the fewest such tiles, of equal height rounded up to
 *                16 rows), in schedule order (see moe_tile), none for an expert without tokens
 *                (such experts cost nothing downstream); `expert` counts from the first local expert (it
 *                indexes w1 / w2)
 *   sched_out    [MOE_SCHED_INTS] int32: records written and the work ranges (see moe_tile)
 */
MOE_API int moe_permute(const moe_config *cfg, const int32_t *ids, int32_t *offsets_out,
                int32_t *sorted_pair_out, int32_t *inv_out, moe_tile *tiles_out,
                int32_t *sched_out, void *stream);

/*
 * Gate/up grouped GEMM with fused SiLU gating (paper Sec. 4.5: "up" and "gate"
 * projection combined via SiLU, on matrix cores with double-buffered tiles).
 * For sorted row r of expert e holding pair p (token t = p / k):
 *   g = x[t,:] . w1[e,i,:],  u = x[t,:] . w1[e,I+i,:],  act[r,i] = g*sigmoid(g)*u
 *   w1 [EL,2I,H] (rows [0,I) gate, [I,2I) up), fp32 accumulation.
 *   bf16: act_out [P,I] bf16, scales NULL.
 *   fp8 : w1_scale [EL,2I/128,H/128], x_scale [T,H/128]; act_out [P,I] fp8 e4m3 and
 *         act_scale_out [P,I/128] fp32 (act re-quantised per 1x128 block, scale = amax/448).
 */
MOE_API int moe_grouped_gemm_swiglu(const moe_config *cfg, const void *x, const float *x_scale,
                            const void *w1, const float *w1_scale, const int32_t *sorted_pair,
                            const moe_tile *tiles, const int32_t *sched,
                            void *act_out, float *act_scale_out, void *stream);

/*
 * Down grouped GEMM (paper Sec. 4.5: "then a down-projection"):
 *   y[r,h] = act[r,:] . w2[e,h,:],  w2 [EL,H,I], fp32 accumulation, y_out [P,H] bf16.
 *   fp8: act_scale [P,I/128], w2_scale [EL,H/128,I/128]; else NULL.
 */
MOE_API int moe_grouped_gemm_down(const moe_config *cfg, const void *act, const float *act_scale,
                          const void *w2, const float *w2_scale, const moe_tile *tiles,
                          const int32_t *sched, void *y_out, void *stream);

/*
 * Weighted combine: out[t,:] = sum_{j<k} w[t,j] * y[inv[t*k+j],:], summed in slot
 * order in fp32 (no atomics), rounded to bf16 (nearest-even).  Dropped pairs
 * (inv < 0) contribute nothing.
 * The paper's description of the operator (Sec. 4.5) ends with the down projection and
 * defines no combine; this step is what the definition of a top-k MoE layer adds to it:
 * a token's output is the sum of its k experts' outputs, each times its routing weight.
 *   y [P,H] bf16, w [T,k] fp32, inv [P] int32, out [T,H] bf16.
 */
MOE_API int moe_combine(const moe_config *cfg, const void *y, const float *w, const int32_t *inv,
                void *out, void *stream);

/*
 * The whole layer (paper Sec. 4.5: routing, sort-scatter, expert FFN; the paper names no
 * entry point of its own, the argument list is the problem statement: hidden states,
 * router weights, expert weights, optional block scales): the five steps above enqueued back to back on `stream`,
 * intermediates in `workspace` (>= moe_workspace_size(cfg) bytes, 256-byte aligned).
 * bias / *_scale may be NULL as described per step.  out [T,H] bf16.
 * With cfg->quantize_x, x is [T,H] bf16 and x_scale is ignored: moe_quantize_act runs first
 * (its outputs live in the workspace), the router reads the bf16 x, the gate/up GEMM the
 * quantised copy.
 */
MOE_API int moe_forward(const moe_config *cfg, const void *x, const float *x_scale, const float *router_w,
                const float *bias, const void *w1, const float *w1_scale, const void *w2,
                const float *w2_scale, void *out, void *workspace, size_t workspace_bytes,
                void *stream);

/*
 * Latency-bound problems in one launch (paper Sec. 4.5 weighs one persistent kernel against a
 * pipeline of several launches and finds the pipeline faster; so it is here, see below).  When
 * switched on, moe_forward runs small bf16 problems - at most 1024 (token, slot) pairs, at most
 * 256 experts, row tiles of at most 64 rows and expert matrices small enough that the narrow GEMM
 * workgroups are used - as ONE persistent kernel instead of one kernel per step.  Its phases run the
 * same device code as the stand-alone kernels and give the same bits in the output and in every
 * intermediate of the workspace; they are separated by grid-wide barriers on counters in
 * library-owned device memory, so two such launches must not overlap on one device (launches on one
 * stream never do).  Waits are bounded: see moe_single_launch_timeouts.
 * Off by default: back to back on one stream the pipeline's launches overlap with its kernels and it
 * is the faster of the two on the device (16 tokens, 8 experts of 256 x 128: 22 us against 25 us per
 * layer; inside the one launch: routing 7 us, sort-scatter + gate/up 8 us, down 3 us, combine 2 us,
 * three barriers 4 us - every phase is a chain of dependent memory round trips that the pipeline
 * overlaps with its next launch); the single launch costs the calling thread a quarter of the time
 * (4 us against 18 us per layer), which is what a host-bound caller buys with it.
 *   moe_single_launch(enable)       process-wide switch
 *   moe_single_launch_mode(cfg)     MOE_SINGLE_LAUNCH_ALL if moe_forward would run cfg as one launch
 *                                   right now, else MOE_SINGLE_LAUNCH_NONE (negative: error code)
 *   moe_single_launch_timeouts(&n)  barrier waits given up on the current device since the library was
 *                                   loaded (0 unless the device was so busy with other work that a
 *                                   launch could not become resident within about two seconds; the
 *                                   output of such a launch is undefined).  Copies from the device: it
 *                                   synchronises with the device's work.
 */
enum { MOE_SINGLE_LAUNCH_NONE = 0, MOE_SINGLE_LAUNCH_ALL = 1 };
MOE_API void moe_single_launch(int enable);
MOE_API int moe_single_launch_mode(const moe_config *cfg);
MOE_API int moe_single_launch_timeouts(uint32_t *count_out /* HOST */);

/*
 * moe_forward with step boundaries marked for timing: `events` is a HOST array of
 * MOE_FORWARD_EVENTS hipEvent_t handles (created by the caller) that are recorded
 * on `stream` before routing and after each of the five steps, in pipeline order
 * (route, sort-scatter, gate/up GEMM, down GEMM, combine; with cfg->quantize_x the
 * quantisation of x is inside the first interval).  The kernels and their
 * launch configuration are exactly those of moe_forward; where one launch covers all the
 * steps (see moe_single_launch) their events are all recorded after it, so the first
 * interval holds the whole launch and the others are empty.
 */
enum { MOE_FORWARD_EVENTS = 6 };
MOE_API int moe_forward_marked(const moe_config *cfg, const void *x, const float *x_scale, const float *router_w,
                       const float *bias, const void *w1, const float *w1_scale, const void *w2,
                       const float *w2_scale, void *out, void *workspace, size_t workspace_bytes,
                       void *stream, void *const *events);

/*
 * moe_forward for callers that cannot allocate device memory or pass a workspace: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * intermediates live in a buffer the library itself holds on every device it runs on
 * (MOE_STATIC_SCRATCH_BYTES, static device memory, kept until the process ends); the call
 * allocates and frees nothing, on the host or the device.  Same kernels, same results, bit for
 * bit, as moe_forward.
 *   - A problem whose moe_workspace_size(cfg) exceeds MOE_STATIC_SCRATCH_BYTES is refused with
 *     MOE_ERR_WORKSPACE before anything is enqueued (the benchmark-sized decode and Mixtral-shaped
 *     layers fit; the 4096-token DeepSeek-shaped prefill does not: use moe_forward there).
 *   - All calls on one device share that buffer: two such calls must not overlap on the device
 *     (put them on one stream, or order the streams); overlapping calls race.  Nothing in the
 *     buffer has to start at zero and nothing is kept from one call to the next.
 *   - The buffer's address is looked up on the first call on a device; moe_init() does the same
 *     lookup for the current device ahead of time (call it before a graph capture starts).
 */
enum { MOE_STATIC_SCRATCH_BYTES = 64 << 20 };
MOE_API int moe_init(void);
MOE_API int moe_forward_static(const moe_config *cfg, const void *x, const float *x_scale, const float *router_w,
                               const float *bias, const void *w1, const float *w1_scale, const void *w2,
                               const float *w2_scale, void *out, void *stream);

/* Text for an error code; the hipError_t of the last failed launch on this thread. */
MOE_API const char *moe_error_string(int code);
MOE_API int moe_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H */
