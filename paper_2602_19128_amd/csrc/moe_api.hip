// C ABI of the MoE library: argument checks, workspace carving, step sequencing.
#include "moe_internal.hpp"

#include <math.h>

namespace moe {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

namespace {

int route_epl(int E) { return E <= 64 ? 1 : E <= 128 ? 2 : E <= 256 ? 4 : 8; }
bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

int validate(const moe_config *c)
{
    if (c == nullptr) return MOE_ERR_INVALID;
    if (c->T < 0 || c->H <= 0 || c->I <= 0 || c->E <= 0 || c->top_k <= 0) return MOE_ERR_INVALID;
    if (c->top_k > c->E) return MOE_ERR_INVALID;
    if (c->scoring != MOE_SCORE_SOFTMAX && c->scoring != MOE_SCORE_SIGMOID) return MOE_ERR_INVALID;
    if (c->dtype != MOE_DTYPE_BF16 && c->dtype != MOE_DTYPE_FP8_E4M3) return MOE_ERR_INVALID;
    if (c->E > kMaxExperts || c->top_k > kMaxTopK) return MOE_ERR_UNSUPPORTED;
    if (c->H % 64 != 0 || c->I % 64 != 0) return MOE_ERR_UNSUPPORTED;
    if (c->dtype == MOE_DTYPE_FP8_E4M3 && (c->H % kQBlock != 0 || c->I % kQBlock != 0)) return MOE_ERR_UNSUPPORTED;
    // fp8 GEMMs keep a column slab's weight scales for the whole contraction in two registers per lane
    if (c->dtype == MOE_DTYPE_FP8_E4M3 && (c->H > kMaxScaleBlocks * kQBlock || c->I > kMaxScaleBlocks * kQBlock))
        return MOE_ERR_UNSUPPORTED;
    if ((long long)c->T * c->top_k > (1ll << 30)) return MOE_ERR_UNSUPPORTED;
    if (c->local_expert_offset < 0 || c->num_local_experts < 0) return MOE_ERR_INVALID;
    if (c->num_local_experts == 0 && c->local_expert_offset != 0) return MOE_ERR_INVALID;
    if (c->local_expert_offset + c->num_local_experts > c->E) return MOE_ERR_INVALID;
    if (c->quantize_x != 0 && c->quantize_x != 1) return MOE_ERR_INVALID;
    if (c->quantize_x == 1 && c->dtype != MOE_DTYPE_FP8_E4M3) return MOE_ERR_INVALID;
    if (c->n_group > 1) {
        if (c->E % c->n_group != 0) return MOE_ERR_INVALID;
        const int gsz = c->E / c->n_group;
        if (c->topk_group < 1 || c->topk_group > c->n_group) return MOE_ERR_INVALID;
        if (c->group_score_topn < 1 || c->group_score_topn > gsz) return MOE_ERR_INVALID;
        if (c->top_k > c->topk_group * gsz) return MOE_ERR_INVALID;
        const int epl = route_epl(c->E);
        if (gsz % epl != 0 || !is_pow2(gsz / epl)) return MOE_ERR_UNSUPPORTED;
    }
    return MOE_OK;
}

// Tile height: the smallest of 16..256 that holds an expert's rows with a binomial safety
// margin (mean + 4 sigma of a balanced router), so that almost every expert is one tile and its
// weights are streamed exactly once.
int tile_rows_for(const moe_config &c)
{
    const double mean = (double)c.T * c.top_k / c.E;
    const double want = mean + 4.0 * sqrt(mean);
    int rows = 16;
    while (rows < 256 && rows < want) rows *= 2;
    return rows;
}

int max_tiles_for(const moe_config &c)
{
    const int P = c.T * c.top_k;
    const int el = local_experts(c);
    return ceil_div(P, tile_rows_for(c)) + (P < el ? P : el);
}

// Workspace sections of moe_forward, in order, each 256-byte aligned.
struct Layout {
    size_t route, ids, w, offsets, sorted_pair, inv, tiles, sched, act, act_scale, y, xq, xq_scale, total;
};

// The problem as the router sees it: with quantise-on-the-path the router scores the bf16 hidden
// states the layer received, not the fp8 copy made for the experts.
moe_config router_view(const moe_config &c)
{
    moe_config r = c;
    if (c.quantize_x) r.dtype = MOE_DTYPE_BF16;
    return r;
}

Layout layout_for(const moe_config &c)
{
    const size_t P = (size_t)c.T * c.top_k;
    const size_t act_elem = c.dtype == MOE_DTYPE_FP8_E4M3 ? 1 : 2;
    Layout l;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off += align_up(bytes ? bytes : 1, 256); return at; };
    l.route = take(route_workspace_bytes(router_view(c)));
    l.ids = take(P * sizeof(int32_t));
    l.w = take(P * sizeof(float));
    l.offsets = take(((size_t)local_experts(c) + 1) * sizeof(int32_t));
    l.sorted_pair = take(P * sizeof(int32_t));
    l.inv = take(P * sizeof(int32_t));
    l.tiles = take((size_t)max_tiles_for(c) * sizeof(moe_tile));
    l.sched = take(MOE_SCHED_INTS * sizeof(int32_t));
    l.act = take(P * c.I * act_elem);
    l.act_scale = take(c.dtype == MOE_DTYPE_FP8_E4M3 ? P * (c.I / kQBlock) * sizeof(float) : 0);
    l.y = take(P * c.H * (down_k_split(c, tile_rows_for(c)) > 1 ? 2 * sizeof(float) : 2));   // bf16 rows, or two fp32 partial sums
    l.xq = take(c.quantize_x ? (size_t)c.T * c.H : 0);
    l.xq_scale = take(c.quantize_x ? (size_t)c.T * (c.H / kQBlock) * sizeof(float) : 0);
    l.total = off;
    return l;
}

bool fp8(const moe_config *c) { return c->dtype == MOE_DTYPE_FP8_E4M3; }

// Library-owned workspace of moe_forward_static: one array per device, held until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; what kernels and copies get
// is the per-device address looked up below.
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_SCRATCH_BYTES];

std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Address of `scratch` on the current device (looked up once per device; the lookup is idempotent, so
// two threads racing through it store the same value).
int static_scratch(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_last_hip_error(e); return MOE_ERR_HIP; }
    if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_UNSUPPORTED;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr) { set_last_hip_error(e); return MOE_ERR_HIP; }
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return MOE_OK;
}

}  // namespace
}  // namespace moe

using namespace moe;

extern "C" {

int32_t moe_tile_rows(const moe_config *cfg) { return validate(cfg) == MOE_OK ? tile_rows_for(*cfg) : 0; }
int32_t moe_max_tiles(const moe_config *cfg) { return validate(cfg) == MOE_OK ? max_tiles_for(*cfg) : 0; }

int moe_gemm_plan(const moe_config *cfg, int which, int32_t *plan)
{
    const int rc = validate(cfg);
    if (rc != MOE_OK) return rc;
    if (!plan || (which != 0 && which != 1)) return MOE_ERR_INVALID;
    const bool swiglu = which == 0, f8 = fp8(cfg);
    const int rows = tile_rows_for(*cfg), est = expected_tiles(*cfg);
    const int ks = swiglu ? 1 : down_k_split(*cfg, rows);
    const GemmWidth wd = ks > 1 ? GEMM_WIDE : gemm_width(rows / 16, swiglu, f8, swiglu ? cfg->I : cfg->H, est);
    const int waves = wd == GEMM_NARROW ? 4 : 8;
    const int blocks = wd == GEMM_WIDE4 ? 4 : 2;
    for (int i = 0; i < MOE_GEMM_PLAN_INTS; ++i) plan[i] = 0;
    plan[0] = rows;
    plan[1] = waves;
    plan[2] = blocks;
    plan[3] = waves * (swiglu ? 16 : 16 * blocks);
    plan[4] = est <= 8 * MOE_WORK_RANGES ? 1 : 0;
    plan[5] = (waves >= 8 && !(f8 && swiglu) && ks == 1) ? 1 : 0;
    plan[6] = ks;
    return MOE_OK;
}

size_t moe_route_workspace_size(const moe_config *cfg)
{
    return validate(cfg) == MOE_OK ? route_workspace_bytes(router_view(*cfg)) : 0;
}

size_t moe_workspace_size(const moe_config *cfg) { return validate(cfg) == MOE_OK ? layout_for(*cfg).total : 0; }

int moe_route(const moe_config *cfg, const void *x, const float *x_scale, const float *router_w,
              const float *bias, int32_t *ids_out, float *w_out, void *workspace, size_t workspace_bytes,
              void *stream)
{
    int rc = validate(cfg);
    if (rc != MOE_OK) return rc;
    if (cfg->T == 0) return MOE_OK;
    if (!x || !router_w || !ids_out || !w_out || !workspace) return MOE_ERR_INVALID;
    const moe_config rv = router_view(*cfg);
    if (fp8(&rv) && !x_scale) return MOE_ERR_INVALID;
    if (workspace_bytes < route_workspace_bytes(rv)) return MOE_ERR_WORKSPACE;
    return launch_route(rv, x, fp8(&rv) ? x_scale : nullptr, router_w, bias, ids_out, w_out, workspace,
                        (hipStream_t)stream);
}

int moe_quantize_act(const moe_config *cfg, const void *x, void *xq_out, float *x_scale_out, void *stream)
{
    if (cfg == nullptr || cfg->T < 0 || cfg->H <= 0) return MOE_ERR_INVALID;
    if (cfg->H % kQBlock != 0) return MOE_ERR_UNSUPPORTED;
    if ((long long)cfg->T * cfg->H > (1ll << 40)) return MOE_ERR_UNSUPPORTED;
    if (cfg->T == 0) return MOE_OK;
    if (!x || !xq_out || !x_scale_out) return MOE_ERR_INVALID;
    return launch_quantize_act(*cfg, x, xq_out, x_scale_out, (hipStream_t)stream);
}

int moe_permute(const moe_config *cfg, const int32_t *ids, int32_t *offsets_out, int32_t *sorted_pair_out,
                int32_t *inv_out, moe_tile *tiles_out, int32_t *sched_out, void *stream)
{
    int rc = validate(cfg);
    if (rc != MOE_OK) return rc;
    if (!offsets_out || !sched_out) return MOE_ERR_INVALID;
    if (cfg->T > 0 && (!ids || !sorted_pair_out || !inv_out || !tiles_out)) return MOE_ERR_INVALID;
    return launch_permute(*cfg, tile_rows_for(*cfg), max_tiles_for(*cfg), ids, offsets_out, sorted_pair_out,
                          inv_out, tiles_out, sched_out, (hipStream_t)stream);
}

int moe_grouped_gemm_swiglu(const moe_config *cfg, const void *x, const float *x_scale, const void *w1,
                            const float *w1_scale, const int32_t *sorted_pair, const moe_tile *tiles,
                            const int32_t *sched, void *act_out, float *act_scale_out, void *stream)
{
    int rc = validate(cfg);
    if (rc != MOE_OK) return rc;
    if (cfg->T == 0) return MOE_OK;
    if (!x || !w1 || !sorted_pair || !tiles || !sched || !act_out) return MOE_ERR_INVALID;
    if (fp8(cfg) && (!x_scale || !w1_scale || !act_scale_out)) return MOE_ERR_INVALID;
    return launch_gemm_swiglu(*cfg, tile_rows_for(*cfg), max_tiles_for(*cfg), x, x_scale, w1, w1_scale,
                              sorted_pair, tiles, sched, act_out, act_scale_out, (hipStream_t)stream);
}

int moe_grouped_gemm_down(const moe_config *cfg, const void *act, const float *act_scale, const void *w2,
                          const float *w2_scale, const moe_tile *tiles, const int32_t *sched, void *y_out,
                          void *stream)
{
    int rc = validate(cfg);
    if (rc != MOE_OK) return rc;
    if (cfg->T == 0) return MOE_OK;
    if (!act || !w2 || !tiles || !sched || !y_out) return MOE_ERR_INVALID;
    if (fp8(cfg) && (!act_scale || !w2_scale)) return MOE_ERR_INVALID;
    return launch_gemm_down(*cfg, tile_rows_for(*cfg), max_tiles_for(*cfg), 1, act, act_scale, w2, w2_scale, tiles,
                            sched, y_out, (hipStream_t)stream);
}

int moe_combine(const moe_config *cfg, const void *y, const float *w, const int32_t *inv, void *out,
                void *stream)
{
    int rc = validate(cfg);
    if (rc != MOE_OK) return rc;
    if (cfg->T == 0) return MOE_OK;
    if (!y || !w || !inv || !out) return MOE_ERR_INVALID;
    return launch_combine(*cfg, y, w, inv, out, (hipStream_t)stream);
}

int moe_forward_marked(const moe_config *cfg, const void *x, const float *x_scale, const float *router_w,
                       const float *bias, const void *w1, const float *w1_scale, const void *w2,
                       const float *w2_scale, void *out, void *workspace, size_t workspace_bytes,
                       void *stream, void *const *events)
{
    int rc = validate(cfg);
    if (rc != MOE_OK) return rc;
    if (cfg->T == 0) return MOE_OK;
    if (!x || !router_w || !w1 || !w2 || !out || !workspace) return MOE_ERR_INVALID;
    if (fp8(cfg) && ((!x_scale && !cfg->quantize_x) || !w1_scale || !w2_scale)) return MOE_ERR_INVALID;
    if (((uintptr_t)workspace & 255u) != 0) return MOE_ERR_INVALID;
    const Layout l = layout_for(*cfg);
    if (workspace_bytes < l.total) return MOE_ERR_WORKSPACE;

    unsigned char *ws = static_cast<unsigned char *>(workspace);
    int32_t *ids = reinterpret_cast<int32_t *>(ws + l.ids);
    float *w = reinterpret_cast<float *>(ws + l.w);
    int32_t *offsets = reinterpret_cast<int32_t *>(ws + l.offsets);
    int32_t *sorted_pair = reinterpret_cast<int32_t *>(ws + l.sorted_pair);
    int32_t *inv = reinterpret_cast<int32_t *>(ws + l.inv);
    moe_tile *tiles = reinterpret_cast<moe_tile *>(ws + l.tiles);
    int32_t *sched = reinterpret_cast<int32_t *>(ws + l.sched);
    void *act = ws + l.act;
    float *act_scale = fp8(cfg) ? reinterpret_cast<float *>(ws + l.act_scale) : nullptr;
    void *y = ws + l.y;
    hipStream_t s = (hipStream_t)stream;
    const int tr = tile_rows_for(*cfg), mt = max_tiles_for(*cfg);
    int mark_at = 0;
    auto mark = [&]() -> int {
        if (events == nullptr) return MOE_OK;
        hipError_t e = hipEventRecord((hipEvent_t)events[mark_at++], s);
        if (e != hipSuccess) { set_last_hip_error(e); return MOE_ERR_HIP; }
        return MOE_OK;
    };

    if ((rc = mark()) != MOE_OK) return rc;
    if (single_launch_mode(*cfg, tr) == MOE_SINGLE_LAUNCH_ALL) {
        rc = launch_fused(*cfg, tr, mt, x, router_w, bias, ws + l.route, ids, w, offsets, sorted_pair, inv, tiles,
                          sched, w1, w2, act, y, out, s);
        if (rc != MOE_ERR_UNSUPPORTED) {                      // (a device too small for it takes the pipeline)
            for (int i = 0; rc == MOE_OK && i < 5; ++i) rc = mark();   // the one launch has done all five steps
            return rc;
        }
    }
    const void *x_route = x;                                  // what the router scores
    const float *x_route_scale = x_scale;
    if (cfg->quantize_x) {
        // bf16 hidden states in: the experts read the e4m3 copy made here, the router the original
        float *xq_scale = reinterpret_cast<float *>(ws + l.xq_scale);
        rc = launch_quantize_act(*cfg, x, ws + l.xq, xq_scale, s);
        if (rc != MOE_OK) return rc;
        x = ws + l.xq;
        x_scale = xq_scale;
        x_route_scale = nullptr;
    }
    rc = launch_route(router_view(*cfg), x_route, x_route_scale, router_w, bias, ids, w, ws + l.route, s);
    if (rc != MOE_OK || (rc = mark()) != MOE_OK) return rc;
    rc = launch_permute(*cfg, tr, mt, ids, offsets, sorted_pair, inv, tiles, sched, s);
    if (rc != MOE_OK || (rc = mark()) != MOE_OK) return rc;
    rc = launch_gemm_swiglu(*cfg, tr, mt, x, x_scale, w1, w1_scale, sorted_pair, tiles, sched, act, act_scale, s);
    if (rc != MOE_OK || (rc = mark()) != MOE_OK) return rc;
    const int ks = down_k_split(*cfg, tr);
    rc = launch_gemm_down(*cfg, tr, mt, ks, act, act_scale, w2, w2_scale, tiles, sched, y, s);
    if (rc != MOE_OK || (rc = mark()) != MOE_OK) return rc;
    rc = launch_combine(*cfg, y, w, inv, out, s, ks);
    if (rc != MOE_OK) return rc;
    return mark();
}

int moe_forward(const moe_config *cfg, const void *x, const float *x_scale, const float *router_w,
                const float *bias, const void *w1, const float *w1_scale, const void *w2,
                const float *w2_scale, void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    return moe_forward_marked(cfg, x, x_scale, router_w, bias, w1, w1_scale, w2, w2_scale, out, workspace,
                              workspace_bytes, stream, nullptr);
}

void moe_single_launch(int enable) { set_single_launch(enable); }

int moe_single_launch_mode(const moe_config *cfg)
{
    const int rc = validate(cfg);
    if (rc != MOE_OK) return rc;
    return single_launch_mode(*cfg, tile_rows_for(*cfg));
}

int moe_single_launch_timeouts(uint32_t *count_out)
{
    if (!count_out) return MOE_ERR_INVALID;
    unsigned n = 0;
    const int rc = single_launch_timeouts(&n);
    *count_out = n;
    return rc;
}

int moe_init(void)
{
    void *p = nullptr;
    return static_scratch(&p);
}

int moe_forward_static(const moe_config *cfg, const void *x, const float *x_scale, const float *router_w,
                       const float *bias, const void *w1, const float *w1_scale, const void *w2,
                       const float *w2_scale, void *out, void *stream)
{
    int rc = validate(cfg);
    if (rc != MOE_OK) return rc;
    if (cfg->T == 0) return MOE_OK;
    if (layout_for(*cfg).total > (size_t)MOE_STATIC_SCRATCH_BYTES) return MOE_ERR_WORKSPACE;   // before anything touches the device
    void *ws = nullptr;
    if ((rc = static_scratch(&ws)) != MOE_OK) return rc;
    return moe_forward_marked(cfg, x, x_scale, router_w, bias, w1, w1_scale, w2, w2_scale, out, ws,
                              (size_t)MOE_STATIC_SCRATCH_BYTES, stream, nullptr);
}

const char *moe_error_string(int code)
{
    switch (code) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID: return "invalid argument";
    case MOE_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case MOE_ERR_WORKSPACE: return "workspace too small (moe_forward_static: the problem needs more than the static scratch)";
    case MOE_ERR_HIP: return "HIP launch failed";
    default: return "unknown error";
    }
}

int moe_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
