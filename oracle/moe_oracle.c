/*
 * TEST INFRASTRUCTURE -- not part of the product path.
 *
 * Plain CPU definition of one Mixture-of-Experts layer forward, as the operator
 * is described in the paper's MoE kernel analysis (Sec. 4.5: per token, score all
 * experts and keep the top-k; run the chosen experts' "gate" and "up"
 * projections, combine them through SiLU, apply the down projection) and the
 * pipeline it names (routing -> reorder tokens by expert -> expert FFN).  The
 * paper leaves the routing formula, the weighted sum over the k experts and the
 * fp8 scale layout unstated; the readings taken are listed next to each function.
 *
 * Everything is computed straight from the definition in naive loops with
 * double-precision accumulation.  Nothing is blocked, fused or reordered; OpenMP
 * only spreads independent output elements over host threads.  The file shares
 * no code, header, table or helper with the GPU library.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force top-k, closed-form softmax
 * over the selected logits, group-routing reductions, permutation identities,
 * dense-MLP special cases against an independent float64 library matmul, the
 * e4m3 decode against a library conversion of all 256 codes, the 1x128 quantiser
 * against a library float8 conversion and its own error bound, linearity/zero
 * invariants.  The paper prints no numeric values for this operator, so parity
 * against paper-printed numbers is unpinned; every function is pinned by the
 * above instead.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_BF16 = 0, ORACLE_FP8_E4M3 = 1 };
enum { ORACLE_SOFTMAX = 0, ORACLE_SIGMOID = 1 };
#define ORACLE_QBLOCK 128
#if FLT_EVAL_METHOD != 0
#error "float expressions must be evaluated in binary32 (the quantiser's divisions depend on it)"
#endif

/* One problem instance: shapes, routing rule, and host pointers to the inputs. */
typedef struct {
    int32_t T, H, I, E, top_k;
    int32_t scoring;            /* ORACLE_SOFTMAX | ORACLE_SIGMOID */
    int32_t renormalize;        /* divide the k weights by their sum */
    int32_t n_group;            /* <=1: no group limiting */
    int32_t topk_group;
    int32_t group_score_topn;
    int32_t dtype;              /* ORACLE_BF16 | ORACLE_FP8_E4M3 (x, w1, w2 payload type) */
    float   routed_scale;
    const void  *x;             /* [T,H] */
    const float *x_scale;       /* [T,H/128]            (fp8 only) */
    const float *router_w;      /* [E,H] fp32 */
    const float *bias;          /* [E] fp32 or NULL */
    const void  *w1;            /* [E,2I,H]; rows [0,I) gate, [I,2I) up */
    const float *w1_scale;      /* [E,2I/128,H/128]     (fp8 only) */
    const void  *w2;            /* [E,H,I] */
    const float *w2_scale;      /* [E,H/128,I/128]      (fp8 only) */
    /* Local-expert mode (one device's share of the experts; the paper's Sec. 4.5 workload has
     * 32 local experts of 256): only experts [local_offset, local_offset + local_count) have
     * weights -- w1, w2 and their scales then hold local_count experts, indexed from
     * local_offset -- and the layer output is the sum over a token's chosen experts that
     * fall in that range.  local_count = 0: every expert is local. */
    int32_t local_offset, local_count;
    /* Quantise-on-the-path mode (the "fp8 packing and scaling" step the paper's kernel table,
     * Sec. 4.3, names as this operator's challenge, taken into the layer): the layer received
     * bf16 hidden states x_bf16 [T,H] and quantised them itself with
     * oracle_quantize_rows_1x128; x / x_scale above hold that result and feed the experts,
     * while the router scores the hidden states as they arrived.  NULL: x arrived quantised
     * (or the layer is bf16) and the router reads x. */
    const uint16_t *x_bf16;
} oracle_problem;

/* ---- element decoding ---------------------------------------------------- */

/* bf16 is the upper half of an IEEE binary32. */
double oracle_bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* OCP e4m3fn: 1 sign, 4 exponent (bias 7), 3 mantissa bits; no infinities;
 * S.1111.111 is NaN; exponent 0 is subnormal with value m/8 * 2^-6. */
double oracle_e4m3_to_f64(uint8_t b)
{
    int s = b >> 7, e = (b >> 3) & 15, m = b & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

/* ---- activation quantisation ---------------------------------------------- */

/* Nearest e4m3 code to v (ties -> the code with an even mantissa field), magnitudes beyond the
 * largest finite value 448 saturate to it.  Written as a search over all 127 non-negative finite
 * codes so that it rests on oracle_e4m3_to_f64 alone. */
uint8_t oracle_f32_to_e4m3(float v)
{
    const double a = fabs((double)v);
    int best = 0;
    double best_d = INFINITY;
    if (isnan(v)) return 0x7f;
    for (int c = 0; c <= 0x7e; ++c) {
        const double d = fabs(oracle_e4m3_to_f64((uint8_t)c) - a);
        if (d < best_d || (d == best_d && (c & 1) == 0)) { best_d = d; best = c; }
    }
    return (uint8_t)(best | (signbit(v) ? 0x80 : 0));
}

/*
 * Per-token, per-128-column quantisation of bf16 rows to e4m3 with one fp32 scale per block
 * (DeepSeek-V3 style 1x128 activation blocks):
 *   scale[r,b] = amax(|x[r, 128b .. 128b+127]|) / 448        (1 when the block is all zero)
 *   q[r,c]     = e4m3_nearest_even( x[r,c] / scale[r,c/128] )
 * The codes are integers decided by floating point, so the precision of the two divisions is
 * part of the definition: both are IEEE binary32 divisions (bf16 values are exact in binary32;
 * float expressions are evaluated in binary32 on the SSE targets this file is built for).
 */
void oracle_quantize_rows_1x128(int32_t R, int32_t K, const uint16_t *x /* [R,K] bf16 */,
                                uint8_t *q /* [R,K] */, float *scale /* [R,K/128] */)
{
    const int nb = K / ORACLE_QBLOCK;
#pragma omp parallel for collapse(2) schedule(static)
    for (int r = 0; r < R; ++r)
        for (int b = 0; b < nb; ++b) {
            const uint16_t *xb = x + (size_t)r * K + (size_t)b * ORACLE_QBLOCK;
            float amax = 0.0f;
            for (int c = 0; c < ORACLE_QBLOCK; ++c) {
                const float v = fabsf((float)oracle_bf16_to_f64(xb[c]));
                if (v > amax) amax = v;
            }
            const float sc = amax > 0.0f ? amax / 448.0f : 1.0f;
            scale[(size_t)r * nb + b] = sc;
            for (int c = 0; c < ORACLE_QBLOCK; ++c) {
                const float v = (float)oracle_bf16_to_f64(xb[c]) / sc;   /* binary32 quotient */
                q[(size_t)r * K + (size_t)b * ORACLE_QBLOCK + c] = oracle_f32_to_e4m3(v);
            }
        }
}

static double payload(const void *p, int dtype, size_t idx)
{
    if (dtype == ORACLE_FP8_E4M3) return oracle_e4m3_to_f64(((const uint8_t *)p)[idx]);
    return oracle_bf16_to_f64(((const uint16_t *)p)[idx]);
}

/* Hidden state x[t,h]; fp8: payload times the scale of its 1x128 block. */
static double x_at(const oracle_problem *q, int t, int h)
{
    double v = payload(q->x, q->dtype, (size_t)t * q->H + h);
    if (q->dtype == ORACLE_FP8_E4M3)
        v *= (double)q->x_scale[(size_t)t * (q->H / ORACLE_QBLOCK) + h / ORACLE_QBLOCK];
    return v;
}

/* Hidden state as the router sees it: the bf16 tensor the layer received when it quantises
 * x itself, else x. */
static double x_route_at(const oracle_problem *q, int t, int h)
{
    if (q->x_bf16) return oracle_bf16_to_f64(q->x_bf16[(size_t)t * q->H + h]);
    return x_at(q, t, h);
}

/* Weight W[e,n,c] of an [E,N,K] tensor; fp8: payload times the scale of its
 * 128x128 block, scale tensor [E,N/128,K/128]. */
static double w_at(const void *w, const float *scale, int dtype, int N, int K, int e, int n, int c)
{
    double v = payload(w, dtype, ((size_t)e * N + n) * K + c);
    if (dtype == ORACLE_FP8_E4M3)
        v *= (double)scale[((size_t)e * (N / ORACLE_QBLOCK) + n / ORACLE_QBLOCK) * (K / ORACLE_QBLOCK)
                           + c / ORACLE_QBLOCK];
    return v;
}

/* ---- routing ------------------------------------------------------------- */

/* Router logits of one token: z[e] = sum_h x[t,h] * Wr[e,h]. */
static void logits_token(const oracle_problem *q, int t, double *z)
{
    for (int e = 0; e < q->E; ++e) {
        double acc = 0.0;
        for (int h = 0; h < q->H; ++h)
            acc += x_route_at(q, t, h) * (double)q->router_w[(size_t)e * q->H + h];
        z[e] = acc;
    }
}

void oracle_router_logits(const oracle_problem *q, double *z /* [T,E] */)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < q->T; ++t) logits_token(q, t, z + (size_t)t * q->E);
}

/*
 * Scores -> k experts + weights for one token.
 *
 * softmax rule : s = softmax over all experts; choice key c = s.
 * sigmoid rule : s = 1/(1+exp(-z)); choice key c = s + bias (bias steers the
 *                choice only; the weight uses the unbiased s).
 * group limit  : experts form n_group contiguous blocks; a block's score is the
 *                sum of its group_score_topn largest keys; only experts in the
 *                topk_group best blocks stay eligible.
 * choice       : the k eligible experts with the largest key, reported in
 *                descending key order; equal keys -> lower index first (for
 *                experts and for blocks).
 * weights      : w_j = s[id_j], divided by their sum when renormalize is set,
 *                then times routed_scale.
 * margin       : how far the decision is from flipping: min of (k-th chosen key
 *                - best eligible key left out) and (worst kept block score - best
 *                dropped block score); +inf where nothing is left out.
 */
static void route_token(const oracle_problem *q, const double *z, int32_t *ids, double *w, double *margin)
{
    const int E = q->E, k = q->top_k;
    double *s = (double *)malloc(sizeof(double) * E);
    double *c = (double *)malloc(sizeof(double) * E);
    char *eligible = (char *)malloc(E);
    char *taken = (char *)calloc(E, 1);
    double mg = INFINITY;

    if (q->scoring == ORACLE_SOFTMAX) {
        double zmax = z[0], den = 0.0;
        for (int e = 1; e < E; ++e) if (z[e] > zmax) zmax = z[e];
        for (int e = 0; e < E; ++e) den += exp(z[e] - zmax);
        for (int e = 0; e < E; ++e) s[e] = exp(z[e] - zmax) / den;
    } else {
        for (int e = 0; e < E; ++e) s[e] = 1.0 / (1.0 + exp(-z[e]));
    }
    for (int e = 0; e < E; ++e) c[e] = s[e] + (q->bias ? (double)q->bias[e] : 0.0);

    memset(eligible, 1, E);
    if (q->n_group > 1) {
        const int G = q->n_group, gsz = E / G;
        double *gs = (double *)malloc(sizeof(double) * G);
        char *kept = (char *)calloc(G, 1);
        char *used = (char *)malloc(gsz);
        for (int g = 0; g < G; ++g) {
            memset(used, 0, gsz);
            gs[g] = 0.0;
            for (int n = 0; n < q->group_score_topn; ++n) {
                int best = -1;
                for (int j = 0; j < gsz; ++j)
                    if (!used[j] && (best < 0 || c[g * gsz + j] > c[g * gsz + best])) best = j;
                used[best] = 1;
                gs[g] += c[g * gsz + best];
            }
        }
        double worst_kept = INFINITY, best_dropped = -INFINITY;
        for (int n = 0; n < q->topk_group; ++n) {
            int best = -1;
            for (int g = 0; g < G; ++g)
                if (!kept[g] && (best < 0 || gs[g] > gs[best])) best = g;
            kept[best] = 1;
            worst_kept = gs[best];
        }
        for (int g = 0; g < G; ++g)
            if (!kept[g] && gs[g] > best_dropped) best_dropped = gs[g];
        if (worst_kept - best_dropped < mg) mg = worst_kept - best_dropped;
        for (int e = 0; e < E; ++e) eligible[e] = kept[e / gsz];
        free(gs); free(kept); free(used);
    }

    double sum = 0.0, kth = INFINITY, left_out = -INFINITY;
    for (int j = 0; j < k; ++j) {
        int best = -1;
        for (int e = 0; e < E; ++e)
            if (eligible[e] && !taken[e] && (best < 0 || c[e] > c[best])) best = e;
        taken[best] = 1;
        ids[j] = best;
        w[j] = s[best];
        sum += s[best];
        kth = c[best];
    }
    for (int e = 0; e < E; ++e)
        if (eligible[e] && !taken[e] && c[e] > left_out) left_out = c[e];
    if (kth - left_out < mg) mg = kth - left_out;
    for (int j = 0; j < k; ++j) {
        if (q->renormalize) w[j] /= sum;
        w[j] *= (double)q->routed_scale;
    }
    *margin = mg;
    free(s); free(c); free(eligible); free(taken);
}

/* Routing for all tokens from given logits z[T,E]. */
void oracle_route(const oracle_problem *q, const double *z,
                  int32_t *ids /* [T,k] */, double *w /* [T,k] */, double *margin /* [T] */)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < q->T; ++t)
        route_token(q, z + (size_t)t * q->E, ids + (size_t)t * q->top_k,
                    w + (size_t)t * q->top_k, margin + t);
}

/* ---- reorder by expert ---------------------------------------------------- */

/*
 * Pairs p = t*k + j are grouped by their expert id, keeping ascending p inside a
 * group (a stable counting sort).  offsets[e] is the first sorted row of expert
 * e and offsets[E] = P; sorted_pair[r] is the pair stored at row r; inv[p] is
 * the row pair p landed on.
 */
void oracle_permute(int32_t P, int32_t E, const int32_t *ids,
                    int32_t *offsets /* [E+1] */, int32_t *sorted_pair /* [P] */, int32_t *inv /* [P] */)
{
    int32_t *cursor = (int32_t *)calloc((size_t)E + 1, sizeof(int32_t));
    for (int e = 0; e <= E; ++e) offsets[e] = 0;
    for (int p = 0; p < P; ++p) offsets[ids[p] + 1] += 1;
    for (int e = 0; e < E; ++e) offsets[e + 1] += offsets[e];
    for (int e = 0; e < E; ++e) cursor[e] = offsets[e];
    for (int p = 0; p < P; ++p) {
        int r = cursor[ids[p]]++;
        sorted_pair[r] = p;
        inv[p] = r;
    }
    free(cursor);
}

/* ---- expert FFN ----------------------------------------------------------- */

/*
 * Gate/up projection + SiLU gating for n (token, expert) rows:
 *   g[i] = sum_h x[t,h] * W1[e,i,h]        (rows [0,I)  of W1[e] = gate)
 *   u[i] = sum_h x[t,h] * W1[e,I+i,h]      (rows [I,2I) of W1[e] = up)
 *   act[r,i] = g * sigmoid(g) * u
 * expert[r] indexes the weight arrays (in local-expert mode: counted from the first local expert).
 */
void oracle_swiglu_rows(const oracle_problem *q, int32_t n, const int32_t *tok, const int32_t *expert,
                        double *act /* [n,I] */)
{
    const int H = q->H, I = q->I;
#pragma omp parallel for collapse(2) schedule(static)
    for (int r = 0; r < n; ++r)
        for (int i = 0; i < I; ++i) {
            const int t = tok[r], e = expert[r];
            double g = 0.0, u = 0.0;
            for (int h = 0; h < H; ++h) {
                const double xv = x_at(q, t, h);
                g += xv * w_at(q->w1, q->w1_scale, q->dtype, 2 * I, H, e, i, h);
                u += xv * w_at(q->w1, q->w1_scale, q->dtype, 2 * I, H, e, I + i, h);
            }
            act[(size_t)r * I + i] = g / (1.0 + exp(-g)) * u;
        }
}

/* Down projection for n rows: y[r,h] = sum_i act[r,i] * W2[e_r,h,i]. */
void oracle_down_rows(const oracle_problem *q, int32_t n, const int32_t *expert,
                      const double *act /* [n,I] */, double *y /* [n,H] */)
{
    const int H = q->H, I = q->I;
#pragma omp parallel for collapse(2) schedule(static)
    for (int r = 0; r < n; ++r)
        for (int h = 0; h < H; ++h) {
            const int e = expert[r];
            double acc = 0.0;
            for (int i = 0; i < I; ++i)
                acc += act[(size_t)r * I + i] * w_at(q->w2, q->w2_scale, q->dtype, H, I, e, h, i);
            y[(size_t)r * H + h] = acc;
        }
}

/* Weighted sum over each token's k expert rows, in slot order j = 0..k-1:
 *   out[t,h] = sum_j w[t,j] * y[inv[t*k+j], h].
 * A pair without a row (inv < 0: its expert is not held here) contributes nothing. */
void oracle_combine(int32_t T, int32_t k, int32_t H, const double *w /* [T,k] */,
                    const int32_t *inv /* [T*k] */, const double *y /* [T*k,H] */, double *out /* [T,H] */)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j) {
                const int32_t row = inv[(size_t)t * k + j];
                if (row >= 0) acc += w[(size_t)t * k + j] * y[(size_t)row * H + h];
            }
            out[(size_t)t * H + h] = acc;
        }
}

/*
 * The whole layer for a list of tokens, straight from the definition (no
 * reordering by expert is needed to define the result):
 *   out[t,:] = sum_j w[t,j] * Down_{e_j}( SiLU(Gate_{e_j} x_t) * Up_{e_j} x_t )
 * In local-expert mode the sum runs over the chosen experts that are local (the routing
 * itself, and the weights w, are those of the full layer).
 * Also returns the routing it used (ids, w, margin) for those tokens.
 */
void oracle_forward_tokens(const oracle_problem *q, int32_t n, const int32_t *tokens,
                           double *out /* [n,H] */, int32_t *ids /* [n,k] */, double *w /* [n,k] */,
                           double *margin /* [n] */)
{
    const int H = q->H, I = q->I, k = q->top_k;
    double *z = (double *)malloc(sizeof(double) * q->E);
    double *act = (double *)malloc(sizeof(double) * I);
    double *y = (double *)malloc(sizeof(double) * H);
    int32_t tok1, exp1;
    for (int r = 0; r < n; ++r) {
        const int t = tokens[r];
        logits_token(q, t, z);
        route_token(q, z, ids + (size_t)r * k, w + (size_t)r * k, margin + r);
        for (int h = 0; h < H; ++h) out[(size_t)r * H + h] = 0.0;
        for (int j = 0; j < k; ++j) {
            tok1 = t;
            exp1 = ids[(size_t)r * k + j];
            if (q->local_count > 0) {
                if (exp1 < q->local_offset || exp1 >= q->local_offset + q->local_count) continue;
                exp1 -= q->local_offset;               /* index into the local weight arrays */
            }
            oracle_swiglu_rows(q, 1, &tok1, &exp1, act);
            oracle_down_rows(q, 1, &exp1, act, y);
            for (int h = 0; h < H; ++h) out[(size_t)r * H + h] += w[(size_t)r * k + j] * y[h];
        }
    }
    free(z); free(act); free(y);
}

/* Threads the OpenMP loops above will use (for reporting beside timings). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
