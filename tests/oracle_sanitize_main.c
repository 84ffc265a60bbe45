/*
 * TEST INFRASTRUCTURE: drives every entry point of the CPU oracle once on small problems, so that
 * a build with -fsanitize=address,undefined can watch its loops (index arithmetic, scale-block
 * indexing, the local-expert branch, the fp8 paths).  Built and run by tests/test_oracle_sanitize.py;
 * prints one checksum line per problem.  The values are not compared here (the pins do that).
 */
#include "../oracle/moe_oracle.c"

#include <stdio.h>

static uint32_t lcg_state = 12345u;
static double lcg_unit(void)                       /* uniform in (-1, 1) */
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return ((double)(lcg_state >> 8) / (double)(1u << 24)) * 2.0 - 1.0;
}

static uint16_t to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static void fill_bf16(uint16_t *p, size_t n, double amp) { for (size_t i = 0; i < n; ++i) p[i] = to_bf16((float)(lcg_unit() * amp)); }
static void fill_f32(float *p, size_t n, double lo, double hi) { for (size_t i = 0; i < n; ++i) p[i] = (float)(lo + (hi - lo) * 0.5 * (lcg_unit() + 1.0)); }
static void fill_e4m3(uint8_t *p, size_t n) { for (size_t i = 0; i < n; ++i) p[i] = oracle_f32_to_e4m3((float)(lcg_unit() * 300.0)); }

static double run(int fp8, int grouped, int local_offset, int local_count, int quantize_x)
{
    oracle_problem q;
    memset(&q, 0, sizeof q);
    q.T = 7; q.H = 256; q.I = 128; q.E = 16; q.top_k = 3;
    q.scoring = grouped ? ORACLE_SIGMOID : ORACLE_SOFTMAX;
    q.renormalize = 1;
    q.n_group = grouped ? 4 : 1; q.topk_group = grouped ? 2 : 1; q.group_score_topn = 2;
    q.dtype = fp8 ? ORACLE_FP8_E4M3 : ORACLE_BF16;
    q.routed_scale = grouped ? 2.5f : 1.0f;
    q.local_offset = local_offset; q.local_count = local_count;
    const int EL = local_count > 0 ? local_count : q.E;
    const size_t es = fp8 ? 1 : 2;
    const size_t nx = (size_t)q.T * q.H, n1 = (size_t)EL * 2 * q.I * q.H, n2 = (size_t)EL * q.H * q.I;
    void *x = malloc(nx * es), *w1 = malloc(n1 * es), *w2 = malloc(n2 * es);
    uint16_t *xb = (uint16_t *)malloc(nx * 2);
    float *xs = (float *)malloc(sizeof(float) * q.T * (q.H / 128));
    float *w1s = (float *)malloc(sizeof(float) * EL * (2 * q.I / 128) * (q.H / 128));
    float *w2s = (float *)malloc(sizeof(float) * EL * (q.H / 128) * (q.I / 128));
    float *rw = (float *)malloc(sizeof(float) * q.E * q.H), *bias = (float *)malloc(sizeof(float) * q.E);
    fill_f32(rw, (size_t)q.E * q.H, -0.06, 0.06);
    fill_f32(bias, q.E, -0.1, 0.1);
    if (fp8) {
        fill_e4m3((uint8_t *)w1, n1); fill_e4m3((uint8_t *)w2, n2);
        fill_f32(w1s, (size_t)EL * (2 * q.I / 128) * (q.H / 128), 1e-4, 3e-4);
        fill_f32(w2s, (size_t)EL * (q.H / 128) * (q.I / 128), 1e-4, 3e-4);
        if (quantize_x) {
            fill_bf16(xb, nx, 2.0);
            for (int c = 0; c < 128; ++c) xb[c] = 0;                       /* an all-zero block */
            oracle_quantize_rows_1x128(q.T, q.H, xb, (uint8_t *)x, xs);
            q.x_bf16 = xb;
        } else {
            fill_e4m3((uint8_t *)x, nx);
            fill_f32(xs, (size_t)q.T * (q.H / 128), 1e-3, 5e-3);
        }
        q.x_scale = xs; q.w1_scale = w1s; q.w2_scale = w2s;
    } else {
        fill_bf16((uint16_t *)x, nx, 1.0); fill_bf16((uint16_t *)w1, n1, 0.06); fill_bf16((uint16_t *)w2, n2, 0.09);
    }
    q.x = x; q.router_w = rw; q.bias = grouped ? bias : NULL; q.w1 = w1; q.w2 = w2;

    const int P = q.T * q.top_k;
    double *z = (double *)malloc(sizeof(double) * q.T * q.E);
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * P);
    double *w = (double *)malloc(sizeof(double) * P), *margin = (double *)malloc(sizeof(double) * q.T);
    oracle_router_logits(&q, z);
    oracle_route(&q, z, ids, w, margin);

    /* staged path on the pairs whose expert is held here */
    int32_t *kept_ids = (int32_t *)malloc(sizeof(int32_t) * P), *kept_pair = (int32_t *)malloc(sizeof(int32_t) * P);
    int kept = 0;
    for (int p = 0; p < P; ++p) {
        int e = ids[p] - local_offset;
        if (e >= 0 && e < EL) { kept_ids[kept] = e; kept_pair[kept] = p; ++kept; }
    }
    int32_t *off = (int32_t *)malloc(sizeof(int32_t) * (EL + 1));
    int32_t *sp = (int32_t *)malloc(sizeof(int32_t) * (kept + 1)), *inv_k = (int32_t *)malloc(sizeof(int32_t) * (kept + 1));
    oracle_permute(kept, EL, kept_ids, off, sp, inv_k);
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (kept + 1)), *ex = (int32_t *)malloc(sizeof(int32_t) * (kept + 1));
    int32_t *inv = (int32_t *)malloc(sizeof(int32_t) * P);
    for (int p = 0; p < P; ++p) inv[p] = -1;
    for (int r = 0; r < kept; ++r) { tok[r] = kept_pair[sp[r]] / q.top_k; ex[r] = kept_ids[sp[r]]; inv[kept_pair[sp[r]]] = r; }
    double *act = (double *)malloc(sizeof(double) * (size_t)(kept + 1) * q.I);
    double *y = (double *)calloc((size_t)P * q.H, sizeof(double));
    oracle_swiglu_rows(&q, kept, tok, ex, act);
    oracle_down_rows(&q, kept, ex, act, y);
    double *out = (double *)malloc(sizeof(double) * (size_t)q.T * q.H);
    oracle_combine(q.T, q.top_k, q.H, w, inv, y, out);

    /* the one-call definition on every token must agree with the staged path */
    int32_t *tokens = (int32_t *)malloc(sizeof(int32_t) * q.T);
    for (int t = 0; t < q.T; ++t) tokens[t] = t;
    double *out2 = (double *)malloc(sizeof(double) * (size_t)q.T * q.H);
    int32_t *ids2 = (int32_t *)malloc(sizeof(int32_t) * P);
    double *w2o = (double *)malloc(sizeof(double) * P), *m2 = (double *)malloc(sizeof(double) * q.T);
    oracle_forward_tokens(&q, q.T, tokens, out2, ids2, w2o, m2);
    double sum = 0.0, diff = 0.0;
    for (size_t i = 0; i < (size_t)q.T * q.H; ++i) { sum += fabs(out2[i]); diff += fabs(out2[i] - out[i]); }
    if (!(diff <= 1e-9 * (sum + 1.0))) { fprintf(stderr, "staged and one-call paths disagree: %g vs %g\n", diff, sum); exit(3); }

    free(x); free(w1); free(w2); free(xb); free(xs); free(w1s); free(w2s); free(rw); free(bias); free(z); free(ids);
    free(w); free(margin); free(kept_ids); free(kept_pair); free(off); free(sp); free(inv_k); free(tok); free(ex);
    free(inv); free(act); free(y); free(out); free(tokens); free(out2); free(ids2); free(w2o); free(m2);
    return sum;
}

int main(void)
{
    for (int c = 0; c < 256; ++c) (void)oracle_e4m3_to_f64((uint8_t)c);
    for (int c = 0; c < 65536; c += 97) (void)oracle_bf16_to_f64((uint16_t)c);
    printf("bf16 softmax          %.6e\n", run(0, 0, 0, 0, 0));
    printf("bf16 grouped local    %.6e\n", run(0, 1, 4, 8, 0));
    printf("fp8 grouped           %.6e\n", run(1, 1, 0, 0, 0));
    printf("fp8 local quantize_x  %.6e\n", run(1, 0, 8, 8, 1));
    printf("threads %d\nok\n", oracle_num_threads());
    return 0;
}
