/* Driver for a sanitizer run of the CPU oracle (gcc -fsanitize=address,undefined): every entry
 * point of oracle/bigmac_oracle.c once on small ragged shapes, all buffers heap blocks of
 * exactly the documented size so that an access one element past any of them is reported.
 * Built and run by tests/test_oracle_sanitizers.py; prints "ok" and exits 0. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_router_logits(int, int, int, const float *, const float *, const float *, float *);
void oracle_topk_gate(int, int, int, const float *, int32_t *, double *);
void oracle_permutation(int, int, int, int, const int32_t *, int32_t *, int32_t *, int32_t *, int32_t *);
void oracle_dispatch(int, int, int, const float *, const int32_t *, float *);
void oracle_expert_rows_ext(int, int, int, const int32_t *, const float *, const float *, const float *, const float *,
                            const float *, double *, double *);
void oracle_combine(int, int, int, const double *, const int32_t *, const double *, double *);
void oracle_stored_low(int, int, int, const float *, const float *, int, float *);
void oracle_bigmac_forward_ext(int, int, int, int, int, int, const float *, const float *, const float *, const float *,
                               const float *, const float *, const float *, const float *, const float *, int, int,
                               const int32_t *, const int32_t *, double *, double *);
void oracle_bigmac_backward_ext(int, int, int, int, int, int, const float *, const float *, const float *, const float *,
                                const float *, const float *, const float *, const float *, const float *, const float *, int,
                                int, const int32_t *, const int32_t *, double *, double *, double *, double *, double *,
                                double *, double *, double *);
void oracle_cdac_forward(int, int, int, int, int, const float *, const float *, const float *, const float *, const float *,
                         int, const int32_t *, const int32_t *, double *);
void oracle_cdac_backward(int, int, int, int, int, const float *, const float *, const float *, const float *, const float *,
                          const float *, int, const int32_t *, const int32_t *, double *, double *, double *, double *);

static uint32_t state = 12345u;
static float rnd(void) {   /* uniform in [-1, 1) */
    state = state * 1664525u + 1013904223u;
    return (float)(state >> 8) / 8388608.0f - 1.0f;
}
static float *fbuf(size_t n, float scale) {
    float *p = malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = scale * rnd();
    return p;
}
static double *dbuf(size_t n) { return calloc(n ? n : 1, sizeof(double)); }
static int32_t *ibuf(size_t n) { return calloc(n ? n : 1, sizeof(int32_t)); }

static void run(int T, int d, int r, int N, int k, int h, int route_low, int with_bias, int capacity) {
    const size_t Tk = (size_t)T * k;
    float *x = fbuf((size_t)T * d, 1.0f), *dy = fbuf((size_t)T * d, 1.0f);
    float *wg = fbuf((size_t)(route_low ? r : d) * N, 0.3f), *gb = fbuf(N, 2.0f);   /* a strong bias: some experts get no row */
    float *wdown = fbuf((size_t)d * r, 0.2f), *wup = fbuf((size_t)r * d, 0.2f);
    float *w1 = fbuf((size_t)N * r * h, 0.2f), *w2 = fbuf((size_t)N * h * r, 0.2f);
    float *b1 = with_bias ? fbuf((size_t)N * h, 0.1f) : NULL, *b2 = with_bias ? fbuf((size_t)N * r, 0.1f) : NULL;
    /* the steps one by one */
    float *xlow = fbuf((size_t)T * r, 0.0f), *logits = fbuf((size_t)T * N, 0.0f);
    oracle_stored_low(T, d, r, x, wdown, route_low, xlow);
    oracle_router_logits(T, route_low ? r : d, N, route_low ? xlow : x, wg, gb, logits);
    int32_t *idx = ibuf(Tk), *offsets = ibuf(N + 1), *slot = ibuf(Tk), *src = ibuf(Tk), *keep = ibuf(Tk);
    double *gate = dbuf(Tk);
    oracle_topk_gate(T, N, k, logits, idx, gate);
    oracle_permutation(T, k, N, capacity, idx, offsets, slot, src, keep);
    const size_t rows = (size_t)offsets[N];
    float *xperm = fbuf(rows * r, 0.0f);
    oracle_dispatch(T, k, r, xlow, slot, xperm);
    double *a = dbuf(rows * h), *o = dbuf(rows * r), *ylow = dbuf((size_t)T * r);
    oracle_expert_rows_ext(N, r, h, offsets, xperm, w1, w2, b1, b2, a, o);
    oracle_combine(T, k, r, o, slot, gate, ylow);
    /* the layer, all tokens and a selection */
    double *y = dbuf((size_t)T * d), *yl = dbuf((size_t)T * r);
    oracle_bigmac_forward_ext(T, d, r, N, k, h, x, wg, gb, wdown, wup, w1, w2, b1, b2, route_low, T, NULL, capacity ? keep : NULL, y, yl);
    const int nsel = T > 3 ? 3 : T;
    int32_t *sel = ibuf(nsel);
    for (int s = 0; s < nsel; ++s) sel[s] = (T - 1) - s * (T / 3 > 0 ? T / 3 : 1) < 0 ? 0 : (T - 1) - s * (T / 3 > 0 ? T / 3 : 1);
    double *ys = dbuf((size_t)nsel * d);
    oracle_bigmac_forward_ext(T, d, r, N, k, h, x, wg, gb, wdown, wup, w1, w2, b1, b2, route_low, nsel, sel, capacity ? keep : NULL, ys, NULL);
    double *dx = dbuf((size_t)T * d), *dwd = dbuf((size_t)d * r), *dwu = dbuf((size_t)r * d), *dwg = dbuf((size_t)(route_low ? r : d) * N);
    double *dw1 = dbuf((size_t)N * r * h), *dw2 = dbuf((size_t)N * h * r);
    double *db1 = with_bias ? dbuf((size_t)N * h) : NULL, *db2 = with_bias ? dbuf((size_t)N * r) : NULL;
    oracle_bigmac_backward_ext(T, d, r, N, k, h, x, dy, wg, gb, wdown, wup, w1, w2, b1, b2, route_low, T, NULL, capacity ? keep : NULL,
                               dx, dwd, dwu, dwg, dw1, dw2, db1, db2);
    oracle_bigmac_backward_ext(T, d, r, N, k, h, x, dy, wg, gb, wdown, wup, w1, w2, b1, b2, route_low, nsel, sel, capacity ? keep : NULL,
                               dx, dwd, dwu, dwg, dw1, dw2, db1, db2);
    /* the fine-grained layer from the same parameters (router on the full-width token only) */
    if (!route_low) {
        float *wdn = fbuf((size_t)N * d * r, 0.2f), *wupe = fbuf((size_t)N * r * d, 0.2f), *wgd = fbuf((size_t)d * N, 0.3f);
        double *yc = dbuf((size_t)T * d), *dxc = dbuf((size_t)T * d), *dwgc = dbuf((size_t)d * N);
        double *dwdn = dbuf((size_t)N * d * r), *dwupe = dbuf((size_t)N * r * d);
        oracle_cdac_forward(T, d, r, N, k, x, wgd, gb, wdn, wupe, T, NULL, NULL, yc);
        oracle_cdac_backward(T, d, r, N, k, x, dy, wgd, gb, wdn, wupe, T, NULL, NULL, dxc, dwgc, dwdn, dwupe);
        free(wdn); free(wupe); free(wgd); free(yc); free(dxc); free(dwgc); free(dwdn); free(dwupe);
    }
    double check = 0.0;
    for (size_t i = 0; i < (size_t)T * d; ++i) check += y[i] + dx[i];
    if (check != check) { printf("not a number in the results\n"); exit(1); }
    free(x); free(dy); free(wg); free(gb); free(wdown); free(wup); free(w1); free(w2); free(b1); free(b2);
    free(xlow); free(logits); free(idx); free(offsets); free(slot); free(src); free(keep); free(gate);
    free(xperm); free(a); free(o); free(ylow); free(y); free(yl); free(sel); free(ys);
    free(dx); free(dwd); free(dwu); free(dwg); free(dw1); free(dw2); free(db1); free(db2);
}

int main(void) {
    run(37, 24, 8, 5, 3, 12, 0, 0, 0);
    run(37, 24, 8, 5, 3, 12, 0, 1, 9);     /* biases, a capacity that drops pairs */
    run(16, 12, 4, 7, 7, 5, 1, 1, 0);      /* k = N, router on x' */
    run(1, 8, 8, 3, 1, 4, 0, 0, 0);        /* one token */
    run(50, 16, 8, 9, 2, 3, 1, 0, 4);
    printf("ok\n");
    return 0;
}
