/*
 * CPU oracle for the BigMac MoE layer.  TEST INFRASTRUCTURE ONLY: it defines what the layer
 * computes so that tests, the smoke check and the benchmark's cpu_baseline leg can compare the
 * HIP library against it.  It is plain and slow on purpose, shares nothing with the HIP
 * library, and must never be called from the product path.
 *
 * What is computed (all matrices row-major, weights are [in, out] as in the paper's x.W):
 *   BigMac layer, Eq. 2:   x' = x W_down ;  y' = sum_{i in T} p_i(x) E_i(x') ;  y = y' W_up
 *   BigMac expert, Eq. 4:  E_i(x') = act(x' W1[i]) W2[i]       (ascend r->h, then descend h->r)
 *   fine-grained layer (CDAC order, Section 3.1) with the expert of Eq. 3:
 *                          y = sum_{i in T} p_i(x) act(x Wdn[i]) Wup[i]   (descend d->r, ascend r->d)
 *   T = the top_k experts of the token (Section 2), p_i = gate value (Eq. 2's text).
 *
 * Readings where the paper is silent (both sides of every parity test follow them):
 *   - router logits are x . W_g (+ bias) on the full-width token x (Section 3.1 chooses x over x'),
 *     in fp32 with a FIXED summation order (below), because the logits decide integers;
 *   - top-k picks the largest logit k times, equal logits go to the lowest expert index;
 *   - the gate value is the softmax over the k selected logits;
 *   - act is the exact (erf) GELU; there are no biases; routing is dropless (Section 3.3).
 * Two variants the paper names are options of the *_ext entry points (off in the plain ones):
 *   - the router may read x' instead of x (Section 3.1 leaves the choice open): W_g is then [r, N],
 *     the router's input is x' rounded to the type it is stored and dispatched in (fp32 or bf16,
 *     ROUTE_LOW_F32 / ROUTE_LOW_BF16), and the gate's gradient reaches x through x' (the rounding
 *     is passed straight through);
 *   - expert biases (the 2rh term of the expert parameter count in Table 3):
 *     E_i(x') = (act(x' W1[i] + b1[i])) W2[i] + b2[i], b1 [N, hid], b2 [N, win].
 *
 * Precision: inputs arrive as fp32 values (already rounded to the run's storage type by the
 * caller).  The router logits are fp32 in the fixed order.  Everything else is accumulated and
 * returned in fp64.
 *
 * Fixed router order, for one (token t, expert n), d a multiple of 64:
 *   p[l] = fma(x[t, 64q + l], W_g[64q + l, n], p[l])  for q = 0 .. d/64-1, starting from 0,
 *   then for off = 32, 16, 8, 4, 2, 1:  p[l] = p[l] + p[l + off]  for l < off,
 *   logit = p[0] (+ bias[n], added last, only when a bias is given).
 *
 * Parity pins live in tests/test_oracle_*.py (brute force in numpy fp64, closed forms, special
 * cases that reduce to a dense FFN, finite differences, the paper's Table 3/4 arithmetic).
 * Unpinned by the paper (readings above): GELU form, bias-free experts, gate = softmax over the
 * selected logits, the fixed router order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define LANES 64

enum { ROUTE_FULL = 0, ROUTE_LOW_F32 = 1, ROUTE_LOW_BF16 = 2 };

/* round to the nearest bfloat16, ties to even (finite inputs) */
static float round_bf16(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&v, &u, 4);
    return v;
}
/* x' as the router of the x'-variant sees it: the stored value */
static float stored_low(double v, int route_low)
{
    float f = (float)v;
    return route_low == ROUTE_LOW_BF16 ? round_bf16(f) : f;
}

/* number of threads the parallel loops below use */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- routing ---------------- */

/* logits[T,N] in the fixed fp32 order.  bias may be NULL. */
void oracle_router_logits(int T, int d, int N, const float *x, const float *w_gate,
                          const float *bias, float *logits)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int n = 0; n < N; ++n) {
            float p[LANES];
            for (int l = 0; l < LANES; ++l) p[l] = 0.0f;
            for (int q = 0; q < d / LANES; ++q)
                for (int l = 0; l < LANES; ++l) {
                    int i = q * LANES + l;
                    p[l] = fmaf(x[(size_t)t * d + i], w_gate[(size_t)i * N + n], p[l]);
                }
            for (int off = LANES / 2; off >= 1; off >>= 1)
                for (int l = 0; l < off; ++l) p[l] = p[l] + p[l + off];
            float v = p[0];
            if (bias) v = v + bias[n];
            logits[(size_t)t * N + n] = v;
        }
    }
}

/* Top-k set of each token (Section 2: top_k experts per token) in descending-logit pick order,
 * ties to the lowest index; gate[t,j] = softmax over the k picked logits (fp64 from fp32 logits). */
void oracle_topk_gate(int T, int N, int k, const float *logits, int32_t *idx, double *gate)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *row = logits + (size_t)t * N;
        char *taken = (char *)calloc((size_t)N, 1);
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int n = 0; n < N; ++n) {
                if (taken[n]) continue;
                if (best < 0 || row[n] > row[best]) best = n;
            }
            taken[best] = 1;
            idx[(size_t)t * k + j] = best;
        }
        free(taken);
        double m = (double)row[idx[(size_t)t * k]];
        double s = 0.0;
        for (int j = 0; j < k; ++j) {
            double e = exp((double)row[idx[(size_t)t * k + j]] - m);
            gate[(size_t)t * k + j] = e;
            s += e;
        }
        for (int j = 0; j < k; ++j) gate[(size_t)t * k + j] /= s;
    }
}

/* The dispatch permutation: the flat (token, choice) pairs f = t*k + j, stably sorted by expert.
 * src_of[s] = f at sorted position s; slot_of[f] = s; offsets[e] = first slot of expert e,
 * offsets[N] = T*k (dropless, Section 3.3: every pair keeps a slot).
 * capacity > 0 is the fixed expert capacity of the paper's training set-up (Table 5 names a
 * capacity factor; the rule itself is the usual one, not the paper's): an expert keeps the first
 * `capacity` of its pairs in flat order, the others get slot_of = -1 and no slot, and
 * offsets[N] = number of kept pairs.  keep ([T*k], may be NULL) receives 1 / 0 per pair. */
void oracle_permutation(int T, int k, int N, int capacity, const int32_t *idx, int32_t *offsets,
                        int32_t *slot_of, int32_t *src_of, int32_t *keep)
{
    int64_t Tk = (int64_t)T * k;
    int32_t s = 0;
    for (int e = 0; e < N; ++e) {          /* a stable sort by expert, written as N passes */
        int32_t held = 0;
        offsets[e] = s;
        for (int64_t f = 0; f < Tk; ++f) {
            if (idx[f] != e) continue;
            if (capacity > 0 && held >= capacity) {
                slot_of[f] = -1;
                if (keep) keep[f] = 0;
                continue;
            }
            src_of[s] = (int32_t)f; slot_of[f] = s; ++s; ++held;
            if (keep) keep[f] = 1;
        }
    }
    offsets[N] = s;
}

/* ---------------------------------------------------------------- pieces ----------------- */

static double gelu(double a) { return 0.5 * a * (1.0 + erf(a * M_SQRT1_2)); }
static double gelu_grad(double a)
{
    return 0.5 * (1.0 + erf(a * M_SQRT1_2)) + a * exp(-0.5 * a * a) * 0.3989422804014326779; /* 1/sqrt(2 pi) */
}

/* out[n] = sum_i v[i] * W[i, n]   (W is [K, Nout] row-major, fp32 storage) */
static void vec_mat(const double *v, const float *W, int K, int Nout, double *out)
{
    for (int n = 0; n < Nout; ++n) out[n] = 0.0;
    for (int i = 0; i < K; ++i) {
        double vi = v[i];
        const float *w = W + (size_t)i * Nout;
        for (int n = 0; n < Nout; ++n) out[n] += vi * (double)w[n];
    }
}
/* out[i] = sum_n v[n] * W[i, n]   (v times W transposed) */
static void vec_matT(const double *v, const float *W, int K, int Nout, double *out)
{
    for (int i = 0; i < K; ++i) {
        const float *w = W + (size_t)i * Nout;
        double s = 0.0;
        for (int n = 0; n < Nout; ++n) s += v[n] * (double)w[n];
        out[i] = s;
    }
}
/* G[i, n] += u[i] * v[n] */
static void outer_acc(double *G, const double *u, const double *v, int K, int Nout)
{
    for (int i = 0; i < K; ++i) {
        double ui = u[i];
        double *g = G + (size_t)i * Nout;
        for (int n = 0; n < Nout; ++n) g[n] += ui * v[n];
    }
}

/* First All-to-All of the layer (Section 3.1), on one device: row f = t*k+j of the token
 * stream goes to slot slot_of[f].  Pure copy. */
void oracle_dispatch(int T, int k, int width, const float *x_low, const int32_t *slot_of,
                     float *x_perm)
{
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            if (slot_of[(size_t)t * k + j] < 0) continue;                 /* dropped pair: no row */
            memcpy(x_perm + (size_t)slot_of[(size_t)t * k + j] * width,
                   x_low + (size_t)t * width, sizeof(float) * (size_t)width);
        }
}

/* The expert of Eq. 4 (or Eq. 3 with the widths swapped) applied to permuted rows: rows
 * [offsets[e], offsets[e+1]) belong to expert e.  a_out (pre-activation) may be NULL. */
void oracle_expert_rows_ext(int N, int win, int hid, const int32_t *offsets, const float *x_perm,
                            const float *w1, const float *w2, const float *b1, const float *b2,
                            double *a_out, double *o_perm);
void oracle_expert_rows(int N, int win, int hid, const int32_t *offsets, const float *x_perm,
                        const float *w1, const float *w2, double *a_out, double *o_perm)
{
    oracle_expert_rows_ext(N, win, hid, offsets, x_perm, w1, w2, NULL, NULL, a_out, o_perm);
}
/* The same with expert biases b1 [N, hid], b2 [N, win] (either may be NULL); a_out then holds
 * the pre-activation with b1 added. */
void oracle_expert_rows_ext(int N, int win, int hid, const int32_t *offsets, const float *x_perm,
                            const float *w1, const float *w2, const float *b1, const float *b2,
                            double *a_out, double *o_perm)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int e = 0; e < N; ++e) {
        double *xin = (double *)malloc(sizeof(double) * (size_t)win);
        double *a = (double *)malloc(sizeof(double) * (size_t)hid);
        const float *W1 = w1 + (size_t)e * win * hid, *W2 = w2 + (size_t)e * hid * win;
        for (int s = offsets[e]; s < offsets[e + 1]; ++s) {
            for (int i = 0; i < win; ++i) xin[i] = (double)x_perm[(size_t)s * win + i];
            vec_mat(xin, W1, win, hid, a);
            if (b1) for (int c = 0; c < hid; ++c) a[c] += (double)b1[(size_t)e * hid + c];
            if (a_out) memcpy(a_out + (size_t)s * hid, a, sizeof(double) * (size_t)hid);
            for (int c = 0; c < hid; ++c) a[c] = gelu(a[c]);
            vec_mat(a, W2, hid, win, o_perm + (size_t)s * win);
            if (b2) for (int c = 0; c < win; ++c) o_perm[(size_t)s * win + c] += (double)b2[(size_t)e * win + c];
        }
        free(xin); free(a);
    }
}

/* Second All-to-All plus the weighted sum of Eq. 2: y_low[t] = sum_j gate[t,j] * o_perm[slot_of[t,j]],
 * added in j order.  gate == NULL means unit weights. */
void oracle_combine(int T, int k, int width, const double *o_perm, const int32_t *slot_of,
                    const double *gate, double *y_low)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double *y = y_low + (size_t)t * width;
        for (int c = 0; c < width; ++c) y[c] = 0.0;
        for (int j = 0; j < k; ++j) {
            double g = gate ? gate[(size_t)t * k + j] : 1.0;
            if (slot_of[(size_t)t * k + j] < 0) continue;                 /* dropped pair */
            const double *o = o_perm + (size_t)slot_of[(size_t)t * k + j] * width;
            for (int c = 0; c < width; ++c) y[c] += g * o[c];
        }
    }
}

/* x' = x W_down (Eq. 2's first step) as it is stored: the fp64 sum rounded to fp32, and on to bf16
 * for ROUTE_LOW_BF16.  This is what the router of the x'-variant reads. */
void oracle_stored_low(int T, int d, int r, const float *x, const float *w_down, int route_low, float *x_low)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double *xd = (double *)malloc(sizeof(double) * (size_t)d);
        double *xl = (double *)malloc(sizeof(double) * (size_t)r);
        for (int i = 0; i < d; ++i) xd[i] = (double)x[(size_t)t * d + i];
        vec_mat(xd, w_down, d, r, xl);
        for (int c = 0; c < r; ++c) x_low[(size_t)t * r + c] = stored_low(xl[c], route_low);
        free(xd); free(xl);
    }
}

/* ---------------------------------------------------------------- layers ----------------- */

/* BigMac layer forward, Eq. 2 with the expert of Eq. 4, token by token, no permutation.
 * sel == NULL: all T tokens (nsel = T); otherwise only tokens sel[0..nsel) are evaluated and
 * row s of y (and y_low) is token sel[s].  y is [nsel, d]; y_low ([nsel, r]) may be NULL.
 * keep ([T, k], NULL = every pair) marks the pairs that survived the expert capacity (from
 * oracle_permutation); a dropped pair adds nothing, and the gate values stay as they are. */
void oracle_bigmac_forward_ext(int T, int d, int r, int N, int k, int h,
                               const float *x, const float *w_gate, const float *bias,
                               const float *w_down, const float *w_up, const float *w1, const float *w2,
                               const float *b1, const float *b2, int route_low,
                               int nsel, const int32_t *sel, const int32_t *keep, double *y, double *y_low);
void oracle_bigmac_forward(int T, int d, int r, int N, int k, int h,
                           const float *x, const float *w_gate, const float *bias,
                           const float *w_down, const float *w_up, const float *w1, const float *w2,
                           int nsel, const int32_t *sel, const int32_t *keep, double *y, double *y_low)
{
    oracle_bigmac_forward_ext(T, d, r, N, k, h, x, w_gate, bias, w_down, w_up, w1, w2, NULL, NULL, ROUTE_FULL,
                              nsel, sel, keep, y, y_low);
}

/* The same with the two variants: route_low != ROUTE_FULL: the router reads the stored x' and
 * w_gate is [r, N] (Section 3.1); b1 [N, h], b2 [N, r] (either may be NULL): expert biases
 * (Table 3's 2rh parameters per expert). */
void oracle_bigmac_forward_ext(int T, int d, int r, int N, int k, int h,
                               const float *x, const float *w_gate, const float *bias,
                               const float *w_down, const float *w_up, const float *w1, const float *w2,
                               const float *b1, const float *b2, int route_low,
                               int nsel, const int32_t *sel, const int32_t *keep, double *y, double *y_low)
{
    (void)T;
#pragma omp parallel for schedule(dynamic, 4)
    for (int s = 0; s < nsel; ++s) {
        int t = sel ? sel[s] : s;
        const float *xt = x + (size_t)t * d;
        float *logit = (float *)malloc(sizeof(float) * (size_t)N);
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
        double *gate = (double *)malloc(sizeof(double) * (size_t)k);
        double *xd = (double *)malloc(sizeof(double) * (size_t)d);
        double *xl = (double *)malloc(sizeof(double) * (size_t)r);
        double *a = (double *)malloc(sizeof(double) * (size_t)h);
        double *o = (double *)malloc(sizeof(double) * (size_t)r);
        double *yl = (double *)malloc(sizeof(double) * (size_t)r);
        for (int i = 0; i < d; ++i) xd[i] = (double)xt[i];
        vec_mat(xd, w_down, d, r, xl);                                  /* x' = x W_down       */
        if (route_low == ROUTE_FULL) {
            oracle_router_logits(1, d, N, xt, w_gate, bias, logit);
        } else {                                                        /* the router reads x' */
            float *xr = (float *)malloc(sizeof(float) * (size_t)r);
            for (int c = 0; c < r; ++c) xr[c] = stored_low(xl[c], route_low);
            oracle_router_logits(1, r, N, xr, w_gate, bias, logit);
            free(xr);
        }
        oracle_topk_gate(1, N, k, logit, idx, gate);
        for (int c = 0; c < r; ++c) yl[c] = 0.0;
        for (int j = 0; j < k; ++j) {
            int e = idx[j];
            if (keep && !keep[(size_t)t * k + j]) continue;
            vec_mat(xl, w1 + (size_t)e * r * h, r, h, a);               /* x' W1[e]            */
            if (b1) for (int c = 0; c < h; ++c) a[c] += (double)b1[(size_t)e * h + c];
            for (int c = 0; c < h; ++c) a[c] = gelu(a[c]);
            vec_mat(a, w2 + (size_t)e * h * r, h, r, o);                /* E_e(x')             */
            if (b2) for (int c = 0; c < r; ++c) o[c] += (double)b2[(size_t)e * r + c];
            for (int c = 0; c < r; ++c) yl[c] += gate[j] * o[c];        /* y' += p_e E_e(x')   */
        }
        vec_mat(yl, w_up, r, d, y + (size_t)s * d);                     /* y = y' W_up         */
        if (y_low) memcpy(y_low + (size_t)s * r, yl, sizeof(double) * (size_t)r);
        free(logit); free(idx); free(gate); free(xd); free(xl); free(a); free(o); free(yl);
    }
}

/* Fine-grained layer forward (CDAC order, expert of Eq. 3): wdn is [N, d, r], wup is [N, r, d]. */
void oracle_cdac_forward(int T, int d, int r, int N, int k,
                         const float *x, const float *w_gate, const float *bias,
                         const float *wdn, const float *wup,
                         int nsel, const int32_t *sel, const int32_t *keep, double *y)
{
    (void)T;
#pragma omp parallel for schedule(dynamic, 4)
    for (int s = 0; s < nsel; ++s) {
        int t = sel ? sel[s] : s;
        const float *xt = x + (size_t)t * d;
        float *logit = (float *)malloc(sizeof(float) * (size_t)N);
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
        double *gate = (double *)malloc(sizeof(double) * (size_t)k);
        double *xd = (double *)malloc(sizeof(double) * (size_t)d);
        double *a = (double *)malloc(sizeof(double) * (size_t)r);
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
        double *yt = y + (size_t)s * d;
        oracle_router_logits(1, d, N, xt, w_gate, bias, logit);
        oracle_topk_gate(1, N, k, logit, idx, gate);
        for (int i = 0; i < d; ++i) xd[i] = (double)xt[i];
        for (int c = 0; c < d; ++c) yt[c] = 0.0;
        for (int j = 0; j < k; ++j) {
            int e = idx[j];
            if (keep && !keep[(size_t)t * k + j]) continue;
            vec_mat(xd, wdn + (size_t)e * d * r, d, r, a);
            for (int c = 0; c < r; ++c) a[c] = gelu(a[c]);
            vec_mat(a, wup + (size_t)e * r * d, r, d, o);
            for (int c = 0; c < d; ++c) yt[c] += gate[j] * o[c];
        }
        free(logit); free(idx); free(gate); free(xd); free(a); free(o);
    }
}

/* Backward of the layer, derived from Eq. 2 / Eq. 4 by the chain rule with the top-k set held
 * fixed (the paper only counts the backward pass, Table 3).  Shared implementation for both
 * orders: with shared == 0 there are no W_down / W_up (fine-grained layer; then win = d and the
 * expert maps win -> hid -> win with hid = r); with shared == 1, win = r, hid = h.
 *
 * Only tokens sel[0..nsel) contribute (sel == NULL: all) - the same as a dy that is zero on the
 * other tokens.  dx is [T, d] and only the selected rows are written.  Every weight-gradient
 * buffer is ADDED to (the caller pre-fills it with zeros or with a running sum); any of them
 * may be NULL.  Gradients:
 *   dy' = dy W_up^T ;  dW_up += y'^T dy
 *   dgate_j = <dy', o_j> ;  do_j = gate_j dy'
 *   dW2[e] += g_j^T do_j ;  dg_j = do_j W2[e]^T ;  da_j = dg_j * act'(a_j)
 *   dW1[e] += x'^T da_j ;  dx' = sum_j da_j W1[e]^T (j order)
 *   dlogit_j = gate_j (dgate_j - sum_m gate_m dgate_m)   (softmax over the selected logits)
 *   dW_g[:, e_j] += x^T dlogit_j ;  dx = dx' W_down^T + sum_j dlogit_j W_g[:, e_j]^T
 *   dW_down += x^T dx'
 * keep ([T, k], NULL = every pair): pairs dropped by the expert capacity have no output, so
 * o_j = 0, dgate_j = 0 and they reach no expert; the gate values are those of the full top-k.
 * Variants: with expert biases, a_j = x' W1[e] + b1[e], o_j = g_j W2[e] + b2[e], and
 *   d_b1[e] += da_j ;  d_b2[e] += do_j.
 * With the router on x' (shared layers only; W_g is [win, N], xr = the stored x'):
 *   dW_g[:, e_j] += xr^T dlogit_j ;  dx' += sum_j dlogit_j W_g[:, e_j]^T ;  dx = dx' W_down^T.
 */
static void layer_backward(int shared, int T, int d, int win, int hid, int N, int k,
                           const float *x, const float *dy,
                           const float *w_gate, const float *bias,
                           const float *w_down, const float *w_up, const float *w1, const float *w2,
                           const float *b1, const float *b2, int route_low,
                           int nsel, const int32_t *sel, const int32_t *keep,
                           double *dx, double *d_w_down, double *d_w_up, double *d_w_gate,
                           double *d_w1, double *d_w2, double *d_b1, double *d_b2)
{
    (void)T;
    size_t ns = (size_t)nsel;
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * ns * k);
    double *gate = (double *)malloc(sizeof(double) * ns * k);
    double *xlow = (double *)malloc(sizeof(double) * ns * win);     /* x' (or x)                 */
    double *dyl = (double *)malloc(sizeof(double) * ns * win);      /* dy' (or dy)               */
    double *opair = (double *)calloc(ns * k * win, sizeof(double)); /* o_j (0 for a dropped pair) */
    double *dxp = (double *)calloc(ns * k * win, sizeof(double));   /* da_j W1^T (0 if dropped)  */
    double *dgt = (double *)calloc(ns * k, sizeof(double));         /* dgate_j (0 if dropped)    */
    double *ylow = (double *)malloc(sizeof(double) * ns * win);     /* y'                        */
    double *dxl = (double *)malloc(sizeof(double) * ns * win);      /* dx'                       */
    double *dlg = (double *)malloc(sizeof(double) * ns * k);        /* dlogit_j                  */
    float *xrt = route_low != ROUTE_FULL ? (float *)malloc(sizeof(float) * ns * win) : NULL; /* stored x' */

    /* phase 1, per token: routing, x', dy' */
#pragma omp parallel for schedule(static)
    for (int s = 0; s < nsel; ++s) {
        int t = sel ? sel[s] : s;
        const float *xt = x + (size_t)t * d, *dyt = dy + (size_t)t * d;
        float *logit = (float *)malloc(sizeof(float) * (size_t)N);
        double *tmp = (double *)malloc(sizeof(double) * (size_t)d);
        if (shared) {
            for (int i = 0; i < d; ++i) tmp[i] = (double)xt[i];
            vec_mat(tmp, w_down, d, win, xlow + (size_t)s * win);
            for (int i = 0; i < d; ++i) tmp[i] = (double)dyt[i];
            vec_matT(tmp, w_up, win, d, dyl + (size_t)s * win);
        } else {
            for (int i = 0; i < d; ++i) xlow[(size_t)s * win + i] = (double)xt[i];
            for (int i = 0; i < d; ++i) dyl[(size_t)s * win + i] = (double)dyt[i];
        }
        if (route_low == ROUTE_FULL) {
            oracle_router_logits(1, d, N, xt, w_gate, bias, logit);
        } else {
            for (int c = 0; c < win; ++c) xrt[(size_t)s * win + c] = stored_low(xlow[(size_t)s * win + c], route_low);
            oracle_router_logits(1, win, N, xrt + (size_t)s * win, w_gate, bias, logit);
        }
        oracle_topk_gate(1, N, k, logit, idx + (size_t)s * k, gate + (size_t)s * k);
        free(logit); free(tmp);
    }

    /* phase 2, per expert (its weight gradients are private to the loop iteration), tokens in order */
#pragma omp parallel for schedule(dynamic, 1)
    for (int e = 0; e < N; ++e) {
        const float *W1 = w1 + (size_t)e * win * hid, *W2 = w2 + (size_t)e * hid * win;
        double *a = (double *)malloc(sizeof(double) * (size_t)hid);
        double *g = (double *)malloc(sizeof(double) * (size_t)hid);
        double *dg = (double *)malloc(sizeof(double) * (size_t)hid);
        double *dout = (double *)malloc(sizeof(double) * (size_t)win);
        for (int s = 0; s < nsel; ++s)
            for (int j = 0; j < k; ++j) {
                if (idx[(size_t)s * k + j] != e) continue;
                if (keep && !keep[(size_t)(sel ? sel[s] : s) * k + j]) continue;   /* dropped by the capacity */
                size_t p = (size_t)s * k + j;
                const double *xl = xlow + (size_t)s * win, *dl = dyl + (size_t)s * win;
                double *o = opair + p * win;
                vec_mat(xl, W1, win, hid, a);
                if (b1) for (int c = 0; c < hid; ++c) a[c] += (double)b1[(size_t)e * hid + c];
                for (int c = 0; c < hid; ++c) g[c] = gelu(a[c]);
                vec_mat(g, W2, hid, win, o);
                if (b2) for (int c = 0; c < win; ++c) o[c] += (double)b2[(size_t)e * win + c];
                double dot = 0.0;
                for (int c = 0; c < win; ++c) dot += dl[c] * o[c];
                dgt[p] = dot;
                for (int c = 0; c < win; ++c) dout[c] = gate[p] * dl[c];
                if (d_w2) outer_acc(d_w2 + (size_t)e * hid * win, g, dout, hid, win);
                if (d_b2) for (int c = 0; c < win; ++c) d_b2[(size_t)e * win + c] += dout[c];
                vec_matT(dout, W2, hid, win, dg);
                for (int c = 0; c < hid; ++c) dg[c] *= gelu_grad(a[c]);         /* now da */
                if (d_w1) outer_acc(d_w1 + (size_t)e * win * hid, xl, dg, win, hid);
                if (d_b1) for (int c = 0; c < hid; ++c) d_b1[(size_t)e * hid + c] += dg[c];
                vec_matT(dg, W1, win, hid, dxp + p * win);
            }
        free(a); free(g); free(dg); free(dout);
    }

    /* phase 3, per token: y', dx', gate backward, dx */
#pragma omp parallel for schedule(static)
    for (int s = 0; s < nsel; ++s) {
        int t = sel ? sel[s] : s;
        double *yl = ylow + (size_t)s * win, *dl = dxl + (size_t)s * win;
        for (int c = 0; c < win; ++c) { yl[c] = 0.0; dl[c] = 0.0; }
        double mix = 0.0;
        for (int j = 0; j < k; ++j) {
            size_t p = (size_t)s * k + j;
            for (int c = 0; c < win; ++c) yl[c] += gate[p] * opair[p * win + c];
            for (int c = 0; c < win; ++c) dl[c] += dxp[p * win + c];
            mix += gate[p] * dgt[p];
        }
        for (int j = 0; j < k; ++j) {
            size_t p = (size_t)s * k + j;
            dlg[p] = gate[p] * (dgt[p] - mix);
        }
        double *dxt = dx + (size_t)t * d;
        if (route_low != ROUTE_FULL)                      /* the gate's gradient enters at x' */
            for (int j = 0; j < k; ++j) {
                size_t p = (size_t)s * k + j;
                int e = idx[p];
                for (int c = 0; c < win; ++c) dl[c] += dlg[p] * (double)w_gate[(size_t)c * N + e];
            }
        if (shared) vec_matT(dl, w_down, d, win, dxt);
        else for (int i = 0; i < d; ++i) dxt[i] = dl[i];
        if (route_low == ROUTE_FULL)
            for (int j = 0; j < k; ++j) {
                size_t p = (size_t)s * k + j;
                int e = idx[p];
                for (int i = 0; i < d; ++i) dxt[i] += dlg[p] * (double)w_gate[(size_t)i * N + e];
            }
    }

    /* phase 4, per output row of the shared matrices */
    if (shared && d_w_up) {
#pragma omp parallel for schedule(static)
        for (int i = 0; i < win; ++i)
            for (int s = 0; s < nsel; ++s) {
                int t = sel ? sel[s] : s;
                double v = ylow[(size_t)s * win + i];
                for (int c = 0; c < d; ++c) d_w_up[(size_t)i * d + c] += v * (double)dy[(size_t)t * d + c];
            }
    }
    if (shared && d_w_down) {
#pragma omp parallel for schedule(static)
        for (int i = 0; i < d; ++i)
            for (int s = 0; s < nsel; ++s) {
                int t = sel ? sel[s] : s;
                double v = (double)x[(size_t)t * d + i];
                for (int c = 0; c < win; ++c) d_w_down[(size_t)i * win + c] += v * dxl[(size_t)s * win + c];
            }
    }
    if (d_w_gate) {
        const int din = route_low != ROUTE_FULL ? win : d;     /* width of the router's input */
#pragma omp parallel for schedule(static)
        for (int i = 0; i < din; ++i)
            for (int s = 0; s < nsel; ++s) {
                int t = sel ? sel[s] : s;
                double v = route_low != ROUTE_FULL ? (double)xrt[(size_t)s * win + i] : (double)x[(size_t)t * d + i];
                for (int j = 0; j < k; ++j)
                    d_w_gate[(size_t)i * N + idx[(size_t)s * k + j]] += v * dlg[(size_t)s * k + j];
            }
    }
    free(idx); free(gate); free(xlow); free(dyl); free(opair); free(dxp); free(dgt);
    free(ylow); free(dxl); free(dlg); free(xrt);
}

void oracle_bigmac_backward(int T, int d, int r, int N, int k, int h,
                            const float *x, const float *dy, const float *w_gate, const float *bias,
                            const float *w_down, const float *w_up, const float *w1, const float *w2,
                            int nsel, const int32_t *sel, const int32_t *keep,
                            double *dx, double *d_w_down, double *d_w_up, double *d_w_gate,
                            double *d_w1, double *d_w2)
{
    layer_backward(1, T, d, r, h, N, k, x, dy, w_gate, bias, w_down, w_up, w1, w2, NULL, NULL, ROUTE_FULL,
                   nsel, sel, keep, dx, d_w_down, d_w_up, d_w_gate, d_w1, d_w2, NULL, NULL);
}

/* With the variants of oracle_bigmac_forward_ext; d_b1 [N, h], d_b2 [N, r] are added to like the
 * other weight gradients (NULL: not wanted); d_w_gate is [r, N] when the router reads x'. */
void oracle_bigmac_backward_ext(int T, int d, int r, int N, int k, int h,
                                const float *x, const float *dy, const float *w_gate, const float *bias,
                                const float *w_down, const float *w_up, const float *w1, const float *w2,
                                const float *b1, const float *b2, int route_low,
                                int nsel, const int32_t *sel, const int32_t *keep,
                                double *dx, double *d_w_down, double *d_w_up, double *d_w_gate,
                                double *d_w1, double *d_w2, double *d_b1, double *d_b2)
{
    layer_backward(1, T, d, r, h, N, k, x, dy, w_gate, bias, w_down, w_up, w1, w2, b1, b2, route_low,
                   nsel, sel, keep, dx, d_w_down, d_w_up, d_w_gate, d_w1, d_w2, d_b1, d_b2);
}

/* Fine-grained layer backward: wdn [N, d, r], wup [N, r, d]; gradients d_wdn, d_wup likewise. */
void oracle_cdac_backward(int T, int d, int r, int N, int k,
                          const float *x, const float *dy, const float *w_gate, const float *bias,
                          const float *wdn, const float *wup, int nsel, const int32_t *sel,
                          const int32_t *keep,
                          double *dx, double *d_w_gate, double *d_wdn, double *d_wup)
{
    layer_backward(0, T, d, d, r, N, k, x, dy, w_gate, bias, NULL, NULL, wdn, wup, NULL, NULL, ROUTE_FULL,
                   nsel, sel, keep, dx, NULL, NULL, d_w_gate, d_wdn, d_wup, NULL, NULL);
}

/* Closed forms of Table 3, MoE-layer terms only (paper symbols: rho = r/d is the paper's r).
 * FLOPs of one iteration (forward + backward) per token per layer spent in the experts and, for
 * BigMac, in the two shared projections; bytes one token puts through the two All-to-Alls,
 * forward + backward, at e_b bytes per element, before the (ep-1)/ep factor. */
double oracle_moe_flops_per_token(int d, int r, int k, int bigmac)
{
    double rho = (double)r / (double)d;
    return 12.0 * (double)d * (double)d * rho * ((double)k + (bigmac ? 1.0 : 0.0));
}
double oracle_a2a_bytes_per_token(int d, int r, int k, int bigmac, int e_b)
{
    double width = bigmac ? (double)r : (double)d;
    return 4.0 * (double)k * width * (double)e_b;
}
