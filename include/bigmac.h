/*
 * bigmac.h - C ABI of the MI355X (gfx950) BigMac MoE layer library.
 *
 * The layer (paper Section 3.1, Eq. 2, "descend-communicate-communicate-ascend"):
 *     x' = x W_down ;   y' = sum_{i in T} p_i(x) E_i(x') ;   y = y' W_up
 * with the BigMac expert (Section 3.2, Eq. 4)  E_i(x') = act(x' W1[i]) W2[i]  (r -> h -> r),
 * T the top_k experts of the token (Section 2) and p_i its gate value.  On one GPU the two
 * All-to-Alls of Section 3.1 are an on-device permute (dispatch) and un-permute (combine) of
 * r-wide rows.  The fine-grained layer the paper compares with (CDAC order, Eq. 3) is the same
 * calls with order = BIGMAC_ORDER_CDAC: dispatch/combine at width d, expert d -> r -> d, no
 * shared projections.
 *
 * Conventions for every call
 *  - All data pointers are DEVICE pointers; `dims`, `params` are HOST structs read during the
 *    call.  Matrices are row-major and contiguous, weights are [in, out] (the paper's x.W),
 *    base pointers 16-byte aligned.  Index arrays are int32.
 *  - dtype is the storage type of x, dy, W_down, W_up, W1, W2 and of every permuted row
 *    (BIGMAC_F32: float, BIGMAC_BF16: bfloat16 bit patterns).  w_gate, gate_bias, gate values,
 *    logits and all weight gradients are always fp32.  All accumulation is fp32.
 *  - Widths: win = dispatch width (r for DCCA, d for CDAC), hid = expert hidden width (h for
 *    DCCA, r for CDAC).  d, r, h must be multiples of 64; 1 <= k <= N <= 1024; k <= 64; T*k < 2^31.
 *    With bf16 storage bigmac_layer_backward also needs N % 8 == 0 (the dense logit gradient is
 *    moved in 16-byte pieces of its N-wide rows): BIGMAC_ERR_UNSUPPORTED otherwise.  A matrix
 *    product whose tiles would span 2 GiB or more of one operand (T*k rows of the widest
 *    [rows, hidden] tensor in bf16) is refused with BIGMAC_ERR_TOO_LARGE.
 *  - The caller owns every buffer (inputs, outputs, workspace, saved block).  The library
 *    allocates nothing, keeps no state and never synchronises: a call only enqueues kernels on
 *    `stream` (a hipStream_t passed as void*; NULL = the default stream) and returns.  Nothing
 *    on the path is read back by the host; per-expert counts stay on the device.
 *  - Return value: 0 on success; negative on failure, in which case nothing was launched by the
 *    failing step: BIGMAC_ERR_INVALID_ARG (NULL required pointer, bad dimension or enum),
 *    BIGMAC_ERR_WORKSPACE (workspace too small), BIGMAC_ERR_UNSUPPORTED, BIGMAC_ERR_TOO_LARGE (a
 *    size beyond a stated limit), BIGMAC_ERR_HIP (a launch failed).  Inputs are assumed finite; NaN/Inf logits give unspecified routing.
 *  - Routing is dropless (Section 3.3) unless dims.capacity > 0: every (token, choice) pair
 *    keeps a row, the rows of an expert are contiguous and ordered by token,
 *    expert_offsets[N] = T*k.
 *  - Fixed expert capacity (the setting of the paper's training runs, Table 5: capacity factor
 *    f = 1.2, i.e. capacity = ceil(f T k / N); the paper gives no rule, this is the usual one):
 *    with dims.capacity = C > 0 an expert keeps the first C of its pairs in flat order
 *    f = t*k + j and drops the rest.  A dropped pair has slot_of = -1, no row, and contributes
 *    nothing to y (its gate value is not redistributed) nor to any gradient;
 *    expert_offsets[N] = number of kept pairs <= T*k, and rows at or beyond it are not touched.
 */
#ifndef BIGMAC_H
#define BIGMAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { BIGMAC_F32 = 0, BIGMAC_BF16 = 1 } bigmac_dtype;
typedef enum { BIGMAC_ACT_GELU_ERF = 0 } bigmac_act;             /* 0.5 a (1 + erf(a / sqrt 2)) */
typedef enum { BIGMAC_ORDER_DCCA = 0, BIGMAC_ORDER_CDAC = 1 } bigmac_order;

enum {
  BIGMAC_FLAG_ACCUMULATE = 1, /* backward: add weight gradients to the caller's buffers (else overwrite) */
  BIGMAC_FLAG_OUT_BF16 = 2,   /* layer calls with dtype BF16: write y / dx as bf16 (default: fp32)       */
  BIGMAC_FLAG_WIRE_BF16 = 4,  /* layer calls with dtype BF16: the rows returning through the second
                                 All-to-All (expert outputs) and, backward, through the first (the
                                 gradient of the dispatched rows) travel in bf16, the format of the
                                 paper's Table 4; default: those win-wide rows stay fp32, which is
                                 what keeps y and dx within 2e-2 of their RMS at the widest shapes,*/
  BIGMAC_FLAG_TILES_LARGE = 8, /* tuning: run every expert product that can on 256 x 256 workgroup tiles,  */
  BIGMAC_FLAG_TILES_SMALL = 16,/* or none of them (default: chosen from the shape).  Results do not depend
                                  on the tile: the same products are added in the same order.            */
  BIGMAC_FLAG_ROUTE_LOW = 32,  /* layer calls, DCCA order: the router reads x' instead of x (Section 3.1
                                  names both inputs): w_gate and d_w_gate are [r, N], the logits are those of
                                  bigmac_route on the stored x' (dtype) with d = r, and the gate's gradient
                                  reaches x through x' (and so W_down).  A fourth of the router's work.   */
  BIGMAC_FLAG_NO_FUSED_DISPATCH = 64  /* layer calls with dtype BF16 fold the dispatch step into a product:
                                  forward-only calls read the expert-up product's rows straight from x' (x
                                  in the CDAC order) through src_of and write no permuted copy; a DCCA
                                  training forward whose router reads x has the descending projection write
                                  each row of x' into the places of its pairs in the permuted copy.  With
                                  this flag the rows are dispatched by the copy kernel of bigmac_dispatch
                                  instead.  Same results bit for bit (tests and measurements).           */
};

enum {
  BIGMAC_OK = 0,
  BIGMAC_ERR_INVALID_ARG = -1,
  BIGMAC_ERR_WORKSPACE = -2,
  BIGMAC_ERR_UNSUPPORTED = -3,
  BIGMAC_ERR_HIP = -4,
  BIGMAC_ERR_TOO_LARGE = -5   /* bigmac_dispatch_static: the problem exceeds the library's static scratch */
};

typedef struct {
  int32_t T, d, r, N, k, h; /* tokens, model width, low width, experts, top_k, expert hidden width */
  int32_t dtype, act, order;
  int32_t flags;
  int32_t capacity;         /* 0: dropless.  C > 0: at most C pairs per expert (see above)         */
  float aux_alpha;          /* 0: none.  > 0: coefficient of the load-balance loss (bigmac_aux_loss) */
} bigmac_dims;

typedef struct {          /* parameters: caller-owned, never written                              */
  const void *w_down;     /* [d, r]   dtype   W'_down of Eq. 2         (ignored for CDAC)          */
  const void *w_up;       /* [r, d]   dtype   W'_up   of Eq. 2         (ignored for CDAC)          */
  const float *w_gate;    /* [d, N]   fp32    router weights                                       */
  const float *gate_bias; /* [N]      fp32 or NULL, added to the logits                            */
  const void *w1;         /* [N, win, hid] dtype   first expert matrix  (Eq. 4: W_i,up; Eq. 3: W_i,down) */
  const void *w2;         /* [N, hid, win] dtype   second expert matrix (Eq. 4: W_i,down; Eq. 3: W_i,up) */
  const void *b1;         /* [N, hid] dtype or NULL   expert biases (the 2rh term of the expert parameters in   */
  const void *b2;         /* [N, win] dtype or NULL   Table 3):  E_i(x') = act(x' W1[i] + b1[i]) W2[i] + b2[i]  */
} bigmac_params;

typedef enum {
  BIGMAC_WS_ROUTE = 0,
  BIGMAC_WS_DISPATCH = 1,
  BIGMAC_WS_GROUPED_FFN = 2,
  BIGMAC_WS_LAYER_FORWARD = 3,   /* inference (saved == NULL)                                      */
  BIGMAC_WS_LAYER_TRAIN = 4,     /* forward with a saved block, and backward                       */
  BIGMAC_WS_SAVED = 5,           /* size of the saved-activation block of a training forward       */
  BIGMAC_WS_AUX_LOSS = 6
} bigmac_ws_kind;

/* Host only, touches no GPU.  Bytes of workspace the given call needs for these dims
 * (0 if the dims are invalid).  Workspace contents are scratch: undefined after a call. */
size_t bigmac_workspace_bytes(const bigmac_dims *dims, int kind);

/* Host only.  Static text for a status code. */
const char *bigmac_status_string(int status);

/* Host only.  Algorithmic work of one call, from the closed forms behind the paper's Table 3:
 * matrix FLOPs of a forward pass (2 flops per multiply-add, real rows only), and the bytes the
 * four permutes (two forward, two backward) must move per layer call at this width. */
double bigmac_forward_matrix_flops(const bigmac_dims *dims);
double bigmac_permute_bytes(const bigmac_dims *dims);

/* Gating (Section 3.1: the router reads the full-width token x).
 * logits[t, n] = sum_i x[t, i] w_gate[i, n] (+ gate_bias[n]) in fp32 in a fixed order: 64
 * partial sums p_l over i = l mod 64 (ascending i, fused multiply-add), then a halving tree
 * p_l += p_{l+off} for off = 32, 16, 8, 4, 2, 1, then the bias.  topk_idx[t, 0..k) are the k
 * largest logits in descending order, equal logits to the lowest expert index; topk_w[t, j] is
 * the softmax over those k logits.  logits_out ([T, N], fp32) may be NULL. */
int bigmac_route(const bigmac_dims *dims, const void *x /*[T,d] dtype*/, const float *w_gate,
                 const float *gate_bias, int32_t *topk_idx /*[T,k]*/, float *topk_w /*[T,k]*/,
                 float *logits_out, void *ws, size_t ws_bytes, void *stream);

/* Load-balance auxiliary loss.  The paper trains with "aux_loss" balancing at coefficient 0.001
 * (Table 5) and gives no formula; this is the common one, stated here as this library's choice:
 *     loss = aux_alpha * N * sum_e f_e * P_e
 * f_e = share of the T*k (token, choice) pairs routed to expert e, counted before any capacity
 * drop; P_e = mean over the T tokens of softmax(logits[t, :])[e] over all N experts.  fp32; the
 * sums run in a fixed order, so equal inputs give equal bits.  Outputs: loss [1], share [N] (the
 * f_e) and, unless NULL, dlogits [T, N]: the gradient with f held fixed,
 *     dlogits[t, n] = aux_alpha * N / T * p[t, n] * (f_n - sum_e f_e p[t, e]).
 * With dims.aux_alpha > 0 bigmac_layer_forward (training form) evaluates the loss into the saved
 * block (bigmac_saved_aux_layout) and bigmac_layer_backward adds this gradient, scaled by an
 * upstream gradient of 1, to the router logits' gradient: it reaches d_w_gate and dx. */
int bigmac_aux_loss(const bigmac_dims *dims, const float *logits /*[T,N]*/, const int32_t *topk_idx /*[T,k]*/,
                    float *loss, float *share, float *dlogits, void *ws, size_t ws_bytes, void *stream);

/* First All-to-All of Section 3.1 on one device.  Builds the stable counting-sort permutation
 * of the flat pairs f = t*k + j by expert (expert_offsets [N+1], slot_of [T,k], src_of [T*k]
 * with src_of[slot_of[f]] = f) and copies x_low[t, :] to x_perm[slot_of[t, j], :] for every j.
 * x_low is [T, win], x_perm is [T*k, win], both dtype.  x_low == NULL (with x_perm == NULL)
 * builds the permutation only.  With dims.capacity > 0 the dropped pairs get slot_of = -1, and
 * x_perm rows and src_of entries at or beyond expert_offsets[N] are left as they were. */
int bigmac_dispatch(const bigmac_dims *dims, const void *x_low, const int32_t *topk_idx,
                    void *x_perm, int32_t *expert_offsets, int32_t *slot_of, int32_t *src_of,
                    void *ws, size_t ws_bytes, void *stream);

/* bigmac_dispatch for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and kernels as bigmac_dispatch, without `ws`: the counting sort's counters live in a 4 MiB array
 * inside the library's device image (one copy per GPU, held until the process ends).  The call
 * allocates and frees nothing.  It needs ceil(T*k / 1024) * N * 4 bytes of that array (T*k / 256
 * chunks while that many times N stays within 32768) and returns BIGMAC_ERR_TOO_LARGE beyond 4 MiB
 * (e.g. T*k = 2^23 pairs over 128 experts still fit).  All calls on one GPU share the array: calls
 * that overlap in time on one GPU (different streams, or threads) race; calls on one stream do not.
 * The first call on a device looks the array's address up (no allocation); make that call outside
 * a graph capture. */
int bigmac_dispatch_static(const bigmac_dims *dims, const void *x_low, const int32_t *topk_idx,
                           void *x_perm, int32_t *expert_offsets, int32_t *slot_of, int32_t *src_of,
                           void *stream);

/* The experts of Eq. 4 (Eq. 3 for CDAC) on permuted rows: for the rows s of expert e,
 * o_perm[s, :] = act(x_perm[s, :] W1[e] + b1[e]) W2[e] + b2[e].  b1 ([N, hid] dtype) and b2 ([N, win]
 * dtype) are the optional expert biases (Table 3 counts 2rh of them per expert); NULL: none.
 * act_saved ([T*k, hid] dtype, the pre-activation x_perm W1 + b1) may be NULL. */
int bigmac_grouped_ffn(const bigmac_dims *dims, const void *x_perm, const int32_t *expert_offsets,
                       const void *w1, const void *w2, const void *b1, const void *b2, void *act_saved,
                       void *o_perm /*[T*k,win] dtype*/, void *ws, size_t ws_bytes, void *stream);

/* Second All-to-All plus the weighted sum of Eq. 2: y_low[t, :] = sum_j topk_w[t, j] *
 * o_perm[slot_of[t, j], :], added in j order in fp32.  topk_w == NULL means unit weights (the
 * backward of dispatch).  A pair with slot_of < 0 (dropped by the capacity) is skipped.  y_low is
 * [T, win] fp32. */
int bigmac_combine(const bigmac_dims *dims, const void *o_perm, const int32_t *slot_of,
                   const float *topk_w, float *y_low, void *stream);

/* Whole layer forward (Eq. 2).  y is [T, d]: fp32, or bf16 with BIGMAC_FLAG_OUT_BF16 (always
 * float for dtype F32).  saved == NULL: inference.  Otherwise `saved` receives the activations
 * the backward call needs (size: BIGMAC_WS_SAVED) and ws must have BIGMAC_WS_LAYER_TRAIN bytes. */
int bigmac_layer_forward(const bigmac_dims *dims, const bigmac_params *params, const void *x,
                         void *y, void *saved, void *ws, size_t ws_bytes, void *stream);

/* Whole layer backward with the top-k set held fixed.  dy is [T, d] dtype, dx is [T, d] (type
 * as y).  Weight gradients are fp32 with the shapes of their weights and are overwritten, or
 * added to with BIGMAC_FLAG_ACCUMULATE; d_w_down / d_w_up are ignored for CDAC.  d_b1 [N, hid] and
 * d_b2 [N, win] are required exactly when params has b1 / b2 (column sums of the gradients of the
 * pre-activation and of the expert outputs over each expert's rows).  `saved` is the block written
 * by the forward call with the same dims, params and x. */
int bigmac_layer_backward(const bigmac_dims *dims, const bigmac_params *params, const void *x,
                          const void *dy, const void *saved, void *dx, float *d_w_down,
                          float *d_w_up, float *d_w_gate, float *d_w1, float *d_w2, float *d_b1,
                          float *d_b2, void *ws, size_t ws_bytes, void *stream);

/* Views into a saved block, for tests and tools: byte offsets of topk_idx [T,k] int32, topk_w
 * [T,k] fp32, expert_offsets [N+1] int32 and slot_of [T,k] int32 inside it.  Host only. */
int bigmac_saved_layout(const bigmac_dims *dims, size_t *off_topk_idx, size_t *off_topk_w,
                        size_t *off_expert_offsets, size_t *off_slot_of);

/* With dims.aux_alpha > 0: byte offsets inside a saved block of the loss (one float) and of the
 * pair shares f_e ([N] floats) that the training forward wrote.  Host only. */
int bigmac_saved_aux_layout(const bigmac_dims *dims, size_t *off_aux_loss, size_t *off_aux_share);

/* Profiling aid for callers that cannot allocate or want per-kernel times (benchmarks).  The
 * layer calls launch one kernel per stage below (a stage that a configuration skips records
 * nothing).  While an event table is set, bigmac_layer_forward / bigmac_layer_backward record
 * events[2*s] before and events[2*s + 1] after stage s on the call's stream; `events` is a HOST
 * array of 2 * BIGMAC_STAGE_COUNT hipEvent_t handles owned by the caller, which must stay alive
 * until it is replaced or cleared with NULL.  This is the library's only process-wide setting;
 * it is not thread-safe.  Returns BIGMAC_OK. */
typedef enum {
  BIGMAC_STAGE_ROUTER_LOGITS = 0, /* F0  x W_g                                   */
  BIGMAC_STAGE_TOPK_GATE,         /* F1  top-k and gate values                   */
  BIGMAC_STAGE_DESCEND,           /* F2  x' = x W_down                           */
  BIGMAC_STAGE_PERMUTATION,       /* F3  counting sort (3 small kernels) + tile map */
  BIGMAC_STAGE_DISPATCH,          /* F4  first All-to-All (row scatter)          */
  BIGMAC_STAGE_EXPERT_UP,         /* F5  act(x_perm W1[e])                       */
  BIGMAC_STAGE_EXPERT_DOWN,       /* F6  . W2[e]                                 */
  BIGMAC_STAGE_COMBINE,           /* F7  second All-to-All + weighted sum        */
  BIGMAC_STAGE_ASCEND,            /* F8  y = y' W_up                             */
  BIGMAC_STAGE_BWD_ASCEND_DGRAD,  /* B8  dy' = dy W_up^T                         */
  BIGMAC_STAGE_BWD_ASCEND_WGRAD,  /* B8  dW_up (split-K product + reduction)     */
  BIGMAC_STAGE_BWD_COMBINE,       /* B7  gate gradients, scaled scatter of dy'   */
  BIGMAC_STAGE_BWD_DOWN_DGRAD,    /* B6  dact = (do W2[e]^T) act'                */
  BIGMAC_STAGE_BWD_DOWN_WGRAD,    /* B6  dW2[e]                                  */
  BIGMAC_STAGE_BWD_UP_WGRAD,      /* B5  dW1[e]                                  */
  BIGMAC_STAGE_BWD_UP_DGRAD,      /* B5  dx_perm = dact W1[e]^T                  */
  BIGMAC_STAGE_BWD_DISPATCH,      /* B4  dx' = sum_j dx_perm                     */
  BIGMAC_STAGE_BWD_GATE,          /* B1  gate backward, router share of dx       */
  BIGMAC_STAGE_BWD_ROUTER_WGRAD,  /* B0  dW_g                                    */
  BIGMAC_STAGE_BWD_DESCEND_WGRAD, /* B2  dW_down                                 */
  BIGMAC_STAGE_BWD_DESCEND_DGRAD, /* B2  dx += dx' W_down^T                      */
  BIGMAC_STAGE_BWD_OUTPUT_CAST,   /* dx to bf16 / fine-grained dx sum            */
  BIGMAC_STAGE_COUNT
} bigmac_stage;
int bigmac_set_stage_events(void *const *events);

/* Measurement aid: the achievable dense bf16 matrix-core rate of the device, against which the
 * rates of the layer's products are set (the published peak is the other yardstick).  Enqueues one
 * kernel of `blocks` workgroups (256 threads) in which every wavefront issues 16 * iters
 * 32x32x16 bf16 MFMAs on register operands, no memory traffic.  sink: device, one float, never
 * written (keeps the arithmetic alive); *flops (host) receives the flops of the launch.  The
 * caller times the launch.  blocks in [1, 65536], iters in [1, 2^20]; else BIGMAC_ERR_INVALID_ARG. */
int bigmac_mfma_probe(int blocks, int iters, float *sink /*device*/, double *flops /*host*/, void *stream);

/* Measurement aid: what the device moves for the access pattern of the combine kernels without
 * any write in the mix, the ceiling their HBM fractions are set against.  Enqueues one kernel in
 * the combine kernels' launch shape (a thread per group of 8 rows and 32 bytes of the row) that
 * reads, for every m in [0, rows), all row_bytes bytes of row order[m] of `table` - 8 independent
 * 32-byte loads per thread, `streaming` != 0: with the non-temporal hint - and stores nothing.
 * table: device, rows * row_bytes bytes; order: device int32 [rows], a permutation of [0, rows)
 * or any indices below rows; sink: device, one uint32, never written.  rows a multiple of 8,
 * row_bytes a multiple of 32, rows * row_bytes < 2^40; else BIGMAC_ERR_INVALID_ARG.  The caller
 * times the launch; it reads rows * row_bytes bytes. */
int bigmac_gather_probe(const void *table, const int32_t *order, int64_t rows, int64_t row_bytes, int streaming,
                        uint32_t *sink, void *stream);
const char *bigmac_stage_name(int stage);
/* Where a layer forward with these dims does its dispatch step (Section 3.1's first All-to-All,
 * on one GPU a row copy): 0 = the copy kernel of bigmac_dispatch; 1 = folded into the expert-up
 * product, which reads its rows through src_of (forward-only calls, saved == NULL); 2 = folded
 * into the descending projection, whose epilogue writes the rows of x' through slot_of (training
 * calls).  See BIGMAC_FLAG_NO_FUSED_DISPATCH.  Measurement code uses it to price the stages.
 * training: 0 = a call with saved == NULL.  Negative: an error code for bad dims. */
int bigmac_dispatch_folding(const bigmac_dims *dims, int training);

#ifdef __cplusplus
}
#endif
#endif /* BIGMAC_H */
