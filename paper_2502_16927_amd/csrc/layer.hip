// C ABI of libbigmac: argument checks, workspace planning and the launch sequences of the
// layer (Eq. 2 with the expert of Eq. 4; CDAC order with the expert of Eq. 3) and its backward.
#include "common.hpp"
#include "tile_map.hpp"

namespace bigmac {

int check_dims(const bigmac_dims* D) {
  if (!D) return BIGMAC_ERR_INVALID_ARG;
  if (D->T < 1 || D->d < 64 || D->r < 64 || D->N < 1 || D->k < 1) return BIGMAC_ERR_INVALID_ARG;
  if (D->d % 64 || D->r % 64) return BIGMAC_ERR_INVALID_ARG;
  if (D->order != BIGMAC_ORDER_DCCA && D->order != BIGMAC_ORDER_CDAC) return BIGMAC_ERR_INVALID_ARG;
  if (D->order == BIGMAC_ORDER_DCCA && (D->h < 64 || D->h % 64)) return BIGMAC_ERR_INVALID_ARG;
  if (D->k > D->N || D->N > 1024 || D->k > 64) return BIGMAC_ERR_INVALID_ARG;
  if ((long long)D->T * D->k >= (1ll << 31)) return BIGMAC_ERR_INVALID_ARG;
  if (D->dtype != BIGMAC_F32 && D->dtype != BIGMAC_BF16) return BIGMAC_ERR_INVALID_ARG;
  if (D->act != BIGMAC_ACT_GELU_ERF) return BIGMAC_ERR_INVALID_ARG;
  if (D->flags & ~(BIGMAC_FLAG_ACCUMULATE | BIGMAC_FLAG_OUT_BF16 | BIGMAC_FLAG_WIRE_BF16 | BIGMAC_FLAG_TILES_LARGE | BIGMAC_FLAG_TILES_SMALL | BIGMAC_FLAG_ROUTE_LOW |
                   BIGMAC_FLAG_NO_FUSED_DISPATCH)) return BIGMAC_ERR_INVALID_ARG;
  if ((D->flags & BIGMAC_FLAG_TILES_LARGE) && (D->flags & BIGMAC_FLAG_TILES_SMALL)) return BIGMAC_ERR_INVALID_ARG;
  if (D->capacity < 0 || !(D->aux_alpha >= 0.0f) || D->aux_alpha > 1e30f) return BIGMAC_ERR_INVALID_ARG;
  if (D->order == BIGMAC_ORDER_CDAC && D->dtype == BIGMAC_BF16 && (D->flags & BIGMAC_FLAG_OUT_BF16)) return BIGMAC_ERR_UNSUPPORTED;
  if ((D->flags & BIGMAC_FLAG_ROUTE_LOW) && D->order == BIGMAC_ORDER_CDAC) return BIGMAC_ERR_INVALID_ARG;   // the fine-grained layer has no x'
  if ((D->flags & BIGMAC_FLAG_ROUTE_LOW) && D->aux_alpha > 0.0f) return BIGMAC_ERR_UNSUPPORTED;
  return BIGMAC_OK;
}

namespace {

void* const* g_stage_events = nullptr;  // profiling aid, see bigmac_set_stage_events

struct StageTimer {  // records the caller's events around the launches of one stage
  hipStream_t s;
  int stage;
  StageTimer(hipStream_t s_, int stage_) : s(s_), stage(stage_) {
    if (g_stage_events) (void)hipEventRecord((hipEvent_t)g_stage_events[2 * stage], s);
  }
  ~StageTimer() {
    if (g_stage_events) (void)hipEventRecord((hipEvent_t)g_stage_events[2 * stage + 1], s);
  }
};
#ifndef BIGMAC_DEEP_MAX_TILES
#define BIGMAC_DEEP_MAX_TILES 256   // 128 x 128 tiles (one per CU) up to which a dense product takes the 128 x 64 x 64 tile
#endif
// Which products take the square tile with 64-deep k tiles (two ring stages) when they do not
// take the tall one: 1 expert-up, 2 expert-down, 4 the GELU' product, 8 the data gradient of the
// first matrix, 16 the data gradient of the descending projection, 32 the ascending projection.
// Measured at gpt_medium: -1 %, +2.5 %, +3 %, -6 %, -11 %, -8 %.
#ifndef BIGMAC_WIDEK_MASK
#define BIGMAC_WIDEK_MASK 56
#endif
#ifndef BIGMAC_DEEP_WGRAD_MAX_TILES
#define BIGMAC_DEEP_WGRAD_MAX_TILES 16   // measured: 16 tiles 15.5 -> 13.2 us; 64 tiles (gpt_xl widths) 43 -> 48 us
#endif
#ifndef BIGMAC_DEEP_K_TILE_US
#define BIGMAC_DEEP_K_TILE_US 0.7
#endif
#define BIGMAC_STAGE(stage) StageTimer stage_timer_##stage(s, stage)

struct Carver {  // hands out 256-byte aligned pieces of one buffer
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t o = off;
    off += align_up(bytes);
    return o;
  }
};

struct SavedPlan {
  size_t topk_idx, topk_w, offsets, slot_of, src_of, tile_map, tile_map_tall, x_perm, act, hact, o_perm, y_low, logits, aux, x_low, total;
};
struct FwdPlan {
  size_t logits, perm, x_low, partials, aux, claims, total;
};
struct BwdPlan {
  size_t dy_low, dgate, do_perm, dx_perm, dact, dx_low, dL, route, dx_f32, part_up, part_gate, part_down, tmp_f32, bias_sums, gate_low, w_up_t, w_down_t, claims, total;
};

inline bool bf(const bigmac_dims& D) { return D.dtype == BIGMAC_BF16; }
inline bool route_low(const bigmac_dims& D) { return (D.flags & BIGMAC_FLAG_ROUTE_LOW) != 0; }
// the router's view of the dims: with the router on x' its input is r wide
inline bigmac_dims router_dims(const bigmac_dims& D) {
  bigmac_dims R = D;
  if (route_low(D)) R.d = D.r;
  return R;
}
// y' and dx' feed a bf16 MFMA product; they are carried as two bf16 halves (hi | lo) so that
// the product sees them at fp32 precision.  Row length of that operand:
inline int low_ld(const bigmac_dims& D) { return bf(D) ? 2 * D.r : D.r; }
// Row pitch of the layer's own [rows, hidden] tensors (activations kept for the backward pass and
// their gradients).  In bf16 the pitch is 64 elements more than the width: with a power-of-two
// pitch the k rows that a weight-gradient product walks through map onto few L2 sets, and on
// experts with many rows the operand tiles shared between workgroups were fetched several times
// (measured: up to 1.3x faster weight-gradient products at 16384 rows per expert).
inline int wide_ld(const bigmac_dims& D) { return widths(D).hid + (bf(D) ? 64 : 0); }
// The rows that come back through the second All-to-All (expert outputs O) and, in the backward
// pass, through the first (dx_perm) are only win wide.  With bf16 storage the layer calls keep
// them in fp32 unless BIGMAC_FLAG_WIRE_BF16 asks for the all-bf16 wire format: rounding them
// costs as much precision as rounding the hidden activations, for a fraction of the bytes, and
// the rounding of O is what the gate gradient <dy', O_j> sees.
inline bool wire_f32(const bigmac_dims& D) { return bf(D) && !(D.flags & BIGMAC_FLAG_WIRE_BF16); }
inline int wire_dtype(const bigmac_dims& D) { return wire_f32(D) ? BIGMAC_F32 : D.dtype; }
inline size_t low_bytes(const bigmac_dims& D) { return (size_t)D.T * (bf(D) ? 2 * D.r * 2 : D.r * 4); }

// Which products run on the GEMM's tall (256-row) workgroup tiles.  The per-expert products on
// permuted rows (expert up/down, the data gradient of the first matrix): when there are enough
// tall tiles to fill the chip a few times over, K is at least 512 and the experts hold 512 rows
// on average (measured: 4-18 % faster at the gpt_xl to zipf_stress shapes; level or slower at
// the gpt_medium shapes, where K = r = 256 or the tile count is low).  The per-expert weight
// gradients: whenever their M divides into tall tiles (22-30 % faster at the large shapes, level
// at gpt_medium).  The products over the token index have few tiles and stay on the square tile.
inline bool tall_rows(const bigmac_dims& D, int cols, int K) {
  if (!bf(D)) return false;
  const long Tk = (long)D.T * D.k;
  const long tiles = (Tk / 256 + D.N) * ((cols + 127) / 128);
  return tiles >= 1536 && K >= 512 && Tk / D.N >= 512;
}
inline bool tall_wgrad(const bigmac_dims& D, int M) {   // up to a fifth of padding in M still pays
  return bf(D) && (long)((M + 255) / 256) * 256 * 5 <= (long)M * 6;
}
// The shared projections and their data gradients: the same rule as for the per-expert products.
inline bool tall_dense(const bigmac_dims& D, int M, int N, int K) {
  return bf(D) && (long)(M / 256) * ((N + 127) / 128) >= 1024 && K >= 512;
}
// Few 128 x 128 tiles under a long K: the narrower tile with deeper k tiles (see launch_gemm).
inline bool deep_dense(const bigmac_dims& D, int M, int N, int K) {
  return bf(D) && K % 64 == 0 && K >= 512 && (long)((M + 127) / 128) * ((N + 127) / 128) <= BIGMAC_DEEP_MAX_TILES;
}
// Expert weights read line by line as a grouped product starts (GemmDesc::touch); bits: 1 expert-up,
// 2 expert-down, 4 GELU' product, 8 the first matrix's data gradient.  Measured: it pays where
// an expert has so few output tiles that they all run at once and each meets its weights in
// memory (expert-up at gpt_medium, 64 tiles per expert and K = 256: 102 -> 81 us), costs a few us
// where an expert's first tiles fetch the weights for many later ones (8192 rows per expert:
// +6 us) or where every matrix is read by one or two row tiles anyway (up to 256 rows per expert:
// +2 to +3 us), and reading more than a fraction of the 256 MB memory-side cache ahead costs more
// than it saves (128 MB at gpt_xl: +30 us); the other three products lose 1 to 4 us by it.
#ifndef BIGMAC_TOUCH_MASK
#define BIGMAC_TOUCH_MASK 1
#endif
#ifndef BIGMAC_TOUCH_MAX_BYTES
#define BIGMAC_TOUCH_MAX_BYTES ((size_t)64 << 20)
#endif
#ifndef BIGMAC_TOUCH_MAX_TILES
#define BIGMAC_TOUCH_MAX_TILES 256
#endif
#ifndef BIGMAC_TOUCH_MIN_ROWS
#define BIGMAC_TOUCH_MIN_ROWS 512
#endif
inline void touch_weights(const bigmac_dims& D, GemmDesc& g, const void* w, int bit) {
  const size_t bytes = (size_t)D.N * g.K * g.N * 2;
  const long rows_per_expert = ((long)D.T * D.k + D.N - 1) / D.N;
  const long tiles_per_expert = ((rows_per_expert + 127) / 128) * ((g.N + 127) / 128);   // 128 x 128 output tiles
  if (bf(D) && (BIGMAC_TOUCH_MASK & bit) && bytes <= BIGMAC_TOUCH_MAX_BYTES && tiles_per_expert <= BIGMAC_TOUCH_MAX_TILES &&
      rows_per_expert >= BIGMAC_TOUCH_MIN_ROWS) {
    g.touch = w;
    g.touch_bytes = bytes;
  }
}
inline bool wide_k_ok(const bigmac_dims& D, int K, int bit) {
  return bf(D) && (BIGMAC_WIDEK_MASK & bit) && K % 64 == 0;
}
// Which products run on 256 x 256 tiles (eight wavefronts, one workgroup per CU): the per-expert
// row products that qualify for the tall tile and have K >= 2048.  Per flop that tile asks the L2
// for two thirds of the operand bytes of the tall one, and these products run at the rate their
// operands arrive at; its epilogue is not overlapped by another workgroup's k loop, which is what
// a shorter K does not pay for.  Measured (tall -> 256 x 256): zipf_stress expert-down and the
// first matrix's data gradient (K = 2048) 1.27 -> 1.19 ms and 1.36 -> 1.27 ms, gpt_xl 0.287 ->
// 0.275 ms and level; expert-up at K = 512 / 1024 3-6 % slower; the ragged-K weight gradients
// 5-7 % slower, so they take it only under BIGMAC_FLAG_TILES_LARGE.
inline bool big_rows(const bigmac_dims& D, int cols, int K) {
  if (!bf(D) || (D.flags & BIGMAC_FLAG_TILES_SMALL)) return false;
  if (D.flags & BIGMAC_FLAG_TILES_LARGE) return true;
  return K >= 2048 && cols % 256 == 0 && tall_rows(D, cols, K);
}
inline bool big_wgrad(const bigmac_dims& D) { return bf(D) && (D.flags & BIGMAC_FLAG_TILES_LARGE) && !(D.flags & BIGMAC_FLAG_TILES_SMALL); }
inline bool any_tall_rows(const bigmac_dims& D) {   // a tile map of 256-row tiles is needed
  const Widths W = widths(D);
  return tall_rows(D, W.hid, W.win) || tall_rows(D, W.win, W.hid) || big_rows(D, W.hid, W.win) || big_rows(D, W.win, W.hid);
}

SavedPlan plan_saved(const bigmac_dims& D) {
  const Widths W = widths(D);
  const size_t Tk = (size_t)D.T * D.k, es = esize(D.dtype);
  Carver c;
  SavedPlan p;
  p.topk_idx = c.take(Tk * 4);
  p.topk_w = c.take(Tk * 4);
  p.offsets = c.take((size_t)(D.N + 1) * 4);
  p.slot_of = c.take(Tk * 4);
  p.src_of = c.take(Tk * 4);
  p.tile_map = c.take(tile_map_ints((int)Tk, D.N, gemm_ragged_tile_rows(D.dtype, 0)) * 4);
  p.tile_map_tall = c.take(any_tall_rows(D) ? tile_map_ints((int)Tk, D.N, gemm_ragged_tile_rows(D.dtype, 1)) * 4 : 0);
  p.x_perm = c.take(Tk * W.win * es);
  p.act = c.take(Tk * wide_ld(D) * es);
  p.hact = c.take(Tk * wide_ld(D) * es);
  p.o_perm = c.take(Tk * W.win * esize(wire_dtype(D)));
  p.y_low = c.take(D.order == BIGMAC_ORDER_DCCA ? low_bytes(D) : 0);
  // load-balance loss: the backward pass needs the logits and the experts' pair shares; aux holds
  // the loss (one float) followed, 256 bytes on, by share[N]
  p.logits = c.take(D.aux_alpha > 0.0f ? (size_t)D.T * D.N * 4 : 0);
  p.aux = c.take(D.aux_alpha > 0.0f ? 256 + (size_t)D.N * 4 : 0);
  // router on x': the backward pass needs x' itself (the router's input) for d_w_gate
  p.x_low = c.take(route_low(D) ? (size_t)D.T * D.r * es : 0);
  p.total = c.off;
  return p;
}

// Split of K for a dense forward product [M,K] x [K,N] with few output tiles and a long K (the
// shared projections at decode sizes: a handful of tiles would otherwise walk K alone on a
// handful of CUs).  fp32 partials, reduced in slice order.  1 = no split.
int forward_ksplit(const bigmac_dims& D, int M, int N, int K) {
  if (!bf(D)) return 1;
  const int tiles = ((M + 127) / 128) * ((N + 127) / 128);
  if (tiles >= 128 && K <= 2048) return 1;
  int ks = K / 256;
  if (ks > 512 / tiles) ks = 512 / tiles;
  if (ks > 32) ks = 32;
  return ks < 1 ? 1 : ks;
}
size_t forward_partials_bytes(const bigmac_dims& D) {
  if (D.order != BIGMAC_ORDER_DCCA) return 0;
  const int ka = forward_ksplit(D, D.T, D.r, D.d), kb = forward_ksplit(D, D.T, D.d, low_ld(D));
  const size_t a = ka > 1 ? (size_t)ka * D.T * D.r * 4 : 0, b = kb > 1 ? (size_t)kb * D.T * D.d * 4 : 0;
  return a > b ? a : b;
}

FwdPlan plan_fwd(const bigmac_dims& D) {
  Carver c;
  FwdPlan p;
  p.logits = c.take((size_t)D.T * D.N * 4);
  p.perm = c.take(permutation_ws_bytes(D.T, D.k, D.N));
  p.x_low = c.take(D.order == BIGMAC_ORDER_DCCA ? (size_t)D.T * D.r * esize(D.dtype) : 0);
  p.partials = c.take(forward_partials_bytes(D));
  p.aux = c.take(D.aux_alpha > 0.0f ? aux_loss_ws_bytes(D) : 0);
  p.claims = c.take(CLAIM_BYTES);
  p.total = c.off;
  return p;
}

// The weight gradients over the token index take the tall tile when there are enough tall
// tiles and enough tokens to be worth it (measured: zipf_stress, T = 32768, d = 4096: 0.34 ->
// 0.25 ms and 0.38 -> 0.28 ms; at T = 8192 with the same widths level or slower).
inline bool tall_token_wgrad(const bigmac_dims& D, int M, int N) {
  return bf(D) && M % 256 == 0 && (long)(M / 256) * ((N + 127) / 128) >= 128 && D.T >= 16384;
}
// Slices of K for a weight gradient over the token index (few output tiles, K = T).  More slices
// fill more of the chip but write and read back more fp32 partials; the count is the power of
// two (slices of at least 256 rows) with the lowest estimate of product + reduction time:
// rounds of 768 resident workgroups x k tiles per slice x 0.6 us (measured per k tile of 32)
// + partial bytes, written and read once, at 5 TB/s.
// (On the tall tile: 512 resident workgroups, 0.85 us per k tile.)
enum TileShape { TILE_SQUARE, TILE_TALL, TILE_DEEP };
int choose_ksplit(int M, int N, int K, TileShape shape = TILE_SQUARE) {
  const int bm = shape == TILE_TALL ? 256 : 128, bn = shape == TILE_DEEP ? 64 : 128, bk = shape == TILE_DEEP ? 64 : 32;
  const long tiles = (long)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
  const long resident = shape == TILE_SQUARE ? 768 : 512;
  const double k_tile_us = shape == TILE_TALL ? 0.85 : (shape == TILE_DEEP ? BIGMAC_DEEP_K_TILE_US : 0.6);
  const double partial_us = (double)M * N * 4 * 2 / 5e6;
  int best = 1;
  double best_us = 1e30;
  for (int ks = 1; ks <= 64 && K / ks >= 256; ks *= 2) {
    const long rounds = (tiles * ks + resident - 1) / resident;
    const double us = rounds * ((K / ks + bk - 1) / bk) * k_tile_us + (ks > 1 ? ks * partial_us : 0.0);
    if (us <= best_us * 1.05) { best_us = us < best_us ? us : best_us; best = ks; }   // near ties go to more workgroups
  }
  return best;
}
// Tile shape and slice count of a weight gradient over the token index ([M, T] x [T, N]); the
// plan of the partials and the launch both take them from here.
// Few output tiles (K = T is long by nature): the 128 x 64 tile with 64-deep k tiles.
inline TileShape token_wgrad_shape(const bigmac_dims& D, int M, int N) {
  if (tall_token_wgrad(D, M, N)) return TILE_TALL;
  if (bf(D) && (long)((M + 127) / 128) * ((N + 127) / 128) <= BIGMAC_DEEP_WGRAD_MAX_TILES) return TILE_DEEP;
  return TILE_SQUARE;
}
inline int token_wgrad_ksplit(const bigmac_dims& D, int M, int N) { return choose_ksplit(M, N, D.T, token_wgrad_shape(D, M, N)); }

// The data gradients of the two shared projections (dy W_up^T, dx' W_down^T) contract over the
// fast index of the weight as it is stored: both operands k-contiguous, half a cache line per
// row and k tile.  Where those products are large enough for the 256-row tile, a transposed copy
// of the weight (8 MB at d = 4096, r = 1024: two launches of a few microseconds) gives them the
// operand layouts of the forward projections and with them the 128 x 256 tile.
inline bool transposed_projections(const bigmac_dims& D) {
  return D.order == BIGMAC_ORDER_DCCA && bf(D) && tall_dense(D, D.T, D.r, D.d) && tall_dense(D, D.T, D.d, low_ld(D)) &&
         D.r % 8 == 0 && D.d % 8 == 0;
}
// out[c][r] = in[r][c] for 16-bit elements, 64 x 64 tiles through the LDS
__global__ __launch_bounds__(256) void transpose_b16_kernel(const uint16_t* __restrict__ in, uint16_t* __restrict__ out, int rows, int cols) {
  __shared__ uint16_t tile[64][66];
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64, tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4)
    if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = in[(size_t)(r0 + i) * cols + c0 + tx];
  __syncthreads();
  for (int i = ty; i < 64; i += 4)
    if (c0 + i < cols && r0 + tx < rows) out[(size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

BwdPlan plan_bwd(const bigmac_dims& D) {
  const Widths W = widths(D);
  const size_t Tk = (size_t)D.T * D.k, es = esize(D.dtype);
  const bool dcca = D.order == BIGMAC_ORDER_DCCA;
  Carver c;
  BwdPlan p;
  p.dy_low = c.take((size_t)D.T * W.win * 4);
  p.dgate = c.take(Tk * 4);
  p.do_perm = c.take(Tk * W.win * es);
  p.dx_perm = wire_f32(D) ? c.take(Tk * W.win * 4) : p.do_perm;   // same width: do_perm is dead once the second matrix's gradients are done
  p.dact = c.take(Tk * wide_ld(D) * es);
  p.dx_low = c.take(dcca ? low_bytes(D) : (size_t)D.T * D.d * 4);
  p.dL = c.take((size_t)D.T * D.N * es);
  p.route = c.take(route_backward_ws_bytes(router_dims(D)));
  p.dx_f32 = c.take((bf(D) && (D.flags & BIGMAC_FLAG_OUT_BF16)) ? (size_t)D.T * D.d * 4 : 0);
  // split-K partials of the three weight gradients over the token index: one region each, so
  // that one launch at the end can reduce all three
  const int dg = router_dims(D).d;   // rows of w_gate
  p.part_gate = c.take((size_t)token_wgrad_ksplit(D, dg, D.N) * dg * D.N * 4);
  p.part_up = c.take(dcca ? (size_t)token_wgrad_ksplit(D, D.r, D.d) * D.r * D.d * 4 : 0);
  p.part_down = c.take(dcca ? (size_t)token_wgrad_ksplit(D, D.d, D.r) * D.d * D.r * 4 : 0);
  p.tmp_f32 = 0;
  // transposed copies of the two shared matrices for the data gradients of the projections (see transposed_projections)
  p.w_up_t = c.take(transposed_projections(D) ? (size_t)D.d * D.r * es : 0);
  p.w_down_t = c.take(transposed_projections(D) ? (size_t)D.d * D.r * es : 0);
  // expert biases: partial column sums (sized for the wider of the two bias vectors; taken always,
  // the plan does not see the parameters); router on x': its share of dx' in fp32
  p.bias_sums = c.take(ragged_colsum_ws_bytes(D.N, W.hid > W.win ? W.hid : W.win));
  p.gate_low = c.take(route_low(D) ? (size_t)D.T * D.r * 4 : 0);
  p.claims = c.take(CLAIM_BYTES);
  p.total = c.off;
  return p;
}

size_t ffn_ws_bytes(const bigmac_dims& D) {
  const Widths W = widths(D);
  const size_t Tk = (size_t)D.T * D.k;
  return align_up(Tk * W.hid * esize(D.dtype)) + 2 * align_up(tile_map_ints((int)Tk, D.N, gemm_ragged_tile_rows(D.dtype, 0)) * 4) +
         align_up(CLAIM_BYTES);
}

template <typename ET>
__global__ void to_f32_kernel(const ET* __restrict__ in, float* __restrict__ out, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = Elem<ET>::load(in + i);
}
__global__ void f32_to_bf16_kernel(const float* __restrict__ in, bf16_t* __restrict__ out, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = f2bf(in[i]);
}
__global__ void add_f32_kernel(float* __restrict__ acc, const float* __restrict__ in, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) acc[i] += in[i];
}
inline dim3 grid1d(size_t n) { return dim3((unsigned)((n + 255) / 256)); }

GemmDesc base_desc(const bigmac_dims& D) {
  GemmDesc g = {};
  g.dtype = D.dtype;
  g.ksplit = 1;
  g.mode = GEMM_DENSE;
  return g;
}

// The two expert products on permuted rows (ragged per-expert row ranges).
int run_experts_forward(const bigmac_dims& D, const void* x_perm, const int* offsets, const int* tile_map, const int* tile_map_tall,
                        const void* w1, const void* w2, const void* b1, const void* b2, void* act, void* hact, int ld_wide, void* o_perm, int o_f32,
                        hipStream_t s, const int* gather = nullptr) {
  const Widths W = widths(D);
  const int Tk = D.T * D.k;
  GemmDesc g = base_desc(D);
  g.mode = GEMM_RAGGED_M;
  g.a_kcontig = 1; g.b_kcontig = 0;
  g.groups = D.N; g.max_rows = Tk; g.offsets = offsets;
  // hact = gelu(x_perm W1[e])
  g.epilogue = EPI_GELU;
  g.big_tile = big_rows(D, W.hid, W.win);
  g.tall_tile = !g.big_tile && tall_rows(D, W.hid, W.win); g.tile_map = (g.tall_tile || g.big_tile) ? tile_map_tall : tile_map;
  if (g.tall_tile) { g.tall_tile = 0; g.long_tile = 1; g.tile_map = tile_map; }   // this product: the tall tile on its side (see launch_mfma_long)
  g.wide_k = !g.tall_tile && !g.big_tile && !g.long_tile && !gather && wide_k_ok(D, W.win, 1);
  g.A = x_perm; g.lda = W.win; g.K = W.win;
  g.gather = gather; g.gather_rows = D.T; g.gather_div = D.k;   // with an index, x_perm is the [T, win] rows before the dispatch
  g.B = w1; g.ldb = W.hid; g.gstride_b = (long)W.win * W.hid; g.N = W.hid;
  g.C = hact; g.ldc = ld_wide; g.aux_out = act;
  g.bias = b1; g.gstride_bias = W.hid;
  if (!g.big_tile) touch_weights(D, g, w1, 1);
  // measured: -3 % at K = 512 (gpt_xl); at K = 256 (gpt_medium) +2 % while the weights came from
  // memory, -4.6 % with the warm-up
  g.kloop_priority = W.win >= 512 || g.touch_bytes != 0;
  int rc;
  {
    BIGMAC_STAGE(BIGMAC_STAGE_EXPERT_UP);
    rc = launch_gemm(g, s);
  }
  if (rc) return rc;
  // o_perm = hact W2[e]
  g.gather = nullptr; g.gather_rows = 0;
  g.epilogue = EPI_STORE; g.out_f32 = o_f32; g.aux_out = nullptr;
  g.A = hact; g.lda = ld_wide; g.K = W.hid;
  g.B = w2; g.ldb = W.win; g.gstride_b = (long)W.hid * W.win; g.N = W.win;
  g.C = o_perm; g.ldc = W.win;
  g.bias = b2; g.gstride_bias = W.win;
  g.big_tile = big_rows(D, W.win, W.hid);
  g.long_tile = 0;
  g.tall_tile = !g.big_tile && tall_rows(D, W.win, W.hid); g.tile_map = (g.tall_tile || g.big_tile) ? tile_map_tall : tile_map;
  g.wide_k = !g.tall_tile && !g.big_tile && wide_k_ok(D, W.hid, 2);
  g.kloop_priority = 1;
  g.touch = nullptr; g.touch_bytes = 0;
  if (!g.big_tile) touch_weights(D, g, w2, 2);
  BIGMAC_STAGE(BIGMAC_STAGE_EXPERT_DOWN);
  return launch_gemm(g, s);
}

// dense fp32 C (+)= A^T-style product over the token index, split over K into fp32 partials; the
// reduction (fixed slice order) is left to the caller as a job for launch_reduce_partials_multi
int run_token_wgrad(const bigmac_dims& D, const void* A, long lda, int M, const void* B, long ldb, int N,
                    float* out, float* partials, ReduceJob* job, hipStream_t s) {
  GemmDesc g = base_desc(D);
  g.a_kcontig = 0; g.b_kcontig = 0;
  g.epilogue = EPI_ACCUM; g.beta = 0;
  g.A = A; g.lda = lda; g.M = M; g.B = B; g.ldb = ldb; g.N = N; g.K = D.T;
  const TileShape shape = token_wgrad_shape(D, M, N);
  g.tall_tile = shape == TILE_TALL;
  g.deep_tile = shape == TILE_DEEP;
  g.ksplit = token_wgrad_ksplit(D, M, N);
  g.C = partials; g.ldc = N; g.gstride_c = (long)M * N;
  job->part = partials; job->out = out; job->n = (size_t)M * N; job->nslices = g.ksplit;
  return launch_gemm(g, s);
}

}  // namespace
}  // namespace bigmac

using namespace bigmac;

extern "C" {

size_t bigmac_workspace_bytes(const bigmac_dims* D, int kind) {
  if (check_dims(D) != BIGMAC_OK) return 0;
  switch (kind) {
    case BIGMAC_WS_ROUTE: return align_up((size_t)D->T * D->N * 4);
    case BIGMAC_WS_DISPATCH: return permutation_ws_bytes(D->T, D->k, D->N);
    case BIGMAC_WS_GROUPED_FFN: return ffn_ws_bytes(*D);
    case BIGMAC_WS_LAYER_FORWARD: return plan_fwd(*D).total + plan_saved(*D).total;
    case BIGMAC_WS_LAYER_TRAIN: {
      const size_t f = plan_fwd(*D).total, b = plan_bwd(*D).total;
      return f > b ? f : b;
    }
    case BIGMAC_WS_SAVED: return plan_saved(*D).total;
    case BIGMAC_WS_AUX_LOSS: return aux_loss_ws_bytes(*D);
    default: return 0;
  }
}

const char* bigmac_status_string(int status) {
  switch (status) {
    case BIGMAC_OK: return "ok";
    case BIGMAC_ERR_INVALID_ARG: return "invalid argument (null pointer, bad dimension or enum)";
    case BIGMAC_ERR_WORKSPACE: return "workspace too small";
    case BIGMAC_ERR_UNSUPPORTED: return "unsupported combination";
    case BIGMAC_ERR_HIP: return "HIP launch failed";
    case BIGMAC_ERR_TOO_LARGE: return "problem exceeds the static scratch of the allocation-free entry point";
    default: return "unknown status";
  }
}

double bigmac_forward_matrix_flops(const bigmac_dims* D) {
  if (check_dims(D) != BIGMAC_OK) return 0.0;
  const Widths W = widths(*D);
  double f = 4.0 * (double)D->T * D->k * W.win * W.hid;
  if (D->order == BIGMAC_ORDER_DCCA) f += 4.0 * (double)D->T * D->d * D->r;
  return f;
}

double bigmac_permute_bytes(const bigmac_dims* D) {
  if (check_dims(D) != BIGMAC_OK) return 0.0;
  return 4.0 * (double)D->T * D->k * widths(*D).win * esize(D->dtype);
}

int bigmac_gather_probe(const void* table, const int32_t* order, int64_t rows, int64_t row_bytes, int streaming, uint32_t* sink, void* stream) {
  if (!table || !order || !sink || rows <= 0 || rows % 8 || row_bytes <= 0 || row_bytes % 32 || rows > (1ll << 31) - 8 || row_bytes > (1ll << 24) ||
      rows * row_bytes >= (1ll << 40))
    return BIGMAC_ERR_INVALID_ARG;
  return launch_gather_probe(table, order, (long)rows, (long)row_bytes, streaming, sink, (hipStream_t)stream);
}

int bigmac_mfma_probe(int blocks, int iters, float* sink, double* flops, void* stream) {
  if (blocks <= 0 || blocks > 65536 || iters <= 0 || iters > (1 << 20) || !sink || !flops) return BIGMAC_ERR_INVALID_ARG;
  const double f = launch_mfma_probe(blocks, iters, sink, (hipStream_t)stream);
  if (f < 0) return BIGMAC_ERR_HIP;
  *flops = f;
  return BIGMAC_OK;
}

int bigmac_set_stage_events(void* const* events) {
  g_stage_events = events;
  return BIGMAC_OK;
}

namespace {
// training forward: the descending projection writes x' straight into the permuted copy (see
// bigmac_layer_forward)
bool descend_scatters(const bigmac_dims& D) {
  if (D.order != BIGMAC_ORDER_DCCA || !bf(D) || route_low(D) || (D.flags & BIGMAC_FLAG_NO_FUSED_DISPATCH)) return false;
  if (forward_ksplit(D, D.T, D.r, D.d) != 1) return false;
  return (size_t)D.T * D.k * (size_t)D.r * 2 < (1ull << 31) && (size_t)D.T * D.k * 4 < (1ull << 31);
}
// forward-only call: the expert-up product reads its rows through src_of (see bigmac_layer_forward);
// the rows behind the index must lie within one 32-bit byte offset
bool expert_up_gathers(const bigmac_dims& D) {
  return bf(D) && !(D.flags & BIGMAC_FLAG_NO_FUSED_DISPATCH) && (size_t)D.T * (size_t)widths(D).win * 2 < (1ull << 31);
}
}  // namespace

int bigmac_dispatch_folding(const bigmac_dims* D, int training) {
  const int rc = check_dims(D);
  if (rc) return rc;
  if (training) return descend_scatters(*D) ? 2 : 0;
  return expert_up_gathers(*D) ? 1 : 0;
}

const char* bigmac_stage_name(int stage) {
  static const char* names[BIGMAC_STAGE_COUNT] = {
      "router_logits", "topk_gate", "descend", "permutation", "dispatch", "expert_up", "expert_down", "combine", "ascend",
      "bwd_ascend_dgrad", "bwd_ascend_wgrad", "bwd_combine", "bwd_down_dgrad", "bwd_down_wgrad", "bwd_up_wgrad",
      "bwd_up_dgrad", "bwd_dispatch", "bwd_gate", "bwd_router_wgrad", "bwd_descend_wgrad", "bwd_descend_dgrad",
      "bwd_output_cast"};
  return stage >= 0 && stage < BIGMAC_STAGE_COUNT ? names[stage] : "?";
}

int bigmac_saved_layout(const bigmac_dims* D, size_t* off_topk_idx, size_t* off_topk_w, size_t* off_expert_offsets,
                        size_t* off_slot_of) {
  int rc = check_dims(D);
  if (rc) return rc;
  const SavedPlan p = plan_saved(*D);
  if (off_topk_idx) *off_topk_idx = p.topk_idx;
  if (off_topk_w) *off_topk_w = p.topk_w;
  if (off_expert_offsets) *off_expert_offsets = p.offsets;
  if (off_slot_of) *off_slot_of = p.slot_of;
  return BIGMAC_OK;
}

int bigmac_saved_aux_layout(const bigmac_dims* D, size_t* off_aux_loss, size_t* off_aux_share) {
  int rc = check_dims(D);
  if (rc) return rc;
  if (!(D->aux_alpha > 0.0f)) return BIGMAC_ERR_INVALID_ARG;
  const SavedPlan p = plan_saved(*D);
  if (off_aux_loss) *off_aux_loss = p.aux;
  if (off_aux_share) *off_aux_share = p.aux + 256;
  return BIGMAC_OK;
}

int bigmac_aux_loss(const bigmac_dims* D, const float* logits, const int32_t* topk_idx, float* loss, float* share,
                    float* dlogits, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_dims(D);
  if (rc) return rc;
  if (!logits || !topk_idx || !loss || !share || !ws) return BIGMAC_ERR_INVALID_ARG;
  if (ws_bytes < aux_loss_ws_bytes(*D)) return BIGMAC_ERR_WORKSPACE;
  return launch_aux_loss(*D, logits, topk_idx, share, loss, dlogits, ws, (hipStream_t)stream);
}

int bigmac_route(const bigmac_dims* D, const void* x, const float* w_gate, const float* gate_bias, int32_t* topk_idx,
                 float* topk_w, float* logits_out, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_dims(D);
  if (rc) return rc;
  if (!x || !w_gate || !topk_idx || !topk_w) return BIGMAC_ERR_INVALID_ARG;
  float* logits = logits_out;
  if (!logits) {
    if (!ws) return BIGMAC_ERR_INVALID_ARG;
    if (ws_bytes < bigmac_workspace_bytes(D, BIGMAC_WS_ROUTE)) return BIGMAC_ERR_WORKSPACE;
    logits = (float*)ws;
  }
  rc = launch_router_logits(*D, x, w_gate, gate_bias, logits, (hipStream_t)stream);
  if (rc) return rc;
  return launch_topk_gate(*D, logits, topk_idx, topk_w, (hipStream_t)stream);
}

int bigmac_dispatch(const bigmac_dims* D, const void* x_low, const int32_t* topk_idx, void* x_perm, int32_t* expert_offsets,
                    int32_t* slot_of, int32_t* src_of, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_dims(D);
  if (rc) return rc;
  if (!topk_idx || !expert_offsets || !slot_of || !src_of || !ws) return BIGMAC_ERR_INVALID_ARG;
  if ((x_low == nullptr) != (x_perm == nullptr)) return BIGMAC_ERR_INVALID_ARG;
  if (ws_bytes < bigmac_workspace_bytes(D, BIGMAC_WS_DISPATCH)) return BIGMAC_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  rc = launch_build_permutation(D->T, D->k, D->N, D->capacity, topk_idx, expert_offsets, slot_of, src_of, ws, s);
  if (rc || !x_low) return rc;
  return launch_dispatch_rows(D->dtype, D->T, D->k, widths(*D).win, x_low, slot_of, x_perm, s);
}

int bigmac_grouped_ffn(const bigmac_dims* D, const void* x_perm, const int32_t* expert_offsets, const void* w1, const void* w2,
                       const void* b1, const void* b2, void* act_saved, void* o_perm, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_dims(D);
  if (rc) return rc;
  if (!x_perm || !expert_offsets || !w1 || !w2 || !o_perm || !ws) return BIGMAC_ERR_INVALID_ARG;
  if (ws_bytes < ffn_ws_bytes(*D)) return BIGMAC_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const Widths W = widths(*D);
  const size_t Tk = (size_t)D->T * D->k;
  void* hact = ws;
  int* tile_map = (int*)((char*)ws + align_up(Tk * W.hid * esize(D->dtype)));
  int* tile_map_tall = (int*)((char*)tile_map + align_up(tile_map_ints((int)Tk, D->N, gemm_ragged_tile_rows(D->dtype, 0)) * 4));
  ClaimScope claims((char*)tile_map_tall + align_up(tile_map_ints((int)Tk, D->N, gemm_ragged_tile_rows(D->dtype, 0)) * 4), s);
  if (claims.status) return claims.status;
  rc = launch_build_tile_map(expert_offsets, D->N, gemm_ragged_tile_rows(D->dtype, 0), tile_map, s);
  if (!rc && any_tall_rows(*D)) rc = launch_build_tile_map(expert_offsets, D->N, gemm_ragged_tile_rows(D->dtype, 1), tile_map_tall, s);
  if (rc) return rc;
  return run_experts_forward(*D, x_perm, expert_offsets, tile_map, tile_map_tall, w1, w2, b1, b2, act_saved, hact, W.hid, o_perm, 0, s);
}

int bigmac_combine(const bigmac_dims* D, const void* o_perm, const int32_t* slot_of, const float* topk_w, float* y_low, void* stream) {
  int rc = check_dims(D);
  if (rc) return rc;
  if (!o_perm || !slot_of || !y_low) return BIGMAC_ERR_INVALID_ARG;
  return launch_combine_rows(D->dtype, D->T, D->k, widths(*D).win, o_perm, slot_of, topk_w, y_low, COMBINE_F32, (hipStream_t)stream);
}

int bigmac_layer_forward(const bigmac_dims* D, const bigmac_params* P, const void* x, void* y, void* saved, void* ws,
                         size_t ws_bytes, void* stream) {
  int rc = check_dims(D);
  if (rc) return rc;
  const bool dcca = D->order == BIGMAC_ORDER_DCCA;
  if (!P || !x || !y || !ws || !P->w_gate || !P->w1 || !P->w2) return BIGMAC_ERR_INVALID_ARG;
  if (dcca && (!P->w_down || !P->w_up)) return BIGMAC_ERR_INVALID_ARG;
  if (ws_bytes < bigmac_workspace_bytes(D, saved ? BIGMAC_WS_LAYER_TRAIN : BIGMAC_WS_LAYER_FORWARD)) return BIGMAC_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const Widths W = widths(*D);
  const FwdPlan F = plan_fwd(*D);
  const SavedPlan S = plan_saved(*D);
  char* wsb = (char*)ws;
  char* sv = saved ? (char*)saved : wsb + F.total;  // inference keeps the same pieces in the workspace
  ClaimScope claims(wsb + F.claims, s);
  if (claims.status) return claims.status;
  int32_t* topk_idx = (int32_t*)(sv + S.topk_idx);
  float* topk_w = (float*)(sv + S.topk_w);
  int32_t* offsets = (int32_t*)(sv + S.offsets);
  int32_t* slot_of = (int32_t*)(sv + S.slot_of);
  int32_t* src_of = (int32_t*)(sv + S.src_of);
  int* tile_map = (int*)(sv + S.tile_map);
  int* tile_map_tall = (int*)(sv + S.tile_map_tall);
  void* x_perm = sv + S.x_perm;
  void* act = saved ? sv + S.act : nullptr;
  void* hact = sv + S.hact;
  void* o_perm = sv + S.o_perm;
  void* y_low = sv + S.y_low;
  const bool out_bf16 = bf(*D) && (D->flags & BIGMAC_FLAG_OUT_BF16);
  const bool aux = D->aux_alpha > 0.0f;                       // the loss lives in the saved block
  float* logits = aux ? (float*)(sv + S.logits) : (float*)(wsb + F.logits);

  const bool low_router = route_low(*D);
  // x' is the workspace's piece, or (router on x': the backward pass reads it again) the saved block's
  void* x_low_buf = (low_router && saved) ? (void*)(sv + S.x_low) : (void*)(wsb + F.x_low);
  auto route = [&](const void* router_in) -> int {
    const bigmac_dims R = router_dims(*D);
    int rr;
    {
      BIGMAC_STAGE(BIGMAC_STAGE_ROUTER_LOGITS);
      rr = launch_router_logits(R, router_in, P->w_gate, P->gate_bias, logits, s);
    }
    if (rr) return rr;
    BIGMAC_STAGE(BIGMAC_STAGE_TOPK_GATE);
    rr = launch_topk_gate(*D, logits, topk_idx, topk_w, s);
    if (!rr && aux)
      rr = launch_aux_loss(*D, logits, topk_idx, (float*)(sv + S.aux + 256), (float*)(sv + S.aux), nullptr, wsb + F.aux, s);
    return rr;
  };
  if (!low_router) {   // Section 3.1's default: the router reads the full-width token
    rc = route(x);
    if (rc) return rc;
  }
  auto permute = [&]() -> int {
    BIGMAC_STAGE(BIGMAC_STAGE_PERMUTATION);
    TileMapJobs maps = {};
    maps.tile_rows[0] = gemm_ragged_tile_rows(D->dtype, 0); maps.map[0] = tile_map;
    if (any_tall_rows(*D)) { maps.tile_rows[1] = gemm_ragged_tile_rows(D->dtype, 1); maps.map[1] = tile_map_tall; }
    return launch_build_permutation(D->T, D->k, D->N, D->capacity, topk_idx, offsets, slot_of, src_of, wsb + F.perm, s, &maps);
  };
  // A training forward on bf16 storage whose router reads x folds the dispatch into the descending
  // projection: the permutation is built first, and the product's epilogue writes every token's
  // narrow row straight into the places of its pairs in the permuted copy (x' itself is not
  // stored: nothing else reads it).  Not where the product is summed from K slices, nor where the
  // copy is too large for one 32-bit byte offset.
  const int descend_ksplit = dcca ? forward_ksplit(*D, D->T, D->r, D->d) : 1;
  const bool descend_tall = dcca && descend_ksplit == 1 && tall_dense(*D, D->T, D->r, D->d);
  const bool descend_deep = dcca && descend_ksplit == 1 && !descend_tall && deep_dense(*D, D->T, D->r, D->d);
  const bool scatter_descend = saved && descend_scatters(*D);
  if (scatter_descend) {
    rc = permute();
    if (rc) return rc;
  }
  const void* x_low = x;
  if (dcca) {  // x' = x W_down
    GemmDesc g = base_desc(*D);
    g.a_kcontig = 1; g.b_kcontig = 0; g.epilogue = EPI_STORE; g.out_f32 = bf(*D) ? 0 : 1;
    g.A = x; g.lda = D->d; g.M = D->T; g.K = D->d;
    g.B = P->w_down; g.ldb = D->r; g.N = D->r;
    g.C = x_low_buf; g.ldc = D->r;
    {
      BIGMAC_STAGE(BIGMAC_STAGE_DESCEND);
      g.ksplit = descend_ksplit;
      g.tall_tile = descend_tall;
      g.deep_tile = descend_deep;
      if (scatter_descend) {
        g.scatter = slot_of; g.scatter_k = D->k; g.scatter_rows = D->T * D->k;
        g.C = x_perm;
      }
      if (g.tall_tile) { g.tall_tile = 0; g.long_tile = 1; }   // k-contiguous A, whole-line B: the tall tile on its side (see launch_mfma_long)
      if (g.ksplit > 1) {   // fp32 partials, then one rounding to bf16
        g.out_f32 = 1; g.C = wsb + F.partials; g.gstride_c = (long)D->T * D->r;
        rc = launch_gemm(g, s);
        if (rc) return rc;
        rc = launch_reduce_partials_bf16((const float*)(wsb + F.partials), g.ksplit, (size_t)D->T * D->r, x_low_buf, s);
      } else {
        rc = launch_gemm(g, s);
      }
    }
    if (rc) return rc;
    x_low = x_low_buf;
  }
  if (low_router) {    // the alternative Section 3.1 names: the router reads x' (as stored)
    rc = route(x_low);
    if (rc) return rc;
  }
  if (!scatter_descend) {
    rc = permute();
    if (rc) return rc;
  }
  // Forward-only calls on bf16 storage fold the dispatch into the expert-up product: its A rows are
  // read from x' (or x) through src_of and no permuted copy is written.  A training forward
  // keeps the copy: the backward pass contracts over its rows.
  const bool fuse_dispatch = !saved && expert_up_gathers(*D);
  if (!fuse_dispatch && !scatter_descend) {
    BIGMAC_STAGE(BIGMAC_STAGE_DISPATCH);
    rc = launch_dispatch_rows(D->dtype, D->T, D->k, W.win, x_low, slot_of, x_perm, s);
  }
  if (rc) return rc;
  rc = run_experts_forward(*D, fuse_dispatch ? x_low : x_perm, offsets, tile_map, tile_map_tall, P->w1, P->w2, P->b1, P->b2, act, hact, wide_ld(*D), o_perm,
                           wire_f32(*D) ? 1 : 0, s, fuse_dispatch ? src_of : nullptr);
  if (rc) return rc;
  if (!dcca) {  // fine-grained layer: the weighted sum is the output
    BIGMAC_STAGE(BIGMAC_STAGE_COMBINE);
    return launch_combine_rows(wire_dtype(*D), D->T, D->k, W.win, o_perm, slot_of, topk_w, y, COMBINE_F32, s);
  }
  {
    BIGMAC_STAGE(BIGMAC_STAGE_COMBINE);
    rc = launch_combine_rows(wire_dtype(*D), D->T, D->k, W.win, o_perm, slot_of, topk_w, y_low, bf(*D) ? COMBINE_SPLIT_BF16 : COMBINE_F32, s);
  }
  if (rc) return rc;
  {  // y = y' W_up
    GemmDesc g = base_desc(*D);
    g.a_kcontig = 1; g.b_kcontig = 0; g.epilogue = EPI_STORE; g.out_f32 = out_bf16 ? 0 : 1;
    g.A = y_low; g.lda = low_ld(*D); g.M = D->T; g.K = low_ld(*D);
    g.B = P->w_up; g.ldb = D->d; g.N = D->d; g.kwrap_b = bf(*D) ? D->r : 0;
    g.C = y; g.ldc = D->d;
    BIGMAC_STAGE(BIGMAC_STAGE_ASCEND);
    g.ksplit = forward_ksplit(*D, D->T, D->d, low_ld(*D));
    g.tall_tile = g.ksplit == 1 && tall_dense(*D, D->T, D->d, low_ld(*D));
    g.wide_k = g.ksplit == 1 && !g.tall_tile && wide_k_ok(*D, low_ld(*D), 32);
    if (g.tall_tile) { g.tall_tile = 0; g.long_tile = 1; }     // as for the descending projection
    if (g.ksplit > 1) {
      g.out_f32 = 1; g.C = wsb + F.partials; g.gstride_c = (long)D->T * D->d;
      rc = launch_gemm(g, s);
      if (rc) return rc;
      if (out_bf16) rc = launch_reduce_partials_bf16((const float*)(wsb + F.partials), g.ksplit, (size_t)D->T * D->d, y, s);
      else rc = launch_reduce_partials((const float*)(wsb + F.partials), g.ksplit, (size_t)D->T * D->d, (float*)y, 0, s);
    } else {
      rc = launch_gemm(g, s);
    }
  }
  return rc;
}

int bigmac_layer_backward(const bigmac_dims* D, const bigmac_params* P, const void* x, const void* dy, const void* saved,
                          void* dx, float* d_w_down, float* d_w_up, float* d_w_gate, float* d_w1, float* d_w2, float* d_b1,
                          float* d_b2, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_dims(D);
  if (rc) return rc;
  const bool dcca = D->order == BIGMAC_ORDER_DCCA;
  if (!P || !x || !dy || !saved || !dx || !ws || !d_w_gate || !d_w1 || !d_w2 || !P->w_gate || !P->w1 || !P->w2)
    return BIGMAC_ERR_INVALID_ARG;
  if (dcca && (!P->w_down || !P->w_up || !d_w_down || !d_w_up)) return BIGMAC_ERR_INVALID_ARG;
  if ((P->b1 != nullptr) != (d_b1 != nullptr) || (P->b2 != nullptr) != (d_b2 != nullptr)) return BIGMAC_ERR_INVALID_ARG;
  if (bf(*D) && D->N % 8) return BIGMAC_ERR_UNSUPPORTED;  // the dense logit gradient has 16-byte rows
  if (ws_bytes < bigmac_workspace_bytes(D, BIGMAC_WS_LAYER_TRAIN)) return BIGMAC_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const Widths W = widths(*D);
  const SavedPlan S = plan_saved(*D);
  const BwdPlan B = plan_bwd(*D);
  const char* sv = (const char*)saved;
  char* wsb = (char*)ws;
  ClaimScope claims(wsb + B.claims, s);
  if (claims.status) return claims.status;
  const int32_t* topk_idx = (const int32_t*)(sv + S.topk_idx);
  const float* topk_w = (const float*)(sv + S.topk_w);
  const int32_t* offsets = (const int32_t*)(sv + S.offsets);
  const int32_t* slot_of = (const int32_t*)(sv + S.slot_of);
  const int* tile_map = (const int*)(sv + S.tile_map);
  const int* tile_map_tall = (const int*)(sv + S.tile_map_tall);
  const void* x_perm = sv + S.x_perm;
  const void* act = sv + S.act;
  const void* hact = sv + S.hact;
  const void* o_perm = sv + S.o_perm;
  const void* y_low = sv + S.y_low;
  float* dy_low = (float*)(wsb + B.dy_low);
  float* dgate = (float*)(wsb + B.dgate);
  void* do_perm = wsb + B.do_perm;
  void* dact = wsb + B.dact;
  void* dx_perm = wsb + B.dx_perm;
  void* dx_low = wsb + B.dx_low;
  void* dL = wsb + B.dL;
  ReduceJob jobs[3];
  int njobs = 0;
  const bool out_bf16 = bf(*D) && (D->flags & BIGMAC_FLAG_OUT_BF16);
  float* dx_f32 = out_bf16 ? (float*)(wsb + B.dx_f32) : (float*)dx;
  const int accumulate = (D->flags & BIGMAC_FLAG_ACCUMULATE) ? 1 : 0;
  const int Tk = D->T * D->k;
  const size_t Td = (size_t)D->T * D->d;

  if (dcca) {
    // dy' = dy W_up^T (kept in fp32)
    GemmDesc g = base_desc(*D);
    g.a_kcontig = 1; g.b_kcontig = 1; g.epilogue = EPI_STORE; g.out_f32 = 1;
    g.A = dy; g.lda = D->d; g.M = D->T; g.K = D->d;
    g.B = P->w_up; g.ldb = D->d; g.N = D->r;
    g.C = dy_low; g.ldc = D->r;
    g.tall_tile = tall_dense(*D, D->T, D->r, D->d);
    g.deep_tile = !g.tall_tile && deep_dense(*D, D->T, D->r, D->d);
    {
      BIGMAC_STAGE(BIGMAC_STAGE_BWD_ASCEND_DGRAD);
      if (transposed_projections(*D)) {   // W_up^T [d, r]: B with the output index fast
        hipLaunchKernelGGL(transpose_b16_kernel, dim3((D->d + 63) / 64, (D->r + 63) / 64), dim3(256), 0, s, (const uint16_t*)P->w_up,
                           (uint16_t*)(wsb + B.w_up_t), D->r, D->d);
        BIGMAC_CHECK_LAUNCH();
        g.B = wsb + B.w_up_t; g.ldb = D->r; g.b_kcontig = 0;
        g.tall_tile = 0; g.long_tile = 1;
      }
      rc = launch_gemm(g, s);
    }
    if (rc) return rc;
    // dW_up (+)= y'^T dy
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_ASCEND_WGRAD);
    rc = run_token_wgrad(*D, y_low, low_ld(*D), D->r, dy, D->d, D->d, d_w_up, (float*)(wsb + B.part_up), &jobs[njobs++], s);
    if (rc) return rc;
  } else {
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_ASCEND_DGRAD);
    if (bf(*D)) hipLaunchKernelGGL(to_f32_kernel<bf16_t>, grid1d(Td), dim3(256), 0, s, (const bf16_t*)dy, dy_low, Td);
    else hipLaunchKernelGGL(to_f32_kernel<float>, grid1d(Td), dim3(256), 0, s, (const float*)dy, dy_low, Td);
    BIGMAC_CHECK_LAUNCH();
  }
  // weighted-sum backward: gate gradients and the scaled scatter of dy' to the expert rows
  {
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_COMBINE);
    rc = launch_combine_backward(D->dtype, wire_dtype(*D), D->T, D->k, W.win, dy_low, o_perm, slot_of, topk_w, dgate, do_perm, s);
  }
  if (rc) return rc;
  if (d_b2) {  // the second bias adds to every expert output: its gradient is the column sum of do_perm over the expert's rows
    rc = launch_ragged_colsum(D->dtype, do_perm, W.win, W.win, offsets, D->N, d_b2, accumulate, wsb + B.bias_sums, s);
    if (rc) return rc;
  }
  {  // dact = (do_perm W2[e]^T) * act'(act)
    GemmDesc g = base_desc(*D);
    g.mode = GEMM_RAGGED_M; g.groups = D->N; g.max_rows = Tk; g.offsets = offsets; g.tile_map = tile_map;
    g.a_kcontig = 1; g.b_kcontig = 1; g.epilogue = EPI_DGELU;
    g.A = do_perm; g.lda = W.win; g.K = W.win;
    g.B = P->w2; g.ldb = W.win; g.gstride_b = (long)W.hid * W.win; g.N = W.hid;
    g.C = dact; g.ldc = wide_ld(*D); g.aux_in = act;
    g.big_tile = big_rows(*D, W.hid, W.win);
    g.tall_tile = !g.big_tile && tall_rows(*D, W.hid, W.win); g.tile_map = (g.tall_tile || g.big_tile) ? tile_map_tall : tile_map;
    g.wide_k = !g.tall_tile && !g.big_tile && wide_k_ok(*D, W.win, 4);
    // with 64-deep k tiles the 256 x 256 tile pays for this product from K = 1024 on (zipf_stress: 1.423 -> 1.404 ms)
    if (g.tall_tile && W.win >= 1024 && W.win % 64 == 0 && W.hid % 256 == 0 && !(D->flags & BIGMAC_FLAG_TILES_SMALL)) { g.tall_tile = 0; g.big_tile = 1; }
    g.kloop_priority = 1;              // measured: -3.5 % (gpt_medium), -1.7 % (gpt_xl)
    if (!g.big_tile) touch_weights(*D, g, P->w2, 4);
    {
      BIGMAC_STAGE(BIGMAC_STAGE_BWD_DOWN_DGRAD);
      rc = launch_gemm(g, s);
    }
    if (rc) return rc;
    if (d_b1) {  // the first bias adds to the pre-activation: column sums of dact
      rc = launch_ragged_colsum(D->dtype, dact, wide_ld(*D), W.hid, offsets, D->N, d_b1, accumulate, wsb + B.bias_sums, s);
      if (rc) return rc;
    }
  }
  {  // dW2[e] (+)= hact_e^T do_perm_e
    GemmDesc g = base_desc(*D);
    g.mode = GEMM_RAGGED_K; g.groups = D->N; g.max_rows = Tk; g.offsets = offsets; g.tile_map = tile_map;
    g.a_kcontig = 0; g.b_kcontig = 0; g.epilogue = EPI_ACCUM; g.beta = accumulate;
    g.A = hact; g.lda = wide_ld(*D); g.M = W.hid;
    g.B = do_perm; g.ldb = W.win; g.N = W.win;
    g.C = d_w2; g.ldc = W.win; g.gstride_c = (long)W.hid * W.win;
    g.big_tile = big_wgrad(*D);
    g.tall_tile = !g.big_tile && tall_wgrad(*D, W.hid);
    {
      BIGMAC_STAGE(BIGMAC_STAGE_BWD_DOWN_WGRAD);
      rc = launch_gemm(g, s);
    }
    if (rc) return rc;
    // dW1[e] (+)= x_perm_e^T dact_e
    g.A = x_perm; g.lda = W.win; g.M = W.win;
    g.B = dact; g.ldb = wide_ld(*D); g.N = W.hid;
    g.C = d_w1; g.ldc = W.hid; g.gstride_c = (long)W.win * W.hid;
    g.big_tile = big_wgrad(*D);
    g.tall_tile = !g.big_tile && tall_wgrad(*D, W.win);
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_UP_WGRAD);
    rc = launch_gemm(g, s);
    if (rc) return rc;
  }
  {  // dx_perm = dact W1[e]^T
    GemmDesc g = base_desc(*D);
    g.mode = GEMM_RAGGED_M; g.groups = D->N; g.max_rows = Tk; g.offsets = offsets; g.tile_map = tile_map;
    g.a_kcontig = 1; g.b_kcontig = 1; g.epilogue = EPI_STORE; g.out_f32 = (bf(*D) && !wire_f32(*D)) ? 0 : 1;
    g.A = dact; g.lda = wide_ld(*D); g.K = W.hid;
    g.B = P->w1; g.ldb = W.hid; g.gstride_b = (long)W.win * W.hid; g.N = W.win;
    g.C = dx_perm; g.ldc = W.win;
    g.big_tile = big_rows(*D, W.win, W.hid);
    g.tall_tile = !g.big_tile && tall_rows(*D, W.win, W.hid); g.tile_map = (g.tall_tile || g.big_tile) ? tile_map_tall : tile_map;
      g.wide_k = !g.tall_tile && !g.big_tile && wide_k_ok(*D, W.hid, 8);
    g.kloop_priority = 1;
    if (!g.big_tile) touch_weights(*D, g, P->w1, 8);
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_UP_DGRAD);
    rc = launch_gemm(g, s);
    if (rc) return rc;
  }
  // Gate backward.  The router's share of the input gradient goes to dx (router on x) or, with the
  // router on x', into an fp32 [T, r] row that the sum of dx' below starts from.
  const bool low_router = route_low(*D);
  const bigmac_dims R = router_dims(*D);
  float* gate_low = low_router ? (float*)(wsb + B.gate_low) : nullptr;
  {
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_GATE);
    const bool aux = D->aux_alpha > 0.0f;
    rc = launch_route_backward(R, P->w_gate, topk_idx, topk_w, dgate, aux ? (const float*)(sv + S.logits) : nullptr,
                               aux ? (const float*)(sv + S.aux + 256) : nullptr, low_router ? gate_low : dx_f32, dL, wsb + B.route, s);
  }
  if (rc) return rc;
  // dispatch backward: dx' = sum_j dx_perm[slot_of[t, j]] (+ the router's share)
  {
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_DISPATCH);
    rc = launch_combine_rows(wire_dtype(*D), D->T, D->k, W.win, dx_perm, slot_of, nullptr, dx_low,
                             (dcca && bf(*D)) ? COMBINE_SPLIT_BF16 : COMBINE_F32, s, gate_low,
                             /*stream_out=*/low_bytes(*D) >= (32u << 20));   // (smaller results are read back from the caches)
  }
  if (rc) return rc;
  {  // dW_g (+)= x^T dL  (router on x': x'^T dL)
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_ROUTER_WGRAD);
    const void* router_in = low_router ? (const void*)(sv + S.x_low) : x;
    rc = run_token_wgrad(*D, router_in, R.d, R.d, dL, D->N, D->N, d_w_gate, (float*)(wsb + B.part_gate), &jobs[njobs++], s);
  }
  if (rc) return rc;
  if (dcca) {
    {  // dx += dx' W_down^T
      GemmDesc g = base_desc(*D);
      g.a_kcontig = 1; g.b_kcontig = 1; g.epilogue = EPI_ACCUM; g.beta = low_router ? 0 : 1;   // dx holds the router's share, or nothing yet
      g.A = dx_low; g.lda = low_ld(*D); g.M = D->T; g.K = low_ld(*D);
      g.B = P->w_down; g.ldb = D->r; g.N = D->d; g.kwrap_b = bf(*D) ? D->r : 0;
      g.C = dx_f32; g.ldc = D->d;
      g.tall_tile = tall_dense(*D, D->T, D->d, low_ld(*D));
      g.wide_k = !g.tall_tile && wide_k_ok(*D, low_ld(*D), 16);
      BIGMAC_STAGE(BIGMAC_STAGE_BWD_DESCEND_DGRAD);
      if (transposed_projections(*D)) {   // W_down^T [r, d]
        hipLaunchKernelGGL(transpose_b16_kernel, dim3((D->r + 63) / 64, (D->d + 63) / 64), dim3(256), 0, s, (const uint16_t*)P->w_down,
                           (uint16_t*)(wsb + B.w_down_t), D->d, D->r);
        BIGMAC_CHECK_LAUNCH();
        g.B = wsb + B.w_down_t; g.ldb = D->d; g.b_kcontig = 0;
        g.tall_tile = 0; g.long_tile = 1;
      }
      rc = launch_gemm(g, s);
      if (rc) return rc;
    }
    // dW_down (+)= x^T dx', and the reduction of all three token-index weight gradients
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_DESCEND_WGRAD);
    rc = run_token_wgrad(*D, x, D->d, D->d, dx_low, low_ld(*D), D->r, d_w_down, (float*)(wsb + B.part_down), &jobs[njobs++], s);
    if (rc) return rc;
    rc = launch_reduce_partials_multi(jobs, njobs, (D->flags & BIGMAC_FLAG_ACCUMULATE) ? 1 : 0, s);
    if (rc) return rc;
  } else {
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_OUTPUT_CAST);
    hipLaunchKernelGGL(add_f32_kernel, grid1d(Td), dim3(256), 0, s, dx_f32, (const float*)dx_low, Td);
    BIGMAC_CHECK_LAUNCH();
    rc = launch_reduce_partials_multi(jobs, njobs, (D->flags & BIGMAC_FLAG_ACCUMULATE) ? 1 : 0, s);
    if (rc) return rc;
  }
  if (out_bf16) {
    BIGMAC_STAGE(BIGMAC_STAGE_BWD_OUTPUT_CAST);
    hipLaunchKernelGGL(f32_to_bf16_kernel, grid1d(Td), dim3(256), 0, s, dx_f32, (bf16_t*)dx, Td);
    BIGMAC_CHECK_LAUNCH();
  }
  return BIGMAC_OK;
}

}  // extern "C"
