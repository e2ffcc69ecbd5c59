// Internal declarations shared by the translation units of libbigmac (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/bigmac.h"

namespace bigmac {

typedef uint16_t bf16_t;  // bfloat16 bit pattern in memory

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
// round to nearest even (the hardware conversion of gfx950)
__device__ __forceinline__ uint32_t f2bf_pair(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)(f2bf_pair(f, 0.0f) & 0xFFFFu); }
__device__ __forceinline__ void unpack_bf16x8(const uint4& v, float* f) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}
__device__ __forceinline__ uint4 pack_bf16x8(const float* f) {
  uint4 v;
  v.x = f2bf_pair(f[0], f[1]);
  v.y = f2bf_pair(f[2], f[3]);
  v.z = f2bf_pair(f[4], f[5]);
  v.w = f2bf_pair(f[6], f[7]);
  return v;
}

// Exact (erf) GELU  0.5 a (1 + erf(a / sqrt 2)) = a Phi(a)  and its derivative Phi(a) + a pdf(a).
// The upper tail 1 - Phi(|a|) = 0.5 erfc(|a| / sqrt 2) is evaluated as exp2(P(|a|)), P a degree-8
// least-squares Chebyshev fit of log2 of the tail on [0, 5.5] (beyond 5.5 the tail is < 2e-8 and
// |a| is clamped); absolute error of the tail < 1.3e-6, of the GELU < 4e-7 (checked against
// scipy's erfc in fp64 with the polynomial evaluated in fp32).
__device__ __forceinline__ float normal_upper_tail(float a) {
  const float x = __builtin_amdgcn_fmed3f(fabsf(a), 0.0f, 5.5f);   // min(|a|, 5.5) in one instruction
  float q = fmaf(x, -9.896420991e-08f, 2.559779935e-07f);
  q = fmaf(x, q, 4.382965935e-05f);
  q = fmaf(x, q, -8.528624129e-04f);
  q = fmaf(x, q, 8.322801297e-03f);
  q = fmaf(x, q, -5.372542357e-02f);
  q = fmaf(x, q, -4.586065007e-01f);
  q = fmaf(x, q, -1.151219477e+00f);
  q = fmaf(x, q, -9.999963850e-01f);
  return __builtin_amdgcn_exp2f(q);
}
__device__ __forceinline__ float gelu_f(float a) {   // max(a, 0) - |a| tail(|a|)
  float relu;   // one v_max: fmaxf() would first quiet a possible signalling NaN with a second one
  asm("v_max_f32 %0, 0, %1" : "=v"(relu) : "v"(a));
  return fmaf(-fabsf(a), normal_upper_tail(a), relu);
}
__device__ __forceinline__ float gelu_grad_f(float a) {
  const float cdf = 0.5f + copysignf(0.5f - normal_upper_tail(a), a);
  const float pdf = __builtin_amdgcn_exp2f(fmaf(a * a, -0.72134752044448170f, -1.32574806473616f));  // exp(-a^2/2) / sqrt(2 pi)
  return fmaf(a, pdf, cdf);
}

// For bf16 results a degree-6 fit of the same tail is enough: relative error of the tail below
// 3e-5 (so of the GELU too, on both signs), two orders below the rounding of the bf16 result.
__device__ __forceinline__ float gelu_bf16_f(float a) {
  const float x = __builtin_amdgcn_fmed3f(fabsf(a), 0.0f, 5.5f);
  float q = fmaf(x, 2.630473060e-05f, -6.637311158e-04f);
  q = fmaf(x, q, 7.507435764e-03f);
  q = fmaf(x, q, -5.203327266e-02f);
  q = fmaf(x, q, -4.602325443e-01f);
  q = fmaf(x, q, -1.150642133e+00f);
  q = fmaf(x, q, -1.000029561e+00f);
  float relu;
  asm("v_max_f32 %0, 0, %1" : "=v"(relu) : "v"(a));
  return fmaf(-fabsf(a), __builtin_amdgcn_exp2f(q), relu);
}
// The derivative for bf16 results, cheaper: with x = |a|, pdf(x) the normal density and
// R(x) = (1 - Phi(x)) / pdf(x) the Mills ratio,  gelu'(a) = 0.5 + sign(a) (0.5 + pdf(x) (x - R(x))).
// x - R(x) is smooth and its error is weighted by pdf(x), so a degree-6 polynomial (pdf-weighted
// least squares on [0, 5.5], |a| clamped there) keeps the absolute error of gelu' below 4e-5
// (checked against scipy's erfc in fp64 with the evaluation in fp32): two orders below the
// rounding of the bf16 product it feeds.  One exponential instead of two.
__device__ __forceinline__ float gelu_grad_bf16_f(float a) {
  const float x = __builtin_amdgcn_fmed3f(fabsf(a), 0.0f, 5.5f);
  float q = fmaf(x, -1.015918907e-03f, 1.451199694e-02f);
  q = fmaf(x, q, -8.408022016e-02f);
  q = fmaf(x, q, 2.745896445e-01f);
  q = fmaf(x, q, -6.029496024e-01f);
  q = fmaf(x, q, 1.996360723e+00f);
  q = fmaf(x, q, -1.253221897e+00f);
  const float pdf = __builtin_amdgcn_exp2f(fmaf(x * x, -0.72134752044448170f, -1.32574806473616f));
  return 0.5f + copysignf(fmaf(pdf, q, 0.5f), a);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf2f(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f2bf(v); }
};

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline int esize(int dtype) { return dtype == BIGMAC_BF16 ? 2 : 4; }

struct Widths {
  int win, hid;  // dispatch width and expert hidden width for the given order
};
inline Widths widths(const bigmac_dims& D) {
  return D.order == BIGMAC_ORDER_CDAC ? Widths{D.d, D.r} : Widths{D.r, D.h};
}
int check_dims(const bigmac_dims* D);  // BIGMAC_OK or an error code

// ----------------------------------------------------------------------------- GEMM -----
// C[M,N] (op)= A[M,K] . B[K,N], fp32 accumulate.  "k-contiguous" says which index is the fast
// one in memory: A k-contiguous = A stored [M][K] (lda between rows m), otherwise stored
// [K][M]; B k-contiguous = B stored [N][K], otherwise stored [K][N].
enum GemmMode { GEMM_DENSE = 0, GEMM_RAGGED_M = 1, GEMM_RAGGED_K = 2 };
enum GemmEpilogue {
  EPI_STORE = 0,   // C = acc                                   (C type: out_f32 ? float : dtype)
  EPI_GELU = 1,    // aux_out = acc (pre-activation, optional); C = gelu(acc)        (dtype)
  EPI_DGELU = 2,   // C = acc * gelu'(aux_in)                                        (dtype)
  EPI_ACCUM = 3    // fp32 C = (beta ? C : 0) + acc
};

struct GemmDesc {
  int dtype;                 // BIGMAC_F32 or BIGMAC_BF16: element type of A, B, aux
  int a_kcontig, b_kcontig;
  int mode, epilogue;
  int out_f32;               // EPI_STORE only
  int beta;                  // EPI_ACCUM only
  const void* A;
  const void* B;
  void* C;
  const void* bias;          // EPI_GELU / EPI_STORE, optional: added to every row of the product before the epilogue's own
  long gstride_bias;         //   work ([N] of dtype; ragged-M: one vector per group, gstride_bias elements apart)
  const void* aux_in;        // EPI_DGELU: saved pre-activation, same shape/ld as C
  void* aux_out;             // EPI_GELU: optional pre-activation output, same shape/ld as C
  long lda, ldb, ldc;
  int M, N, K;               // dense: all three.  ragged-M: N, K (rows from offsets).  ragged-K: M, N.
  int groups;                // ragged modes: number of groups (experts)
  int max_rows;              // ragged-M: total rows (upper bound for the tile count)
  const int* offsets;        // device [groups+1]: row ranges (ragged-M) or k ranges (ragged-K)
  const int* tile_map;       // device, from launch_build_tile_map: ragged-M needs it; ragged-K takes its cost-balanced schedule from it (optional)
  long gstride_b;            // ragged-M: elements between the B matrices of consecutive groups
  long gstride_c;            // ragged-K / split-K: elements between consecutive C outputs
  int ksplit;                // dense: number of K slices (each writes C + z*gstride_c); 1 = none
  int kwrap_b;               // B's k index is taken modulo this (0 = off); multiple of 64
  int tall_tile;             // bf16 only: 256-row workgroup tiles (ragged-M: the tile map must be built for them)
  int wide_k;                // bf16, k-contiguous A, K % 64 == 0: the square tile with 64-deep k tiles, two ring stages
  int kloop_priority;        // MFMA kernels: raise the wave priority inside the k loop (see the kernel)
  int deep_tile;             // bf16, dense, store or accumulate (K % 64 == 0 with a k-contiguous operand): 128 x 64 outputs, 64-deep k tiles
  int long_tile;             // bf16, k-contiguous A only; ragged-M with the GELU epilogue or dense with the plain store: 128 x 256 outputs
                             //   (four wavefronts side by side, each 128 x 64); ragged-M: tile map of 128-row tiles
  int big_tile;              // bf16: 256 x 256 outputs by eight wavefronts, one workgroup per CU (ragged-M: tile map of 256-row tiles)
  const int* gather;         // ragged-M MFMA kernels with a k-contiguous A, GELU or store epilogue: row m of the product is row gather[m] / gather_div of A (device [max_rows]); NULL: A holds the rows in order
  int gather_rows, gather_div; //   rows of A behind the index; the index is divided by gather_div first (flat (row, pick) pairs)
  const int* scatter;        // dense bf16 products with a k-contiguous A, B not k-contiguous, plain bf16 store: row m of the product is
                             //   written to the rows scatter[m * scatter_k + j], j < scatter_k, of C (negative: no row); NULL: row m of C
  int scatter_k, scatter_rows; //   copies per row; rows of C behind the index
  unsigned* claim;           // MFMA kernels, optional: zeroed tile counters of this launch (ClaimScope hands them out; see tile order in gemm_core.hpp)
  const void* touch;         // MFMA kernels, optional: a region (device) every line of which is read once as the kernel starts,
  size_t touch_bytes;        //   so that its first use in a k loop meets the caches and not the memory (0 = off)
};
// Tile counters for the MFMA kernels' dynamic tile order: one slot per launch, one counter per XCD
// (64 bytes apart).  An entry point opens a scope over a piece of its workspace; the scope clears
// the piece with a fill kernel on the stream, and every launch_gemm of this thread inside the scope
// takes the next slot (launches beyond the last slot run in the static order).
constexpr int CLAIM_SLOTS = 48, CLAIM_SLOT_INTS = 8 * 16;
constexpr size_t CLAIM_BYTES = (size_t)CLAIM_SLOTS * CLAIM_SLOT_INTS * 4;
struct ClaimScope {
  ClaimScope(void* region, hipStream_t s);
  ~ClaimScope();
  int status;   // BIGMAC_OK, or the fill kernel's launch error
};
// Rows per M tile of the ragged-M schedule for this dtype (the tile map must be built with it).
int gemm_ragged_tile_rows(int dtype, int tall_tile);
int launch_gemm(const GemmDesc& g, hipStream_t s);
// tile_map capacity in int32 for a ragged-M problem: header, the group order of the ragged-K
// schedule (one int per group), then a (group, first row) pair per M tile
inline size_t tile_map_ints(int total_rows, int groups, int tile_rows) {
  return 16 + (size_t)groups + 2 * ((size_t)total_rows / tile_rows + groups + 1);
}
double launch_mfma_probe(int blocks, int iters, float* sink, hipStream_t s);   // returns the flops issued, < 0 on a launch error
int launch_build_tile_map(const int* offsets, int groups, int tile_rows, int* tile_map, hipStream_t s);
// out[i] = (beta ? out[i] : 0) + sum_z part[z*n + i]
int launch_reduce_partials(const float* part, int nslices, size_t n, float* out, int beta, hipStream_t s);
// the same for up to 3 independent reductions in one launch
struct ReduceJob {
  const float* part;
  float* out;
  size_t n;
  int nslices;
};
int launch_reduce_partials_multi(const ReduceJob* jobs, int count, int beta, hipStream_t s);
// out[i] = bf16(sum_z part[z*n + i]); n a multiple of 8
int launch_reduce_partials_bf16(const float* part, int nslices, size_t n, void* out, hipStream_t s);

// ----------------------------------------------------------------------------- route ----
int launch_router_logits(const bigmac_dims& D, const void* x, const float* w_gate, const float* bias,
                         float* logits, hipStream_t s);
int launch_topk_gate(const bigmac_dims& D, const float* logits, int32_t* topk_idx, float* topk_w, hipStream_t s);
// Gate backward (softmax over the k picked logits) and the router's share of dx:
//   dlogit[t,j] = w[t,j] (dgate[t,j] - sum_m w[t,m] dgate[t,m])
//   dL_out [T,N] (storage dtype) = dlogit scattered to its expert columns, zeros elsewhere
//   dx_f32[t,:] = sum_j dlogit[t,j] * w_gate[:, idx[t,j]]      (overwritten)
// ws: route_backward_ws_bytes (a transposed or bf16 copy of w_gate, or the k picked entries of dL per token).
size_t route_backward_ws_bytes(const bigmac_dims& D);
// With logits and share (the load-balance loss is on) the loss's gradient
//   D.aux_alpha N / T * p[t,n] (share[n] - sum_e share[e] p[t,e]),  p = softmax(logits[t,:]),
// is added to every entry of dL_out and takes part in dx_f32.
int launch_route_backward(const bigmac_dims& D, const float* w_gate, const int32_t* topk_idx,
                          const float* topk_w, const float* dgate, const float* logits, const float* share,
                          float* dx_f32, void* dL_out, void* ws, hipStream_t s);
// Load-balance loss  D.aux_alpha N sum_e f_e P_e:  f_e = share of the T k pairs routed to e (before
// any capacity drop), P_e = mean over tokens of softmax(logits)[e].  share [N] and loss [1] are
// written; dlogits ([T,N], may be NULL) receives the gradient with f held fixed.
size_t aux_loss_ws_bytes(const bigmac_dims& D);
int launch_aux_loss(const bigmac_dims& D, const float* logits, const int32_t* topk_idx, float* share, float* loss,
                    float* dlogits, void* ws, hipStream_t s);

// ----------------------------------------------------------------------------- permute --
size_t permutation_ws_bytes(int T, int k, int N);
// tile_maps (optional): tile maps of the expert offsets, built by the same launch that finds them
struct TileMapJobs;
int launch_build_permutation(int T, int k, int N, int capacity, const int32_t* topk_idx, int32_t* expert_offsets,
                             int32_t* slot_of, int32_t* src_of, void* ws, hipStream_t s, const TileMapJobs* tile_maps = nullptr);
int launch_gather_probe(const void* table, const int32_t* order, long rows, long row_bytes, int streaming, unsigned* sink, hipStream_t s);
int launch_dispatch_rows(int dtype, int T, int k, int width, const void* x_low, const int32_t* slot_of,
                         void* x_perm, hipStream_t s);
enum CombineOut { COMBINE_F32 = 0, COMBINE_SPLIT_BF16 = 1 };  // fp32 [T,w]  |  bf16 [T,2w] = (hi | lo)
// dtype: element type of the gathered rows (BIGMAC_F32 or BIGMAC_BF16)
// addend (optional, fp32 [T, width]): the sum of a token starts from its row instead of zero
int launch_combine_rows(int dtype, int T, int k, int width, const void* o_perm, const int32_t* slot_of,
                        const float* topk_w, void* y_low, int out_kind, hipStream_t s, const float* addend = nullptr, int stream_out = 0);
// backward of the weighted combine: dgate[t,j] = <dy_low[t], o_perm[slot]>, do_perm[slot] = w[t,j]*dy_low[t]
// (o_dtype: element type of o_perm; do_perm has the storage type `dtype`)
int launch_combine_backward(int dtype, int o_dtype, int T, int k, int width, const float* dy_low, const void* o_perm,
                            const int32_t* slot_of, const float* topk_w, float* dgate, void* do_perm,
                            hipStream_t s);

// out[g, :] (fp32, [groups, cols]) (+)= sum over the rows of group g (offsets [groups + 1]) of src[row, :cols]
size_t ragged_colsum_ws_bytes(int groups, int cols);
int launch_ragged_colsum(int dtype, const void* src, long ld, int cols, const int32_t* offsets, int groups, float* out, int beta,
                         void* ws, hipStream_t s);

#define BIGMAC_CHECK_LAUNCH()                                   \
  do {                                                          \
    if (hipGetLastError() != hipSuccess) return BIGMAC_ERR_HIP; \
  } while (0)

}  // namespace bigmac
