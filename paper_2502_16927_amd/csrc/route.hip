// Gating of the BigMac layer (Section 3.1: the router reads the full-width token x; T is the
// set of top_k experts, p_i the gate value).  The logits decide integers, so their fp32
// summation order is fixed and every product is a fused multiply-add:
//   p_l  = fma(x[t, 64q + l], W_g[64q + l, n], p_l),  q ascending, l = 0..63   (one lane each)
//   tree = p_l + p_{l+off} for off = 32, 16, 8, 4, 2, 1;  logit = tree (+ bias[n], added last)
// The tree is evaluated as a reduce-scatter over the wavefront: same pairs, 1/6 of the adds.
#include "common.hpp"

namespace bigmac {

namespace {

#ifndef ROUTER_TB_LARGE
#define ROUTER_TB_LARGE 8   // tokens per wavefront of the pipelined router kernel when there are plenty of tokens
#endif
#ifndef ROUTER_TILE_BLOCKS
#define ROUTER_TILE_BLOCKS 2      // 64-row blocks of d per LDS tile of the pipelined router kernel
#endif
#ifndef ROUTER_TILE_STAGES
#define ROUTER_TILE_STAGES 3      // tiles in its ring (at most 4: the waits count up to two younger tiles); 2 to 4 measured alike
#endif
#ifndef ROUTER_SLICES
#define ROUTER_SLICES 2     // 16-expert slices per workgroup of the pipelined router kernel when there are plenty of workgroups
#endif
constexpr int R_TB = 8;     // tokens per wave
constexpr int R_NB = 16;    // experts per pass
constexpr int R_QT = 4;     // 64-row blocks of W_g staged per LDS tile
constexpr int ROUTER_DX_PICKS = 1024;   // (token, pick) pairs a workgroup of the router's dx kernel stages
#ifndef ROUTER_DX_CPL
#define ROUTER_DX_CPL 4                 // output columns per lane of that kernel
#endif
#ifndef ROUTER_DX_THREADS
#define ROUTER_DX_THREADS 1024
#endif
#ifndef ROUTER_DX_TOKENS
#define ROUTER_DX_TOKENS 128
#endif
constexpr int R_PAD = 20;   // floats per staged row (16 + 4: conflict-free 16-byte reads)

// Block = 4 wavefronts x 8 tokens, one pass of 16 experts (blockIdx.y); the 16 router columns are
// staged through LDS in tiles of 256 rows and shared by the four wavefronts.
template <typename XT>
__global__ __launch_bounds__(256) void router_logits_kernel(const XT* __restrict__ x, const float* __restrict__ wg,
                                                            const float* __restrict__ bias, float* __restrict__ logits,
                                                            int T, int d, int N) {
  __shared__ float sw[R_QT * 64 * R_PAD];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t0 = blockIdx.x * (4 * R_TB) + wave * R_TB;
  const int n0 = blockIdx.y * R_NB;
  const int nq = d / 64;
  const bool vec = (N % 4) == 0;
  float acc[R_TB * R_NB];
#pragma unroll
  for (int v = 0; v < R_TB * R_NB; ++v) acc[v] = 0.0f;
  for (int q0 = 0; q0 < nq; q0 += R_QT) {
    // this tile's tokens first: R_QT x R_TB independent loads in flight
    float xv[R_QT][R_TB];
#pragma unroll
    for (int qq = 0; qq < R_QT; ++qq)
#pragma unroll
      for (int i = 0; i < R_TB; ++i) {
        const int t = t0 + i;
        xv[qq][i] = (t < T && q0 + qq < nq) ? Elem<XT>::load(x + (size_t)t * d + (size_t)(q0 + qq) * 64 + lane) : 0.0f;
      }
    __syncthreads();
    if (vec) {
      for (int e = threadIdx.x; e < R_QT * 64 * (R_NB / 4); e += 256) {
        const int row = e / (R_NB / 4), c = (e % (R_NB / 4)) * 4;
        const int gi = q0 * 64 + row, gn = n0 + c;
        float4 w = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gi < d && gn < N) w = *(const float4*)(wg + (size_t)gi * N + gn);
        *(float4*)(sw + row * R_PAD + c) = w;
      }
    } else {
      for (int e = threadIdx.x; e < R_QT * 64 * R_NB; e += 256) {
        const int row = e / R_NB, c = e % R_NB;
        const int gi = q0 * 64 + row, gn = n0 + c;
        sw[row * R_PAD + c] = (gi < d && gn < N) ? wg[(size_t)gi * N + gn] : 0.0f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int qq = 0; qq < R_QT; ++qq) {
      if (q0 + qq >= nq) break;
      const float4* wrow = (const float4*)(sw + (qq * 64 + lane) * R_PAD);
      float wv[R_NB];
#pragma unroll
      for (int c4 = 0; c4 < R_NB / 4; ++c4) {
        float4 w = wrow[c4];
        wv[c4 * 4 + 0] = w.x; wv[c4 * 4 + 1] = w.y; wv[c4 * 4 + 2] = w.z; wv[c4 * 4 + 3] = w.w;
      }
#pragma unroll
      for (int i = 0; i < R_TB; ++i)
#pragma unroll
        for (int c = 0; c < R_NB; ++c) acc[i * R_NB + c] = fmaf(xv[qq][i], wv[c], acc[i * R_NB + c]);
    }
  }
  // halving tree as a reduce-scatter: at distance off the lanes with that bit set keep the
  // upper half of the values, the others the lower half; value 2*lane + {0,1} ends on lane.
#pragma unroll
  for (int off = 32, half = R_TB * R_NB / 2; off >= 1; off >>= 1, half >>= 1) {
    const bool hi = (lane & off) != 0;
#pragma unroll
    for (int v = 0; v < half; ++v) {
      const float send = hi ? acc[v] : acc[v + half];
      const float keep = hi ? acc[v + half] : acc[v];
      acc[v] = keep + __shfl_xor(send, off, 64);
    }
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int v = 2 * lane + u;
    const int t = t0 + v / R_NB, n = n0 + v % R_NB;
    if (t < T && n < N) {
      float val = acc[u];
      if (bias) val = val + bias[n];
      logits[(size_t)t * N + n] = val;
    }
  }
}

// LDS reads with a compile-time instruction offset, as assembly (see the kernel below for why).
template <int OFFSET>
__device__ __forceinline__ void router_lds_read_u16(unsigned addr, unsigned& v) {
  asm volatile("ds_read_u16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET) : "memory");
}
template <int OFFSET>
__device__ __forceinline__ void router_lds_read_b32(unsigned addr, unsigned& v) {
  asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET) : "memory");
}
typedef unsigned int router_u32x4 __attribute__((ext_vector_type(4)));
template <int OFFSET>
__device__ __forceinline__ void router_lds_read_b128(unsigned addr, router_u32x4& v) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET) : "memory");
}
template <int I> struct RouterIndex { static constexpr int value = I; };
template <int BEGIN, int END, typename F>
__device__ __forceinline__ void router_static_for(F&& f) {
  if constexpr (BEGIN < END) {
    f(RouterIndex<BEGIN>{});
    router_static_for<BEGIN + 1, END>(f);
  }
}

// Same computation for N % 4 == 0, software-pipelined: token tiles (32 tokens x 64 QQT elements)
// and router tiles (64 QQT rows x 16 columns) travel global -> LDS directly (16 bytes per lane, no
// registers) through a ring of S stages, S - 1 tiles in flight while the 128 QQT fused
// multiply-adds per lane of the current one run.  Token rows past T and router rows past d lie
// outside the buffer ranges and arrive as zeros; they are never used anyway.
#define BIGMAC_ROUTER_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))
// TB = tokens per wavefront (8 for large T; 1 or 2 when T is small, so that the few tokens still
// spread over many CUs).  The summation order does not depend on it.
// SL = 16-expert slices a workgroup computes one after the other on its token tile: the next
// slice's first tiles are requested before the reduction of the current one, so the fixed cost
// of a workgroup (set-up, first-tile latency) is paid once per SL slices.
template <typename XT, int TB, int SL>
__global__ __launch_bounds__(256) void router_logits_pipelined_kernel(const XT* __restrict__ x, const float* __restrict__ wg,
                                                                      const float* __restrict__ bias, float* __restrict__ logits,
                                                                      int T, int d, int N) {
  constexpr int QQT = ROUTER_TILE_BLOCKS;           // 64-row blocks of d per tile
  constexpr int S = sizeof(XT) == 2 ? ROUTER_TILE_STAGES : 3;   // ring of S tiles, S - 1 in flight while one is consumed
  static_assert(S >= 2 && S <= 4 && QQT >= 1 && QQT <= 4, "the counter waits below cover up to two younger tiles");
  constexpr int TROWS = 64 * QQT;                   // rows of d per tile
  constexpr int XROW = TROWS * sizeof(XT) / 16;     // 16-byte chunks per token row of a tile
  constexpr int TOKENS = 4 * TB;                    // tokens per workgroup
  constexpr int XCH = TOKENS * XROW;                // chunks of a token tile
  constexpr int WCH = TROWS * 4;                    // chunks of a router tile (TROWS rows x 16 floats)
  constexpr int XL = (XCH + 255) / 256, WL = (WCH + 255) / 256;   // loads per thread
  constexpr int LPT = XL + WL;
  __shared__ uint4 xring[S * XL * 256];             // (a tile of fewer than 256 chunks is padded: the surplus lanes load out of range)
  __shared__ uint4 wring[S * WL * 256];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  // Workgroup -> (token block, expert slices).  The workgroups that share a token block (one per
  // group of SL slices) get linear indices 8 apart: consecutive indices go round the 8 XCDs, so
  // these land on one XCD at about the same time and the block's token rows come from memory
  // once, then from that XCD's L2; every XCD keeps all of w_gate.  (With the slice index as the
  // slow grid dimension the token rows were fetched once per slice group and the router columns
  // did not stay in the L2 behind them: 8 times the algorithmic bytes at d = 4096, N = 128.)
  const int slice_groups = (N + SL * R_NB - 1) / (SL * R_NB);
  const int lin = (int)(blockIdx.x >> 3);
  const int token_block = (lin / slice_groups) * 8 + (int)(blockIdx.x & 7);
  const int tb = token_block * TOKENS, t0 = tb + wave * TB;
  if (tb >= T) return;
  int n0 = (lin % slice_groups) * (SL * R_NB);
  const int nq = d / 64, ntiles = (nq + QQT - 1) / QQT;
  const int rows = min(TOKENS, T - tb);
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)(x + (size_t)tb * d), 0, (int)((size_t)rows * d * sizeof(XT)), 0x00020000);
  auto router_columns = [&](int first) {   // the slice's 16 columns of w_gate as a buffer
    const int cols = min(R_NB, N - first);
    return __builtin_amdgcn_make_buffer_rsrc((void*)(wg + first), 0, (int)(((size_t)(d - 1) * N + cols) * 4), 0x00020000);
  };
  __amdgpu_buffer_rsrc_t rw = router_columns(n0);
  const int wave_chunk = __builtin_amdgcn_readfirstlane((int)(threadIdx.x & ~63u));
  unsigned xoff[XL], woff[WL];
#pragma unroll
  for (int i = 0; i < XL; ++i) {
    const int q = i * 256 + threadIdx.x;
    xoff[i] = q < XCH ? (unsigned)((q / XROW) * d * sizeof(XT) + (q % XROW) * 16) : 0x80000000u;
  }
  // LDS position q holds column chunk (q & 3) ^ ((row >> 2) & 3) of row q >> 2: the 16 rows that one
  // pass of a 16-byte read touches (64 bytes apart, 4 to every 256 bytes the banks span) then fall
  // on 16 different bank groups
#pragma unroll
  for (int i = 0; i < WL; ++i) {
    const int q = i * 256 + threadIdx.x, row = q >> 2;
    woff[i] = q < WCH ? (unsigned)((row * N + (((q & 3) ^ ((row >> 2) & 3)) << 2)) * 4) : 0x80000000u;
  }
  auto issue = [&](int tile) {
    uint4* xs = xring + (tile % S) * (XL * 256);
    uint4* ws = wring + (tile % S) * (WL * 256);
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
    for (int i = 0; i < XL; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void*)(xs + i * 256 + wave_chunk), 16,
                                               xoff[i] + (unsigned)(tile * TROWS * sizeof(XT)), 0, 0, 0);
#pragma unroll
    for (int i = 0; i < WL; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (__attribute__((address_space(3))) void*)(ws + i * 256 + wave_chunk), 16,
                                               woff[i] + (unsigned)(tile * TROWS * N * 4), 0, 0, 0);
#else
    (void)xs; (void)ws;
#endif
  };
  constexpr int ACCS = TB * R_NB;
  float acc[ACCS];
  // The tile reads are assembly: for LDS accesses it can see, the compiler waits for every
  // direct-to-LDS load in flight, the next tiles' included, which would put the loads and the
  // arithmetic one after the other instead of side by side.  The only waits on the loads are the
  // counter waits of the loop below.
  const unsigned xring_at = (unsigned)(size_t)(__attribute__((address_space(3))) const void*)xring + (unsigned)(((wave * TB) * TROWS + lane) * sizeof(XT));
  const unsigned wring_at = (unsigned)(size_t)(__attribute__((address_space(3))) const void*)wring;
  unsigned wlane[4];   // the swizzle term (row >> 2) & 3 is the same in every 64-row block
#pragma unroll
  for (int c4 = 0; c4 < 4; ++c4) wlane[c4] = wring_at + (unsigned)((lane * 4 + (c4 ^ ((lane >> 2) & 3))) * 16);
  auto compute = [&](int tile) {
    // one address register for the token rows, four for the router columns; everything else is
    // instruction offsets
    const unsigned stage = (unsigned)(tile % S);
    const unsigned xat = xring_at + stage * (XL * 256 * 16);
    unsigned wat[4];
#pragma unroll
    for (int c4 = 0; c4 < 4; ++c4) wat[c4] = wlane[c4] + stage * (WL * 256 * 16);
    unsigned xraw[2][TB];
    router_u32x4 wraw[2][4];
    // the reads of 64-row block QQ of the tile, into register set QQ % 2
    auto request = [&](auto block) {
      constexpr int QQ = decltype(block)::value;
      router_static_for<0, TB>([&](auto token) {
        constexpr int I = decltype(token)::value;
        if constexpr (sizeof(XT) == 2) router_lds_read_u16<(I * TROWS + QQ * 64) * 2>(xat, xraw[QQ & 1][I]);
        else router_lds_read_b32<(I * TROWS + QQ * 64) * 4>(xat, xraw[QQ & 1][I]);
      });
      router_static_for<0, 4>([&](auto chunk) {
        constexpr int C4 = decltype(chunk)::value;
        router_lds_read_b128<QQ * 64 * 4 * 16>(wat[C4], wraw[QQ & 1][C4]);
      });
    };
    request(RouterIndex<0>{});
    router_static_for<0, QQT>([&](auto block) {
      constexpr int QQ = decltype(block)::value;
      if (tile * QQT + QQ >= nq) return;
      // block QQ has arrived (it was requested before the previous block's arithmetic); the next
      // block is requested now and arrives while this one's 128 multiply-adds run
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int i = 0; i < TB; ++i) asm volatile("" : "+v"(xraw[QQ & 1][i]));
#pragma unroll
      for (int c4 = 0; c4 < 4; ++c4) asm volatile("" : "+v"(wraw[QQ & 1][c4]));
      if constexpr (QQ + 1 < QQT) request(RouterIndex<QQ + 1>{});   // (a block past d holds zeros or stale rows: never used)
      float xv[TB], wv[R_NB];
#pragma unroll
      for (int i = 0; i < TB; ++i) xv[i] = __uint_as_float(sizeof(XT) == 2 ? xraw[QQ & 1][i] << 16 : xraw[QQ & 1][i]);
#pragma unroll
      for (int c4 = 0; c4 < 4; ++c4) {
        const router_u32x4 w = wraw[QQ & 1][c4];
        wv[c4 * 4 + 0] = __uint_as_float(w.x); wv[c4 * 4 + 1] = __uint_as_float(w.y);
        wv[c4 * 4 + 2] = __uint_as_float(w.z); wv[c4 * 4 + 3] = __uint_as_float(w.w);
      }
#pragma unroll
      for (int i = 0; i < TB; ++i)
#pragma unroll
        for (int c = 0; c < R_NB; ++c) acc[i * R_NB + c] = fmaf(xv[i], wv[c], acc[i * R_NB + c]);
    });
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // a request past the last block used: done before the stage is refilled
  };
  // The ring: tiles 0 .. S-2 are requested up front; at tile t a wavefront waits until only the
  // tiles requested after t are in flight, the barrier makes that true for everyone's part of t
  // and says that everyone has left tile t - 1, whose stage then takes tile t + S - 1.
  auto start_ring = [&]() {
#pragma unroll
    for (int a = 0; a < S - 1; ++a)
      if (a < ntiles) issue(a);
  };
  start_ring();
#pragma unroll 1
  for (int sl = 0; sl < SL; ++sl) {
#pragma unroll
  for (int v = 0; v < ACCS; ++v) acc[v] = 0.0f;
  for (int tile = 0; tile < ntiles; ++tile) {
    const int younger = min(S - 2, ntiles - 1 - tile);
    if (younger >= 2) BIGMAC_ROUTER_WAIT_VMCNT(2 * LPT);
    else if (younger == 1) BIGMAC_ROUTER_WAIT_VMCNT(LPT);
    else BIGMAC_ROUTER_WAIT_VMCNT(0);
    __builtin_amdgcn_s_barrier();
    if (tile + S - 1 < ntiles) issue(tile + S - 1);
    compute(tile);
  }
  // once every wavefront has left the last tile, the next slice's first tiles can be on their way
  // while this slice is reduced and stored
  const int n_cur = n0;
  const bool more = sl + 1 < SL && n0 + R_NB < N;
  if (more) {
    __builtin_amdgcn_s_barrier();
    n0 += R_NB;
    rw = router_columns(n0);
    start_ring();
  }
  // Halving tree (lane l with lane l ^ off, off = 32 .. 1).  While a lane still holds two or more
  // sums the step is a reduce-scatter: each half of the pair keeps one half of the sums (see
  // router_logits_kernel); once a lane is down to one sum, both lanes of a pair add the other's
  // (the same addition, a + b, in both).  The sum of accumulator v ends on the lanes whose top
  // bits spell v.
  constexpr int SCATTER_STEPS = ACCS >= 64 ? 6 : (ACCS == 32 ? 5 : 4);
  static_assert(ACCS == 128 || ACCS == 64 || ACCS == 32 || ACCS == 16, "1, 2, 4 or 8 tokens per wavefront");
#pragma unroll
  for (int step = 0; step < 6; ++step) {
    const int off = 32 >> step;
    if (step < SCATTER_STEPS && off >= 16) {
      // distances 32 and 16: one swap instruction exchanges the upper half (odd 16-lane rows) of
      // acc[v] with the lower half (even rows) of acc[v + half]; afterwards every lane holds what
      // it keeps in one register and what its partner sent in the other, and a + b = b + a
      const int half = ACCS >> (step + 1);
#pragma unroll
      for (int v = 0; v < half; ++v) {
        const unsigned a = __float_as_uint(acc[v]), b = __float_as_uint(acc[v + half]);
        if (off == 32) {
          const auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
          acc[v] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
        } else {
          const auto r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
          acc[v] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
        }
      }
    } else if (step < SCATTER_STEPS) {
      const int half = ACCS >> (step + 1);
      const bool hi = (lane & off) != 0;
#pragma unroll
      for (int v = 0; v < half; ++v) {
        const float send = hi ? acc[v] : acc[v + half];
        const float keep = hi ? acc[v + half] : acc[v];
        acc[v] = keep + __shfl_xor(send, off, 64);
      }
    } else {
      acc[0] = acc[0] + __shfl_xor(acc[0], off, 64);
    }
  }
  constexpr int LEFT = ACCS >> SCATTER_STEPS;          // sums per lane at the end: 2 (ACCS = 128) or 1
  constexpr int SHARE = 6 - SCATTER_STEPS;             // low lane bits that hold copies of the same sum
  if ((lane & ((1 << SHARE) - 1)) == 0) {
#pragma unroll
    for (int u = 0; u < LEFT; ++u) {
      const int v = LEFT * (lane >> SHARE) + u;
      const int t = t0 + v / R_NB, n = n_cur + v % R_NB;
      if (t < T && n < N) {
        float val = acc[u];
        if (bias) val = val + bias[n];
        logits[(size_t)t * N + n] = val;
      }
    }
  }
  if (!more) break;
  }
}

// One wavefront per token.  More than 128 experts: every lane ranks its logits against all N by broadcast (rank = how
// many logits come first: greater, or equal with a lower index, which is the order k rounds of
// arg-max with ties to the lowest index would pick them in); ranks below k are the selection, in
// pick order.  Then the softmax over the k picked logits, summed in pick order.  PER = logits
// held per lane.
template <int PER>
__global__ __launch_bounds__(256) void topk_gate_kernel(const float* __restrict__ logits, int T, int N, int k,
                                                        int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  // "a comes first": greater logit, equal logits by lower index (a strict total order)
  auto first = [](float av, int ai, float bv, int bi) { return av > bv || (av == bv && ai < bi); };
  // one compare-exchange step of a bitonic network over the wavefront: partner lane ^ j, the pair's
  // first element goes to the lane for which want_first holds
  auto exchange = [&](float& mv, int& mi, int j, bool want_first) {
    const float ov = __shfl_xor(mv, j, 64);
    const int oi = __shfl_xor(mi, j, 64);
    if (first(mv, mi, ov, oi) != want_first) { mv = ov; mi = oi; }
  };
  auto sort64 = [&](float& mv, int& mi) {   // lane 0 ends with the first element
#pragma unroll
    for (int size = 2; size <= 64; size <<= 1)
#pragma unroll
      for (int j = size >> 1; j > 0; j >>= 1) exchange(mv, mi, j, ((lane & j) == 0) == ((lane & size) == 0));   // lower lane of an ascending block
  };
  if constexpr (PER <= 2) {
    // Up to 64 experts: one logit per lane, sorted across the wavefront by a bitonic network (the
    // order is strict and total, so the result is the unique sorted sequence); lanes 0 .. k-1 then
    // hold the picks in pick order.  Up to 128: two logits per lane, both halves sorted the same
    // way; the first 64 of their union are, lane by lane, the first of (half 0 at lane l, half 1
    // at lane 63 - l), a bitonic sequence that six more steps sort.  k <= 64 picks are all there.
    float mv = lane < N ? logits[(size_t)t * N + lane] : -INFINITY;
    int mi = lane;
    sort64(mv, mi);
    if constexpr (PER == 2) {
      float uv = 64 + lane < N ? logits[(size_t)t * N + 64 + lane] : -INFINITY;
      int ui = 64 + lane;
      sort64(uv, ui);
      const float rv = __shfl(uv, 63 - lane, 64);
      const int ri = __shfl(ui, 63 - lane, 64);
      if (!first(mv, mi, rv, ri)) { mv = rv; mi = ri; }
#pragma unroll
      for (int j = 32; j > 0; j >>= 1) exchange(mv, mi, j, (lane & j) == 0);
    }
    const float m = __shfl(mv, 0, 64);
    const float e = lane < k ? expf(mv - m) : 0.0f;
    float s = 0.0f;
    for (int j = 0; j < k; ++j) s += __shfl(e, j, 64);
    if (lane < k) {
      topk_idx[(size_t)t * k + lane] = mi;
      topk_w[(size_t)t * k + lane] = e / s;
    }
    return;
  }
  float v[PER];
  int rank[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int n = i * 64 + lane;
    v[i] = n < N ? logits[(size_t)t * N + n] : -INFINITY;
    rank[i] = 0;
  }
#pragma unroll
  for (int io = 0; io < PER; ++io) {
    const int live = min(64, N - io * 64);        // lanes of this register that hold a logit
    for (int l = 0; l < live; ++l) {
      const float o = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v[io]), l));
      const int on = io * 64 + l;
#pragma unroll
      for (int i = 0; i < PER; ++i) rank[i] += (o > v[i] || (o == v[i] && on < i * 64 + lane)) ? 1 : 0;
    }
  }
  // lane j < k collects the j-th pick: its index and logit
  float selv = 0.0f;
  int seli = 0;
  for (int j = 0; j < k; ++j) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const unsigned long long hit = __ballot(rank[i] == j && i * 64 + lane < N);
      if (hit) {                                  // wave-uniform: exactly one (i, lane) has rank j
        const int src = __ffsll((long long)hit) - 1;
        const float pv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v[i]), src));
        if (lane == j) { selv = pv; seli = i * 64 + src; }
      }
    }
  }
  const float m = __shfl(selv, 0, 64);
  const float e = lane < k ? expf(selv - m) : 0.0f;
  float s = 0.0f;
  for (int j = 0; j < k; ++j) s += __shfl(e, j, 64);
  if (lane < k) {
    topk_idx[(size_t)t * k + lane] = seli;
    topk_w[(size_t)t * k + lane] = e / s;
  }
}

__global__ void transpose_f32_kernel(const float* __restrict__ in, float* __restrict__ out, int rows, int cols) {
  __shared__ float tile[32][33];
  int c = blockIdx.x * 32 + threadIdx.x, r0 = blockIdx.y * 32;
  for (int i = threadIdx.y; i < 32; i += 8)
    if (r0 + i < rows && c < cols) tile[i][threadIdx.x] = in[(size_t)(r0 + i) * cols + c];
  __syncthreads();
  int r = r0 + threadIdx.x, c0 = blockIdx.x * 32;
  for (int i = threadIdx.y; i < 32; i += 8)
    if (c0 + i < cols && r < rows) out[(size_t)(c0 + i) * rows + r] = tile[threadIdx.x][i];
}

// softmax over all N logits of one token by one wavefront: lane l holds experts l, l + 64, ...
template <int PER>
__device__ __forceinline__ void softmax_row(const float* __restrict__ row, int N, int lane, float (&p)[PER]) {
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int n = i * 64 + lane;
    p[i] = n < N ? row[n] : -INFINITY;
    m = fmaxf(m, p[i]);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  float sum = 0.0f;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    p[i] = i * 64 + lane < N ? expf(p[i] - m) : 0.0f;
    sum += p[i];
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int i = 0; i < PER; ++i) p[i] *= inv;
}

// Gradient of the load-balance loss  alpha N sum_e f_e P_e  with respect to one token's logits,
// the pair shares f held fixed:  scale p_n (f_n - sum_e f_e p_e),  scale = alpha N / T.
template <int PER>
__device__ __forceinline__ void aux_grad_row(const float* __restrict__ row, const float* __restrict__ share, int N, int lane,
                                             float scale, float (&g)[PER]) {
  float f[PER];
  softmax_row<PER>(row, N, lane, g);
  float mix = 0.0f;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int n = i * 64 + lane;
    f[i] = n < N ? share[n] : 0.0f;
    mix = fmaf(f[i], g[i], mix);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mix += __shfl_xor(mix, off, 64);
#pragma unroll
  for (int i = 0; i < PER; ++i) g[i] = scale * g[i] * (f[i] - mix);
}

// Column sums of softmax(logits) over a strided share of the tokens: workgroup b, wavefront w
// takes tokens (b * 4 + w) + i * 4 * gridDim.x.  partial[b][n], the four wavefronts added in order.
template <int PER>
__global__ __launch_bounds__(256) void aux_colsum_kernel(const float* __restrict__ logits, int T, int N, float* __restrict__ partial) {
  __shared__ float sums[4][1024];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float col[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) col[i] = 0.0f;
  for (int t = blockIdx.x * 4 + wave; t < T; t += 4 * gridDim.x) {
    float p[PER];
    softmax_row<PER>(logits + (size_t)t * N, N, lane, p);
#pragma unroll
    for (int i = 0; i < PER; ++i) col[i] += p[i];
  }
#pragma unroll
  for (int i = 0; i < PER; ++i)
    if (i * 64 + lane < N) sums[wave][i * 64 + lane] = col[i];
  __syncthreads();
  for (int n = threadIdx.x; n < N; n += 256)
    partial[(size_t)blockIdx.x * N + n] = ((sums[0][n] + sums[1][n]) + sums[2][n]) + sums[3][n];
}

// One workgroup: pair counts per expert (integer, order-free), P_e from the partial column sums,
// share[e] = f_e, and the loss  alpha N sum_e f_e P_e.  Every sum has a fixed order: the 1024
// threads are G groups x NP experts (NP = N rounded up to a power of two); group g adds its
// contiguous range of partials in order, the G group sums are added in group order, and the N
// terms f_e P_e go through a fixed tree.
__global__ __launch_bounds__(1024) void aux_finish_kernel(const int32_t* __restrict__ topk_idx, const float* __restrict__ partial,
                                                          int nparts, int T, int N, int NP, int k, float alpha,
                                                          float* __restrict__ share, float* __restrict__ loss) {
  __shared__ int cnt[1024];
  __shared__ float psum[1024];
  cnt[threadIdx.x] = 0;
  __syncthreads();
  const int Tk = T * k;
  const int quads = Tk / 4;                        // 16-byte reads; the base pointer is 16-byte aligned
  for (int q = threadIdx.x; q < quads; q += 1024) {
    const int4 v = ((const int4*)topk_idx)[q];
    atomicAdd(&cnt[v.x], 1); atomicAdd(&cnt[v.y], 1); atomicAdd(&cnt[v.z], 1); atomicAdd(&cnt[v.w], 1);
  }
  for (int f = quads * 4 + threadIdx.x; f < Tk; f += 1024) atomicAdd(&cnt[topk_idx[f]], 1);
  const int G = 1024 / NP, e = threadIdx.x % NP, g = threadIdx.x / NP;
  const int per = (nparts + G - 1) / G;
  const int b_beg = min(g * per, nparts), b_end = min(b_beg + per, nparts);
  float mine = 0.0f;
  if (e < N)
    for (int b = b_beg; b < b_end; ++b) mine += partial[(size_t)b * N + e];
  psum[g * NP + e] = mine;
  __syncthreads();
  float term = 0.0f;
  if ((int)threadIdx.x < N) {
    float P = 0.0f;
    for (int h = 0; h < G; ++h) P += psum[h * NP + threadIdx.x];
    const float f = (float)cnt[threadIdx.x] / (float)Tk;
    share[threadIdx.x] = f;
    term = f * (P / (float)T);
  }
  __syncthreads();
  psum[threadIdx.x] = term;
  __syncthreads();
  for (int half = 512; half >= 1; half >>= 1) {
    if ((int)threadIdx.x < half) psum[threadIdx.x] += psum[threadIdx.x + half];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = alpha * (float)N * psum[0];
}

// dlogits[t, :] of the load-balance loss, one wavefront per token
template <int PER>
__global__ __launch_bounds__(256) void aux_grad_kernel(const float* __restrict__ logits, const float* __restrict__ share, int T, int N,
                                                       float scale, float* __restrict__ dlogits) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  float g[PER];
  aux_grad_row<PER>(logits + (size_t)t * N, share, N, lane, scale, g);
#pragma unroll
  for (int i = 0; i < PER; ++i)
    if (i * 64 + lane < N) dlogits[(size_t)t * N + i * 64 + lane] = g[i];
}

// Backward of the gate (softmax over the k picked logits) and the router's share of dx.
// One wavefront per token.  dL (dense [T, N], storage type DT) feeds d_w_gate = x^T dL.
// With the load-balance loss (logits != NULL) its gradient joins every entry of the row and the
// router's share of dx runs over all N experts instead of the k picked ones (dx == NULL: left to
// the caller).
template <typename DT, int PER>
__global__ __launch_bounds__(256) void gate_backward_kernel(const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w,
                                                            const float* __restrict__ dgate, const float* __restrict__ wg_t /*[N,d]*/,
                                                            const float* __restrict__ logits, const float* __restrict__ share, float aux_scale,
                                                            DT* __restrict__ dL, float* __restrict__ dx, float* __restrict__ dl_picked,
                                                            int T, int d, int N, int k) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  float aux[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) aux[i] = 0.0f;
  if (logits) aux_grad_row<PER>(logits + (size_t)t * N, share, N, lane, aux_scale, aux);
  float w = 0.0f, g = 0.0f;
  int e = 0;
  if (lane < k) {
    w = topk_w[(size_t)t * k + lane];
    g = dgate[(size_t)t * k + lane];
    e = topk_idx[(size_t)t * k + lane];
  }
  float mix = 0.0f;
  for (int j = 0; j < k; ++j) mix = fmaf(__shfl(w, j, 64), __shfl(g, j, 64), mix);
  const float dl = w * (g - mix);
  if (dl_picked && lane < k) dl_picked[(size_t)t * k + lane] = dl;
  // every lane takes part in the shuffles (uniform trip counts); only loads and stores are guarded
#pragma unroll
  for (int i = 0; i < PER; ++i) {        // dense row of dL: the k picked experts, zeros (or the loss term) elsewhere
    if (i * 64 >= N) break;
    const int n = i * 64 + lane;
    float val = 0.0f;
    for (int j = 0; j < k; ++j) {
      const float dj = __shfl(dl, j, 64);
      if (__shfl(e, j, 64) == n) val = dj;
    }
    aux[i] += val;                       // the whole dlogits entry from here on
    if (n < N) Elem<DT>::store(dL + (size_t)t * N + n, logits ? aux[i] : val);
  }
  if (!dx) return;                        // the caller forms the router's share of dx as a product with dL
  for (int c0 = 0; c0 < d; c0 += 256) {
    const int c = c0 + lane * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (!logits) {
      for (int j = 0; j < k; ++j) {
        const float dj = __shfl(dl, j, 64);
        const int ej = __shfl(e, j, 64);
        if (c < d) {
          const float4 wv = *(const float4*)(wg_t + (size_t)ej * d + c);
          acc.x = fmaf(dj, wv.x, acc.x); acc.y = fmaf(dj, wv.y, acc.y);
          acc.z = fmaf(dj, wv.z, acc.z); acc.w = fmaf(dj, wv.w, acc.w);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        if (i * 64 >= N) break;
        const int live = min(64, N - i * 64);
        for (int l = 0; l < live; ++l) {
          const float dn = __shfl(aux[i], l, 64);
          if (c < d) {
            const float4 wv = *(const float4*)(wg_t + (size_t)(i * 64 + l) * d + c);
            acc.x = fmaf(dn, wv.x, acc.x); acc.y = fmaf(dn, wv.y, acc.y);
            acc.z = fmaf(dn, wv.z, acc.z); acc.w = fmaf(dn, wv.w, acc.w);
          }
        }
      }
    }
    if (c < d) *(float4*)(dx + (size_t)t * d + c) = acc;
  }
}

// The router's share of dx without the loss:  dx[t, c] = sum_j dl[t, j] w_gate[c, e_j].  A
// workgroup keeps CPL*64 rows of w_gate, transposed (wt[n][c]: one expert's weights for the
// workgroup's columns lie side by side), and its tokens' picks in the LDS, so each pick costs a
// lane one LDS read of its CPL adjacent columns instead of a cached global row.
template <int CPL, int NMAX>
__global__ __launch_bounds__(ROUTER_DX_THREADS) void router_dx_kernel(const int32_t* __restrict__ topk_idx, const float* __restrict__ dl_picked,
                                                        const float* __restrict__ w_gate /*[d,N]*/, float* __restrict__ dx,
                                                        int T, int d, int N, int k, int tokens_per_block) {
  constexpr int TC = CPL * 64, PITCH = TC + 4;
  constexpr int PER_THREAD = TC * NMAX / 4 / ROUTER_DX_THREADS, BATCH = PER_THREAD > 8 ? 8 : (PER_THREAD < 1 ? 1 : PER_THREAD);
  typedef float cols_t __attribute__((ext_vector_type(CPL)));
  __shared__ __attribute__((aligned(16))) float wt[NMAX * PITCH];
  __shared__ float s_dl[ROUTER_DX_PICKS];
  __shared__ int s_e[ROUTER_DX_PICKS];
  const int c0 = blockIdx.x * TC;
  // A workgroup fills its rows of w_gate once and then walks the token groups blockIdx.y,
  // blockIdx.y + gridDim.y, ...: the picks of a group are requested before the work in front of
  // them (the fill; the sums of the group before) and stored into the LDS behind it.
  constexpr int PICK_LOADS = (ROUTER_DX_PICKS + ROUTER_DX_THREADS - 1) / ROUTER_DX_THREADS;
  const int groups = (T + tokens_per_block - 1) / tokens_per_block;
  float pick_dl[PICK_LOADS];
  int pick_e[PICK_LOADS];
  auto request_picks = [&](int group) {
    const int t_beg = group * tokens_per_block, picks_here = (min(T, t_beg + tokens_per_block) - t_beg) * k;
#pragma unroll
    for (int u = 0; u < PICK_LOADS; ++u) {
      const size_t at = (size_t)t_beg * k + min(u * ROUTER_DX_THREADS + (int)threadIdx.x, picks_here - 1);
      pick_dl[u] = dl_picked[at];
      pick_e[u] = topk_idx[at];
    }
  };
  auto stage_picks = [&](int group) {
    const int t_beg = group * tokens_per_block, picks_here = (min(T, t_beg + tokens_per_block) - t_beg) * k;
#pragma unroll
    for (int u = 0; u < PICK_LOADS; ++u) {
      const int i = u * ROUTER_DX_THREADS + (int)threadIdx.x;
      if (i < picks_here) { s_dl[i] = pick_dl[u]; s_e[i] = pick_e[u]; }
    }
  };
  int group = blockIdx.y;
  if (group >= groups) return;
  request_picks(group);
  if ((N & 3) == 0) {
    // 16-byte loads, a batch in flight per lane.  Work item g = (group, quad in row % 4, row % 16):
    // 16 lanes take the same quad of 16 consecutive rows, 4 such sets make a wavefront.  Its four
    // transposing stores then write 16 consecutive words in each of 4 rows of wt that lie
    // 4 * PITCH = 16 (mod 64) words apart: all 64 banks once.  (In row-major order of w_gate the
    // stores of a wavefront would fall on 4 banks.)  Rows past d are clamped to the last one
    // (their outputs are never stored).
    const int qrow = N >> 2, qsets = (qrow + 3) >> 2, items = (TC / 16) * qsets * 64, last_row = d - 1 - c0;
    const float4* src = (const float4*)(w_gate + (size_t)c0 * N);
    for (int g0 = 0; g0 < items; g0 += ROUTER_DX_THREADS * BATCH) {
      float4 v[BATCH];
#pragma unroll
      for (int u = 0; u < BATCH; ++u) {
        const int g = g0 + u * ROUTER_DX_THREADS + (int)threadIdx.x, group = g >> 6;
        const int c = min((group % (TC / 16)) * 16 + (g & 15), last_row);
        const int n4 = min((group / (TC / 16)) * 4 + ((g >> 4) & 3), qrow - 1);
        v[u] = src[c * qrow + n4];
      }
#pragma unroll
      for (int u = 0; u < BATCH; ++u) {
        const int g = g0 + u * ROUTER_DX_THREADS + (int)threadIdx.x, group = g >> 6;
        const int c = (group % (TC / 16)) * 16 + (g & 15), n4 = (group / (TC / 16)) * 4 + ((g >> 4) & 3);
        if (g < items && n4 < qrow) {
          float* dst = wt + n4 * 4 * PITCH + c;
          dst[0] = v[u].x; dst[PITCH] = v[u].y; dst[2 * PITCH] = v[u].z; dst[3 * PITCH] = v[u].w;
        }
      }
    }
  } else {
    for (int i = threadIdx.x; i < TC * N; i += ROUTER_DX_THREADS) {
      const int c = i / N, n = i - c * N;
      wt[n * PITCH + c] = c0 + c < d ? w_gate[(size_t)(c0 + c) * N + n] : 0.0f;
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* mine = wt + lane * CPL;
  while (true) {
    stage_picks(group);
    __syncthreads();                    // the picks (and, the first time, the rows of w_gate) are in the LDS
    const int next = group + (int)gridDim.y;
    if (next < groups) request_picks(next);
    const int t_beg = group * tokens_per_block, t_end = min(T, t_beg + tokens_per_block);
    for (int t = t_beg + wave; t < t_end; t += ROUTER_DX_THREADS / 64) {
      const int base = (t - t_beg) * k;
      // lane j holds pick j (k <= 64); every lane then reads them back one by one
      const int at = base + min(lane, k - 1);
      const int dl_bits = __float_as_int(s_dl[at]), e_mine = s_e[at];
      cols_t acc = 0.0f;
      // U picks at a time: their LDS reads are independent, the sums keep the order j = 0, 1, ...
      auto picks = [&](auto width, int j) {
        constexpr int U = decltype(width)::value;
        float dj[U];
        cols_t w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          dj[u] = __int_as_float(__builtin_amdgcn_readlane(dl_bits, j + u));
          w[u] = *(const cols_t*)(mine + __builtin_amdgcn_readlane(e_mine, j + u) * PITCH);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int q = 0; q < CPL; ++q) acc[q] = fmaf(dj[u], w[u][q], acc[q]);
      };
      int j = 0;
      for (; j + 8 <= k; j += 8) picks(std::integral_constant<int, 8>{}, j);
      if (j + 4 <= k) { picks(std::integral_constant<int, 4>{}, j); j += 4; }
      for (; j < k; ++j) picks(std::integral_constant<int, 1>{}, j);
      const int c = c0 + lane * CPL;
      if (c < d) __builtin_nontemporal_store(acc, (cols_t*)(dx + (size_t)t * d + c));
    }
    if (next >= groups) break;
    __syncthreads();                    // everyone is done with this group's picks
    group = next;
  }
}

}  // namespace

int launch_router_logits(const bigmac_dims& D, const void* x, const float* w_gate, const float* bias, float* logits, hipStream_t s) {
  const bool pipelined = D.N % 4 == 0 && (size_t)D.d * D.N * 4 < (1ull << 31);   // 16-byte router rows, 32-bit buffer range
  const dim3 block(256);
  const unsigned gy = (unsigned)((D.N + R_NB - 1) / R_NB);
  if (!pipelined) {
    const dim3 grid((D.T + 31) / 32, gy);
    if (D.dtype == BIGMAC_BF16) hipLaunchKernelGGL(router_logits_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)x, w_gate, bias, logits, D.T, D.d, D.N);
    else hipLaunchKernelGGL(router_logits_kernel<float>, grid, block, 0, s, (const float*)x, w_gate, bias, logits, D.T, D.d, D.N);
    BIGMAC_CHECK_LAUNCH();
    return BIGMAC_OK;
  }
  // tokens per wavefront: 8 unless that leaves most CUs without a workgroup; two expert slices per
  // workgroup while that still gives every CU two workgroups
  const long groups8 = (long)((D.T + 31) / 32) * gy;
  const int tb = groups8 >= 1024 ? 8 : (groups8 * 4 >= 512 ? 2 : 1);
  const int sl = tb == 8 && gy >= 2 && (long)((D.T + 31) / 32) * ((gy + 1) / 2) >= 512 ? ROUTER_SLICES : 1;
#define BIGMAC_ROUTER(XT, TBV, SLV)                                                                                  \
  hipLaunchKernelGGL((router_logits_pipelined_kernel<XT, TBV, SLV>),                                                  \
                     dim3((((D.T + 4 * TBV - 1) / (4 * TBV) + 7) / 8) * 8 * ((gy + SLV - 1) / SLV)), block, 0, s,     \
                     (const XT*)x, w_gate, bias, logits, D.T, D.d, D.N)
  if (D.dtype == BIGMAC_BF16) {
    if (tb == 8 && sl == 2) BIGMAC_ROUTER(bf16_t, 8, 2);
    else if (tb == 8) BIGMAC_ROUTER(bf16_t, 8, 1);
    else if (tb == 2) BIGMAC_ROUTER(bf16_t, 2, 1);
    else BIGMAC_ROUTER(bf16_t, 1, 1);
  } else {
    if (tb == 8 && sl == 2) BIGMAC_ROUTER(float, 8, 2);
    else if (tb == 8) BIGMAC_ROUTER(float, 8, 1);
    else if (tb == 2) BIGMAC_ROUTER(float, 2, 1);
    else BIGMAC_ROUTER(float, 1, 1);
  }
#undef BIGMAC_ROUTER
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

int launch_topk_gate(const bigmac_dims& D, const float* logits, int32_t* topk_idx, float* topk_w, hipStream_t s) {
  const dim3 g2((D.T + 3) / 4), block(256);
  const int per = (D.N + 63) / 64;
#define BIGMAC_TOPK(P) hipLaunchKernelGGL(topk_gate_kernel<P>, g2, block, 0, s, logits, D.T, D.N, D.k, topk_idx, topk_w)
  if (per <= 1) BIGMAC_TOPK(1);
  else if (per <= 2) BIGMAC_TOPK(2);
  else if (per <= 4) BIGMAC_TOPK(4);
  else if (per <= 8) BIGMAC_TOPK(8);
  else BIGMAC_TOPK(16);
#undef BIGMAC_TOPK
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

size_t route_backward_ws_bytes(const bigmac_dims& D) {
  // transposed router weights, or the picked entries of dL
  return align_up(std::max((size_t)D.N * D.d, (size_t)D.T * D.k) * sizeof(float));
}

__global__ void router_to_bf16_kernel(const float* __restrict__ in, bf16_t* __restrict__ out, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = f2bf(in[i]);
}

int launch_route_backward(const bigmac_dims& D, const float* w_gate, const int32_t* topk_idx,
                          const float* topk_w, const float* dgate, const float* logits, const float* share,
                          float* dx_f32, void* dL_out, void* ws, hipStream_t s) {
  // With the loss every entry of a dL row is non-zero, and the router's share of dx is the dense
  // product dL w_gate^T: on bf16 runs it goes to the matrix cores (dL is stored in bf16 anyway,
  // w_gate is rounded to bf16 for this product only); otherwise the kernel walks all N rows.
  const bool by_product = logits && D.dtype == BIGMAC_BF16 && D.N % 32 == 0;   // N is the product's K: whole k tiles
  const bool tiled = !logits && D.N <= 128 && D.k <= 64 && D.d % 4 == 0;         // w_gate rows fit the LDS tile
  float* wg_t = (float*)ws;
  if (tiled) {
    // nothing to prepare: the second kernel reads w_gate as it lies
  } else if (by_product) {
    const size_t n = (size_t)D.d * D.N;
    hipLaunchKernelGGL(router_to_bf16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, w_gate, (bf16_t*)ws, n);
  } else {
    hipLaunchKernelGGL(transpose_f32_kernel, dim3((D.N + 31) / 32, (D.d + 31) / 32), dim3(32, 8), 0, s, w_gate, wg_t, D.d, D.N);
  }
  BIGMAC_CHECK_LAUNCH();
  const dim3 grid((D.T + 3) / 4), block(256);
  const float aux_scale = logits ? D.aux_alpha * (float)D.N / (float)D.T : 0.0f;
  const int per = (D.N + 63) / 64;
  float* dx_kernel = by_product || tiled ? nullptr : dx_f32;
  float* dl_picked = tiled ? (float*)ws : nullptr;
#define BIGMAC_GATE_BWD(DT, P)                                                                                          \
  hipLaunchKernelGGL((gate_backward_kernel<DT, P>), grid, block, 0, s, topk_idx, topk_w, dgate, wg_t, logits, share, aux_scale, \
                     (DT*)dL_out, dx_kernel, dl_picked, D.T, D.d, D.N, D.k)
#define BIGMAC_GATE_BWD_PER(DT)          \
  if (per <= 1) BIGMAC_GATE_BWD(DT, 1);  \
  else if (per <= 2) BIGMAC_GATE_BWD(DT, 2); \
  else if (per <= 4) BIGMAC_GATE_BWD(DT, 4); \
  else if (per <= 8) BIGMAC_GATE_BWD(DT, 8); \
  else BIGMAC_GATE_BWD(DT, 16)
  if (D.dtype == BIGMAC_BF16) {
    BIGMAC_GATE_BWD_PER(bf16_t);
  } else {
    BIGMAC_GATE_BWD_PER(float);
  }
#undef BIGMAC_GATE_BWD_PER
#undef BIGMAC_GATE_BWD
  BIGMAC_CHECK_LAUNCH();
  if (tiled) {
    // tokens per workgroup: as many as the staging holds, fewer while the grid would leave CUs idle
    const int width = ROUTER_DX_CPL * 64;
    const unsigned gx = (unsigned)((D.d + width - 1) / width);
    int tokens = std::min(ROUTER_DX_TOKENS, ROUTER_DX_PICKS / D.k);
    while (tokens > 16 && (long)gx * ((D.T + tokens - 1) / tokens) < 256) tokens /= 2;
    // token groups per workgroup: the rows of w_gate are filled once per workgroup, so each walks
    // several groups once the grid has four workgroups per CU anyway
    unsigned gy_dx = (unsigned)((D.T + tokens - 1) / tokens);
    if ((long)gx * gy_dx > 1024) gy_dx = std::max(1u, 1024u / gx);
    const dim3 grid_dx(gx, gy_dx);
    if (D.N <= 64)
      hipLaunchKernelGGL((router_dx_kernel<ROUTER_DX_CPL, 64>), grid_dx, dim3(ROUTER_DX_THREADS), 0, s,
                         topk_idx, dl_picked, w_gate, dx_f32, D.T, D.d, D.N, D.k, tokens);
    else
      hipLaunchKernelGGL((router_dx_kernel<ROUTER_DX_CPL, 128>), grid_dx, dim3(ROUTER_DX_THREADS), 0, s,
                         topk_idx, dl_picked, w_gate, dx_f32, D.T, D.d, D.N, D.k, tokens);
    BIGMAC_CHECK_LAUNCH();
    return BIGMAC_OK;
  }
  if (by_product) {   // dx_f32[T, d] = dL[T, N] . w_gate[d, N]^T
    GemmDesc g = {};
    g.dtype = BIGMAC_BF16; g.mode = GEMM_DENSE; g.ksplit = 1;
    g.a_kcontig = 1; g.b_kcontig = 1; g.epilogue = EPI_STORE; g.out_f32 = 1;
    g.A = dL_out; g.lda = D.N; g.M = D.T; g.K = D.N;
    g.B = ws; g.ldb = D.N; g.N = D.d;
    g.C = dx_f32; g.ldc = D.d;
    return launch_gemm(g, s);
  }
  return BIGMAC_OK;
}

// Workgroups of the column-sum pass: a fixed function of T, so that the order of the sums is too.
static int aux_parts(int T) {
  const int groups = (T + 3) / 4;
  return groups < 256 ? groups : 256;
}

size_t aux_loss_ws_bytes(const bigmac_dims& D) { return align_up((size_t)aux_parts(D.T) * D.N * sizeof(float)); }

int launch_aux_loss(const bigmac_dims& D, const float* logits, const int32_t* topk_idx, float* share, float* loss,
                    float* dlogits, void* ws, hipStream_t s) {
  float* partial = (float*)ws;
  const int parts = aux_parts(D.T), per = (D.N + 63) / 64;
#define BIGMAC_AUX_PER(KERNEL, GRID, ...)                                                         \
  if (per <= 1) hipLaunchKernelGGL(KERNEL<1>, GRID, dim3(256), 0, s, __VA_ARGS__);                \
  else if (per <= 2) hipLaunchKernelGGL(KERNEL<2>, GRID, dim3(256), 0, s, __VA_ARGS__);           \
  else if (per <= 4) hipLaunchKernelGGL(KERNEL<4>, GRID, dim3(256), 0, s, __VA_ARGS__);           \
  else if (per <= 8) hipLaunchKernelGGL(KERNEL<8>, GRID, dim3(256), 0, s, __VA_ARGS__);           \
  else hipLaunchKernelGGL(KERNEL<16>, GRID, dim3(256), 0, s, __VA_ARGS__)
  BIGMAC_AUX_PER(aux_colsum_kernel, dim3(parts), logits, D.T, D.N, partial);
  BIGMAC_CHECK_LAUNCH();
  int NP = 1;
  while (NP < D.N) NP <<= 1;
  hipLaunchKernelGGL(aux_finish_kernel, dim3(1), dim3(1024), 0, s, topk_idx, partial, parts, D.T, D.N, NP, D.k, D.aux_alpha, share, loss);
  BIGMAC_CHECK_LAUNCH();
  if (dlogits) {
    const float scale = D.aux_alpha * (float)D.N / (float)D.T;
    BIGMAC_AUX_PER(aux_grad_kernel, dim3((D.T + 3) / 4), logits, share, D.T, D.N, scale, dlogits);
    BIGMAC_CHECK_LAUNCH();
  }
#undef BIGMAC_AUX_PER
  return BIGMAC_OK;
}

}  // namespace bigmac
