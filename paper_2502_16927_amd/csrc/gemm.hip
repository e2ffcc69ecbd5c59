// Matrix products of the BigMac layer on gfx950: the shared projections of Eq. 2, the expert
// matrices of Eq. 4 / Eq. 3 over ragged per-expert row ranges, and their backward products.
//
// bf16 storage: MFMA 32x32x16 bf16 tiles with fp32 accumulation.  Operand tiles are staged in LDS
// in the same orientation they have in memory (so global reads are row-contiguous for every
// transposition) with XOR swizzles against bank conflicts; operands whose contraction index is
// not the fast one in memory are fetched with the gfx950 LDS transpose read (ds_read_b64_tr_b16).
// fp32 storage: a plain tiled FMA kernel (only the tiny fp32 workload uses it).
#include "common.hpp"

namespace bigmac {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

struct TileCoord {
  int m0, n0;        // first row / column of the C tile (absolute)
  int m_end;         // rows of A and C at or beyond this are not touched
  int kbeg, kend;    // contraction range
  const void* B;     // group-resolved operand / output pointers
  void* C;
  bool valid;
};

// Works out which tile this block owns.  BM/BN: tile shape.
template <int BM, int BN>
__device__ __forceinline__ TileCoord resolve_tile(const GemmDesc& p, int esz) {
  TileCoord t;
  t.valid = true;
  t.B = p.B;
  t.C = p.C;
  t.n0 = blockIdx.x * BN;
  if (p.mode == GEMM_RAGGED_M) {
    int tile = blockIdx.y;
    if (tile >= p.tile_map[0]) { t.valid = false; return t; }
    int g = p.tile_map[1 + 2 * tile];
    t.m0 = p.tile_map[2 + 2 * tile];
    t.m_end = p.offsets[g + 1];
    t.kbeg = 0;
    t.kend = p.K;
    t.B = (const char*)p.B + (size_t)g * p.gstride_b * esz;
  } else if (p.mode == GEMM_RAGGED_K) {
    int g = blockIdx.z;
    t.m0 = blockIdx.y * BM;
    t.m_end = p.M;
    t.kbeg = p.offsets[g];
    t.kend = p.offsets[g + 1];
    t.C = (char*)p.C + (size_t)g * p.gstride_c * sizeof(float);
  } else {
    t.m0 = blockIdx.y * BM;
    t.m_end = p.M;
    int per = (p.K + p.ksplit - 1) / p.ksplit;
    per = (per + 63) / 64 * 64;
    t.kbeg = blockIdx.z * per;
    t.kend = min(p.K, t.kbeg + per);
    if (t.kend < t.kbeg) t.kend = t.kbeg;
    if (p.ksplit > 1) t.C = (char*)p.C + (size_t)blockIdx.z * p.gstride_c * sizeof(float);
  }
  return t;
}

// ------------------------------------------------------------------------ MFMA kernel ------

// 16-byte chunk index inside an LDS tile.  "kc" tiles keep k contiguous (CPR = BK/8 chunks per
// row); "tr" tiles keep the m (or n) index contiguous (CPR = BM/8 chunks per k row).
template <int CPR>
__device__ __forceinline__ int lds_chunk_kc(int row, int cc) {
  int L = row * CPR + cc;
  int line = L >> 3;
  return (line << 3) | ((L & 7) ^ (line & 7));
}
template <int CPR>
__device__ __forceinline__ int lds_chunk_tr(int krow, int cc) {
  return krow * CPR + ((((cc >> 1) ^ (krow & 3)) << 1) | (cc & 1));
}

template <int ROWS, int COLS, int THREADS, bool KC>
struct TileLoader {
  // global tile of ROWS x COLS elements (COLS contiguous), moved as 16-byte chunks
  static constexpr int CPR = COLS / 8;
  static constexpr int NCH = ROWS * COLS / 8 / THREADS;
  static_assert(ROWS * COLS / 8 % THREADS == 0, "tile does not divide over the block");
  uint4 reg[NCH];
  __device__ __forceinline__ void load(const bf16_t* base, long ld, int row0, int col0, int row_end, int col_end) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int q = i * THREADS + threadIdx.x;
      int row = q / CPR, cc = q % CPR;
      int gr = row0 + row, gc = col0 + cc * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (gr < row_end && gc < col_end) v = *(const uint4*)(base + (size_t)gr * ld + gc);
      reg[i] = v;
    }
  }
  __device__ __forceinline__ void store(uint4* lds) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int q = i * THREADS + threadIdx.x;
      int row = q / CPR, cc = q % CPR;
      int c = KC ? lds_chunk_kc<CPR>(row, cc) : lds_chunk_tr<CPR>(row, cc);
      lds[c] = reg[i];
    }
  }
};

// One 32x8 operand fragment of the 32x32x16 MFMA: lane l holds k = 8*(l/32) .. +8 of row l%32.
template <int CPR>
__device__ __forceinline__ bf16x8_t frag_kc(const uint4* lds, int rb, int ks, int lane) {
  int row = rb + (lane & 31);
  uint4 v = lds[lds_chunk_kc<CPR>(row, ks * 2 + (lane >> 5))];
  return __builtin_bit_cast(bf16x8_t, v);
}
template <int CPR>
__device__ __forceinline__ bf16x8_t frag_tr(const uint4* lds, int rb, int ks, int lane) {
  // Transposing LDS read: in each group of 16 lanes, lane i gives the address of 4 consecutive
  // elements of row (i/4) and receives column i of the resulting 4 x 16 block.
  int c = rb + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  int cc = c >> 3;
  s16x4_t part[2];
#pragma unroll
  for (int jj = 0; jj < 2; ++jj) {
    int krow = ks * 16 + (lane >> 5) * 8 + jj * 4 + ((lane & 15) >> 2);
    const char* addr = (const char*)lds + lds_chunk_tr<CPR>(krow, cc) * 16 + (c & 7) * 2;
    part[jj] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)addr);
  }
  s16x8_t v = __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8_t, v);
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool AK, bool BKC, int EPI, bool OUTF32>
__global__ __launch_bounds__(64 * WAVES_M* WAVES_N) void mfma_gemm_kernel(GemmDesc p) {
  constexpr int THREADS = 64 * WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_CHUNKS = BM * BK / 8, B_CHUNKS = BN * BK / 8;
  __shared__ uint4 lds_a[2][A_CHUNKS];
  __shared__ uint4 lds_b[2][B_CHUNKS];

  TileCoord t = resolve_tile<BM, BN>(p, 2);
  if (!t.valid) return;
  const bf16_t* A = (const bf16_t*)p.A;
  const bf16_t* B = (const bf16_t*)t.B;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave / WAVES_N) * WM, wn = (wave % WAVES_N) * WN;

  using LoadA = TileLoader<AK ? BM : BK, AK ? BK : BM, THREADS, AK>;
  using LoadB = TileLoader<BKC ? BN : BK, BKC ? BK : BN, THREADS, BKC>;
  LoadA la;
  LoadB lb;
  auto fetch = [&](int kt) {
    int kb = p.kwrap_b ? kt % p.kwrap_b : kt;
    int kb_end = p.kwrap_b ? kb + (t.kend - kt) : t.kend;
    if (AK) la.load(A, p.lda, t.m0, kt, t.m_end, t.kend);
    else    la.load(A, p.lda, kt, t.m0, t.kend, p.M);
    if (BKC) lb.load(B, p.ldb, t.n0, kb, p.N, kb_end);
    else     lb.load(B, p.ldb, kb, t.n0, kb_end, p.N);
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int nk = (t.kend - t.kbeg + BK - 1) / BK;
  if (nk > 0) {
    fetch(t.kbeg);
    la.store(lds_a[0]);
    lb.store(lds_b[0]);
  }
  __syncthreads();
  for (int it = 0; it < nk; ++it) {
    const int cur = it & 1;
    if (it + 1 < nk) fetch(t.kbeg + (it + 1) * BK);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8_t fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = AK ? frag_kc<BK / 8>(lds_a[cur], wm + i * 32, ks, lane) : frag_tr<BM / 8>(lds_a[cur], wm + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = BKC ? frag_kc<BK / 8>(lds_b[cur], wn + j * 32, ks, lane) : frag_tr<BN / 8>(lds_b[cur], wn + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (it + 1 < nk) {
      la.store(lds_a[cur ^ 1]);
      lb.store(lds_b[cur ^ 1]);
    }
    __syncthreads();
  }

  // epilogue: lane l of a 32x32 tile holds column l%32, rows 8*(v/4) + 4*(l/32) + v%4
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = t.n0 + wn + j * 32 + (lane & 31);
      if (col >= p.N) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = t.m0 + wm + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (row >= t.m_end) continue;
        const size_t off = (size_t)row * p.ldc + col;
        const float a = acc[i][j][v];
        if (EPI == EPI_STORE) {
          if (OUTF32) ((float*)t.C)[off] = a;
          else ((bf16_t*)t.C)[off] = f2bf(a);
        } else if (EPI == EPI_GELU) {
          if (p.aux_out) ((bf16_t*)p.aux_out)[off] = f2bf(a);
          ((bf16_t*)t.C)[off] = f2bf(gelu_f(a));
        } else if (EPI == EPI_DGELU) {
          ((bf16_t*)t.C)[off] = f2bf(a * gelu_grad_f(bf2f(((const bf16_t*)p.aux_in)[off])));
        } else {
          float* c = (float*)t.C + off;
          *c = p.beta ? *c + a : a;
        }
      }
    }
}

// ------------------------------------------------------------------------ fp32 kernel ------

template <bool AK, bool BKC, int EPI>
__global__ __launch_bounds__(256) void fma_gemm_kernel(GemmDesc p) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float sa[BK][BM + 1];
  __shared__ float sb[BK][BN + 1];
  TileCoord t = resolve_tile<BM, BN>(p, 4);
  if (!t.valid) return;
  const float* A = (const float*)p.A;
  const float* B = (const float*)t.B;
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  float acc[4][4] = {};
  for (int kt = t.kbeg; kt < t.kend; kt += BK) {
    const int kb = p.kwrap_b ? kt % p.kwrap_b : kt;
    for (int e = tid; e < BM * BK; e += 256) {
      int m = AK ? e / BK : e % BM, kk = AK ? e % BK : e / BM;
      int gm = t.m0 + m, gk = kt + kk;
      float v = 0.0f;
      if (gm < t.m_end && gk < t.kend) v = AK ? A[(size_t)gm * p.lda + gk] : A[(size_t)gk * p.lda + gm];
      sa[kk][m] = v;
    }
    for (int e = tid; e < BN * BK; e += 256) {
      int n = BKC ? e / BK : e % BN, kk = BKC ? e % BK : e / BN;
      int gn = t.n0 + n, gk = kt + kk;
      float v = 0.0f;
      if (gn < p.N && gk < t.kend) v = BKC ? B[(size_t)gn * p.ldb + kb + kk] : B[(size_t)(kb + kk) * p.ldb + gn];
      sb[kk][n] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = sa[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = sb[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = t.m0 + ty * 4 + i, col = t.n0 + tx * 4 + j;
      if (row >= t.m_end || col >= p.N) continue;
      const size_t off = (size_t)row * p.ldc + col;
      const float a = acc[i][j];
      float* c = (float*)t.C + off;
      if (EPI == EPI_STORE) *c = a;
      else if (EPI == EPI_GELU) {
        if (p.aux_out) ((float*)p.aux_out)[off] = a;
        *c = gelu_f(a);
      } else if (EPI == EPI_DGELU) *c = a * gelu_grad_f(((const float*)p.aux_in)[off]);
      else *c = p.beta ? *c + a : a;
    }
}

// ------------------------------------------------------------------------ helpers ----------

// tile_map[0] = number of M tiles; then (group, first row) per tile, groups in order.
__global__ void build_tile_map_kernel(const int* __restrict__ offsets, int groups, int tile_rows, int* __restrict__ tile_map) {
  __shared__ int scan[1024];
  const int g = threadIdx.x;
  int beg = 0, cnt = 0;
  if (g < groups) {
    beg = offsets[g];
    cnt = (offsets[g + 1] - beg + tile_rows - 1) / tile_rows;
  }
  scan[g] = cnt;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    int v = g >= off ? scan[g - off] : 0;
    __syncthreads();
    scan[g] += v;
    __syncthreads();
  }
  const int first = scan[g] - cnt;
  for (int i = 0; i < cnt; ++i) {
    tile_map[1 + 2 * (first + i)] = g;
    tile_map[2 + 2 * (first + i)] = beg + i * tile_rows;
  }
  if (g == 1023) tile_map[0] = scan[1023];
}

__global__ void reduce_partials_kernel(const float* __restrict__ part, int nslices, size_t n, float* __restrict__ out, int beta) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = beta ? out[i] : 0.0f;
  for (int z = 0; z < nslices; ++z) s += part[(size_t)z * n + i];
  out[i] = s;
}

int gemm_ragged_tile_rows(int dtype) { return dtype == BIGMAC_BF16 ? 128 : 64; }

int launch_build_tile_map(const int* offsets, int groups, int tile_rows, int* tile_map, hipStream_t s) {
  if (groups > 1024) return BIGMAC_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(build_tile_map_kernel, dim3(1), dim3(1024), 0, s, offsets, groups, tile_rows, tile_map);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

int launch_reduce_partials(const float* part, int nslices, size_t n, float* out, int beta, hipStream_t s) {
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, part, nslices, n, out, beta);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

namespace {

template <int BM, int BN>
dim3 grid_for(const GemmDesc& g) {
  unsigned gx = (g.N + BN - 1) / BN;
  if (g.mode == GEMM_RAGGED_M) return dim3(gx, (unsigned)(g.max_rows / BM + g.groups + 1), 1);
  unsigned gy = (g.M + BM - 1) / BM;
  if (g.mode == GEMM_RAGGED_K) return dim3(gx, gy, g.groups);
  return dim3(gx, gy, g.ksplit);
}

template <bool AK, bool BKC>
int launch_mfma(const GemmDesc& g, hipStream_t s) {
  constexpr int BM = 128, BN = 128, BK = 64, WMs = 2, WNs = 2;
  dim3 grid = grid_for<BM, BN>(g), block(64 * WMs * WNs);
#define BIGMAC_MFMA(EPI, OUTF32) \
  hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, WMs, WNs, AK, BKC, EPI, OUTF32>), grid, block, 0, s, g)
  switch (g.epilogue) {
    case EPI_STORE:
      if (g.out_f32) BIGMAC_MFMA(EPI_STORE, true);
      else BIGMAC_MFMA(EPI_STORE, false);
      break;
    case EPI_GELU: BIGMAC_MFMA(EPI_GELU, false); break;
    case EPI_DGELU: BIGMAC_MFMA(EPI_DGELU, false); break;
    case EPI_ACCUM: BIGMAC_MFMA(EPI_ACCUM, true); break;
    default: return BIGMAC_ERR_INVALID_ARG;
  }
#undef BIGMAC_MFMA
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

template <bool AK, bool BKC>
int launch_fma(const GemmDesc& g, hipStream_t s) {
  dim3 grid = grid_for<64, 64>(g), block(256);
  switch (g.epilogue) {
    case EPI_STORE: hipLaunchKernelGGL((fma_gemm_kernel<AK, BKC, EPI_STORE>), grid, block, 0, s, g); break;
    case EPI_GELU: hipLaunchKernelGGL((fma_gemm_kernel<AK, BKC, EPI_GELU>), grid, block, 0, s, g); break;
    case EPI_DGELU: hipLaunchKernelGGL((fma_gemm_kernel<AK, BKC, EPI_DGELU>), grid, block, 0, s, g); break;
    case EPI_ACCUM: hipLaunchKernelGGL((fma_gemm_kernel<AK, BKC, EPI_ACCUM>), grid, block, 0, s, g); break;
    default: return BIGMAC_ERR_INVALID_ARG;
  }
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

}  // namespace

int launch_gemm(const GemmDesc& g, hipStream_t s) {
  // host-side shape checks: the kernels move 16-byte chunks and 64-wide k tiles
  if (g.N <= 0 || (g.mode != GEMM_RAGGED_M && g.M <= 0) || (g.mode != GEMM_RAGGED_K && g.K <= 0)) return BIGMAC_ERR_INVALID_ARG;
  if (g.mode != GEMM_DENSE && (!g.offsets || g.groups <= 0)) return BIGMAC_ERR_INVALID_ARG;
  if (g.mode == GEMM_RAGGED_M && !g.tile_map) return BIGMAC_ERR_INVALID_ARG;
  if (g.dtype == BIGMAC_BF16) {
    if (g.lda % 8 || g.ldb % 8 || g.N % 8 || ((g.a_kcontig || g.b_kcontig) && g.K % 8) ||
        (g.mode != GEMM_RAGGED_M && !g.a_kcontig && g.M % 8) || g.kwrap_b % 64)
      return BIGMAC_ERR_INVALID_ARG;
    if ((g.a_kcontig || g.b_kcontig) && g.mode == GEMM_RAGGED_K) return BIGMAC_ERR_UNSUPPORTED;  // k ranges start anywhere
  }
  if (g.mode == GEMM_DENSE && g.ksplit < 1) return BIGMAC_ERR_INVALID_ARG;
  const int combo = g.a_kcontig * 2 + g.b_kcontig;
  if (g.dtype == BIGMAC_BF16) {
    switch (combo) {
      case 2: return launch_mfma<true, false>(g, s);
      case 3: return launch_mfma<true, true>(g, s);
      case 0: return launch_mfma<false, false>(g, s);
      default: return BIGMAC_ERR_UNSUPPORTED;
    }
  }
  switch (combo) {
    case 2: return launch_fma<true, false>(g, s);
    case 3: return launch_fma<true, true>(g, s);
    case 0: return launch_fma<false, false>(g, s);
    default: return BIGMAC_ERR_UNSUPPORTED;
  }
}

}  // namespace bigmac
