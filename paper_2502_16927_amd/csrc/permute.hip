// The two All-to-Alls of the layer (Section 3.1) as on-device permutes of win-wide rows:
// a stable counting sort of the (token, choice) pairs by expert, a row scatter (dispatch), a
// weighted row gather-sum (combine, the middle term of Eq. 2) and their backward forms.
// Slot assignment uses no atomics whose order could matter: counts are order-free, ranks come
// from ballots inside one wavefront walking its chunk in order.
#include "common.hpp"
#include "tile_map.hpp"

#include <atomic>

// Scratch of the allocation-free dispatch (bigmac_dispatch_static): the per-chunk expert counters
// of the counting sort.  One copy per GPU the library runs on, held until the process ends.
#define BIGMAC_STATIC_SCRATCH_BYTES (4u << 20)
static __device__ __align__(256) unsigned char scratch[BIGMAC_STATIC_SCRATCH_BYTES];

namespace bigmac {

namespace {

// Flat pairs per chunk of the counting sort: small chunks give the count and rank kernels more
// workgroups, but the one-workgroup scan walks chunks x experts counters; 256 while those stay
// below 32768 (gpt_medium: permutation 26.6 -> 23.6 us), else 1024.
constexpr int P_CHUNK_SMALL = 256, P_CHUNK_LARGE = 1024;
inline int perm_chunk(int Tk, int N) { return (size_t)((Tk + P_CHUNK_SMALL - 1) / P_CHUNK_SMALL) * N <= 32768 ? P_CHUNK_SMALL : P_CHUNK_LARGE; }

// counts[c][e] = number of pairs of chunk c routed to expert e
__global__ __launch_bounds__(256) void perm_count_kernel(const int32_t* __restrict__ idx, int Tk, int N, int chunk, int32_t* __restrict__ counts) {
  extern __shared__ int cnt[];
  for (int e = threadIdx.x; e < N; e += 256) cnt[e] = 0;
  __syncthreads();
  const int base = blockIdx.x * chunk;
  for (int i = threadIdx.x; i < chunk; i += 256) {
    const int f = base + i;
    if (f < Tk) atomicAdd(&cnt[idx[f]], 1);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < N; e += 256) counts[(size_t)blockIdx.x * N + e] = cnt[e];
}

// Inclusive scan over the 1024 threads of a workgroup: shuffles inside each wavefront, the 16
// wavefront totals through LDS.
__device__ __forceinline__ int block_scan_1024(int v, int* wave_totals) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(v, d, 64);
    if (lane >= d) v += o;
  }
  __syncthreads();                 // wave_totals may still be read from a previous call
  if (lane == 63) wave_totals[wave] = v;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += wave_totals[w];
  return v + before;
}

// in place: counts[c][e] -> first slot of expert e's pairs of chunk c;  offsets[e] = first slot of e.
// With a capacity (> 0) an expert's range holds at most that many slots; the per-chunk first
// slots still count every pair in front, so a pair is past its expert's range exactly when its
// slot reaches offsets[e] + capacity.
// The 1024 threads are G groups x NP experts (NP = N rounded up to a power of two, G = 1024 / NP);
// group g owns a contiguous range of chunks, so all chunk rows are read by many threads at once.
// At the end the workgroup also builds the tile maps asked for: the offsets are at hand, and a
// kernel of their own would cost a launch and a round trip through memory.
__global__ __launch_bounds__(1024) void perm_scan_kernel(int32_t* __restrict__ counts, int nchunks, int N, int NP, int capacity,
                                                         int32_t* __restrict__ offsets, TileMapJobs maps) {
  __shared__ int part[1024];        // [g][e]: pairs of expert e in the chunks of group g
  __shared__ int wave_totals[16];
  __shared__ int first_slot[1025];  // offsets[0 .. N], for the tile maps
  const int G = 1024 / NP;
  const int e = threadIdx.x % NP, g = threadIdx.x / NP;
  const int per = (nchunks + G - 1) / G;
  const int c_beg = min(g * per, nchunks), c_end = min(c_beg + per, nchunks);
  int mine = 0;
  if (e < N)
    for (int c0 = c_beg; c0 < c_end; c0 += 8) {
      int v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = c0 + u < c_end ? counts[(size_t)(c0 + u) * N + e] : 0;
#pragma unroll
      for (int u = 0; u < 8; ++u) mine += v[u];
    }
  part[g * NP + e] = mine;
  __syncthreads();
  int total = 0, before_me = 0;      // expert e: all pairs, and those in the groups in front of g
  for (int h = 0; h < G; ++h) {
    const int v = part[h * NP + e];
    total += v;
    if (h < g) before_me += v;
  }
  // exclusive scan over the experts (threads of group 0 carry the totals, the others zero)
  const int held = capacity > 0 ? min(total, capacity) : total;   // slots of expert e
  const int incl = block_scan_1024(g == 0 && e < N ? held : 0, wave_totals);
  __syncthreads();
  if (g == 0) part[e] = incl - held;    // first slot of expert e (part[0 .. NP) is free to reuse: every thread has read it)
  __syncthreads();
  if (e < N) {
    int run = part[e] + before_me;
    if (g == 0) offsets[e] = first_slot[e] = part[e];
    if (g == 0 && e == N - 1) offsets[N] = first_slot[N] = part[e] + held;
    for (int c0 = c_beg; c0 < c_end; c0 += 8) {
      int v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = c0 + u < c_end ? counts[(size_t)(c0 + u) * N + e] : 0;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u < c_end) counts[(size_t)(c0 + u) * N + e] = run;
        run += v[u];
      }
    }
  }
  __syncthreads();
  if (maps.map[0]) build_tile_map_block(first_slot, N, maps.tile_rows[0], maps.map[0]);
  if (maps.map[1]) build_tile_map_block(first_slot, N, maps.tile_rows[1], maps.map[1], maps.map[0]);
}

// One wavefront per chunk walks its pairs in flat order, 64 at a time (all read up front).  A
// pair's slot is the running first-free slot of its expert plus the number of earlier lanes with
// the same expert.  With a capacity, a pair whose slot falls past its expert's range is dropped:
// slot_of = -1, no src_of entry.
template <int ROUNDS>   // chunk = 64 * ROUNDS pairs
__global__ __launch_bounds__(64) void perm_rank_kernel(const int32_t* __restrict__ idx, int Tk, int N, int nbits, int capacity,
                                                       const int32_t* __restrict__ base, const int32_t* __restrict__ offsets,
                                                       int32_t* __restrict__ slot_of, int32_t* __restrict__ src_of) {
  extern __shared__ int run[];      // [N] running first-free slot, [N] end of the expert's range
  const int lane = threadIdx.x;
  constexpr int P_CHUNK = 64 * ROUNDS;
  int mine[ROUNDS];
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const int f = blockIdx.x * P_CHUNK + r * 64 + lane;
    mine[r] = f < Tk ? idx[f] : -1;
  }
  int* range_end = run + N;
  for (int e = lane; e < N; e += 64) {
    run[e] = base[(size_t)blockIdx.x * N + e];
    range_end[e] = capacity > 0 ? offsets[e] + capacity : 0x7fffffff;
  }
  __syncthreads();
  const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const int f = blockIdx.x * P_CHUNK + r * 64 + lane;
    const bool live = mine[r] >= 0;
    const int e = live ? mine[r] : 0;
    unsigned long long same = __ballot(live);
    for (int b = 0; b < nbits; ++b) {
      const unsigned long long bal = __ballot((e >> b) & 1);
      same &= ((e >> b) & 1) ? bal : ~bal;
    }
    if (live) {
      const int slot = run[e] + __popcll(same & below);
      if (slot < range_end[e]) {
        slot_of[f] = slot;
        src_of[slot] = f;
      } else {
        slot_of[f] = -1;
      }
    }
    __syncthreads();
    if (live && (same >> lane) == 1ull) run[e] += __popcll(same);  // highest lane of each expert group
    __syncthreads();
  }
}

// The whole counting sort for a few pairs (decode batches) in one workgroup of 1024 threads:
// pair f = (round, wavefront, lane) in flat order; per (round, wavefront) the pairs of each expert
// are counted by ballots (one writer per counter, no atomics), the counters are scanned per expert
// in that same order, and a pair's slot is its expert's first slot + the pairs of the expert in
// earlier (round, wavefront) groups + the earlier lanes of its own group with the same expert.
// The same slots as the three-kernel form; also writes the offsets and the tile maps.
constexpr int PS_MAX_ROUNDS = 4;            // up to 4096 pairs
constexpr int PS_MAX_COUNTERS = 8192;       // rounds x 16 wavefronts x experts, 32 KB of LDS
template <int ROUNDS>
__global__ __launch_bounds__(1024) void perm_small_kernel(const int32_t* __restrict__ idx, int Tk, int N, int nbits, int capacity,
                                                          int32_t* __restrict__ offsets, int32_t* __restrict__ slot_of,
                                                          int32_t* __restrict__ src_of, TileMapJobs maps) {
  __shared__ int cnt[PS_MAX_COUNTERS];   // [round][wavefront][expert]
  __shared__ int wave_totals[16];
  __shared__ int first_slot[1025];
  __shared__ int range_end[1024];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < ROUNDS * 16 * N; i += 1024) cnt[i] = 0;
  __syncthreads();
  const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  int mine[ROUNDS], rank[ROUNDS];
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const int f = r * 1024 + tid;
    mine[r] = f < Tk ? idx[f] : -1;
    const bool live = mine[r] >= 0;
    const int e = live ? mine[r] : 0;
    unsigned long long same = __ballot(live);
    for (int b = 0; b < nbits; ++b) {
      const unsigned long long bal = __ballot((e >> b) & 1);
      same &= ((e >> b) & 1) ? bal : ~bal;
    }
    rank[r] = __popcll(same & below);
    if (live && (same >> lane) == 1ull) cnt[(r * 16 + wave) * N + e] = __popcll(same);   // highest lane of each expert group
  }
  __syncthreads();
  int total = 0;
  if (tid < N)
    for (int g = 0; g < ROUNDS * 16; ++g) {      // counters -> pairs of the expert in earlier groups
      const int c = cnt[g * N + tid];
      cnt[g * N + tid] = total;
      total += c;
    }
  const int held = capacity > 0 ? min(total, capacity) : total;
  const int incl = block_scan_1024(tid < N ? held : 0, wave_totals);
  if (tid < N) {
    offsets[tid] = first_slot[tid] = incl - held;
    range_end[tid] = incl;
    if (tid == N - 1) offsets[N] = first_slot[N] = incl;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const int f = r * 1024 + tid;
    if (mine[r] >= 0) {
      const int e = mine[r];
      const int slot = first_slot[e] + cnt[(r * 16 + wave) * N + e] + rank[r];
      if (slot < range_end[e]) {
        slot_of[f] = slot;
        src_of[slot] = f;
      } else {
        slot_of[f] = -1;
      }
    }
  }
  if (maps.map[0]) build_tile_map_block(first_slot, N, maps.tile_rows[0], maps.map[0]);
  if (maps.map[1]) build_tile_map_block(first_slot, N, maps.tile_rows[1], maps.map[1], maps.map[0]);
}

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
// 16-byte chunks: thread (t, c) copies chunk c of row t to its k destination rows
__global__ __launch_bounds__(256) void dispatch_rows_kernel(const uint4* __restrict__ x_low, const int32_t* __restrict__ slot_of,
                                                            uint4* __restrict__ x_perm, int T, int k, int cpr) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= (size_t)T * cpr) return;
  const int t = (int)(g / cpr), c = (int)(g % cpr);
  const uint4 v = x_low[g];
  for (int j = 0; j < k; ++j) {
    const int slot = slot_of[(size_t)t * k + j];
    if (slot >= 0) x_perm[(size_t)slot * cpr + c] = v;   // a dropped pair has no row
  }
}

// Rows that are read exactly once (the permuted expert outputs and gradients): loaded with the
// non-temporal hint so that they do not push the rows still to come out of the caches.
__device__ __forceinline__ void load_row8(const float* p, float* f) {
  const f32x4_t a = __builtin_nontemporal_load((const f32x4_t*)p), b = __builtin_nontemporal_load((const f32x4_t*)p + 1);
  f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
}
__device__ __forceinline__ void load_row8(const bf16_t* p, float* f) {
  const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)p);
  uint4 q;
  q.x = v.x; q.y = v.y; q.z = v.z; q.w = v.w;
  unpack_bf16x8(q, f);
}

// y_low[t] = sum_j w[t,j] * o_perm[slot_of[t,j]], j ascending, fp32.  Thread = (token, 8 columns).
// The k picks are taken KU at a time (KU divides k): their slots and weights are read first, then
// all KU row pieces are requested before the first multiply-add, so that a thread has KU
// independent gathers in flight instead of a chain of dependent ones.  A dropped pair
// (slot < 0) reads row 0 and is left out of the sum.  ROW: element type of the gathered rows.
// UNIFORM (rows of a multiple of 512 columns): a wavefront's 64 threads all belong to one token, so
// its slots and weights are read once per wavefront by scalar loads instead of by every thread.
typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr_t;
typedef const float __attribute__((address_space(4))) * const_f32_ptr_t;
template <typename ROW, int OUT, int KU, bool UNIFORM>
__global__ __launch_bounds__(256) void combine_rows_kernel(const ROW* __restrict__ o_perm, const int32_t* __restrict__ slot_of,
                                                           const float* __restrict__ w, const float* __restrict__ addend,
                                                           void* __restrict__ y, int T, int k, int width, int stream_out) {
  const int cpr = width / 8;
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= (size_t)T * cpr) return;
  int t = (int)(g / cpr);
  const int c = (int)(g % cpr);
  if (UNIFORM) t = __builtin_amdgcn_readfirstlane(t);
  float acc[8] = {};
  if (addend) {   // the sum starts from a row of its own ([T, width] fp32) instead of zero
    const float4 a = *(const float4*)(addend + (size_t)t * width + c * 8), b = *(const float4*)(addend + (size_t)t * width + c * 8 + 4);
    acc[0] = a.x; acc[1] = a.y; acc[2] = a.z; acc[3] = a.w; acc[4] = b.x; acc[5] = b.y; acc[6] = b.z; acc[7] = b.w;
  }
  for (int j0 = 0; j0 < k; j0 += KU) {
    int slot[KU];
    float wj[KU];
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      if (UNIFORM) {   // the tables are written before this kernel starts and only read by it
        slot[u] = ((const_i32_ptr_t)(unsigned long long)slot_of)[(size_t)t * k + j0 + u];
        wj[u] = w ? ((const_f32_ptr_t)(unsigned long long)w)[(size_t)t * k + j0 + u] : 1.0f;
      } else {
        slot[u] = slot_of[(size_t)t * k + j0 + u];
        wj[u] = w ? w[(size_t)t * k + j0 + u] : 1.0f;
      }
    }
    float o[KU][8];
#pragma unroll
    for (int u = 0; u < KU; ++u) load_row8(o_perm + (size_t)max(slot[u], 0) * width + c * 8, o[u]);
#pragma unroll
    for (int u = 0; u < KU; ++u)
      if (slot[u] >= 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = fmaf(wj[u], o[u][i], acc[i]);
      }
  }
  if (OUT == COMBINE_F32) {
    float4* out = (float4*)((float*)y + (size_t)t * width + c * 8);
    out[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    out[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
  } else {  // bf16 (hi | lo): acc = hi + lo up to 2^-17 relative
    float lo[8];
    uint4 hi = pack_bf16x8(acc);
    float hf[8];
    unpack_bf16x8(hi, hf);
#pragma unroll
    for (int i = 0; i < 8; ++i) lo[i] = acc[i] - hf[i];
    uint4* out = (uint4*)((bf16_t*)y + (size_t)t * 2 * width);
    const uint4 lo_p = pack_bf16x8(lo);
    if (stream_out) {   // the caller's choice: see launch_combine_rows
      __builtin_nontemporal_store(*(const u32x4_t*)&hi, (u32x4_t*)(out + c));
      __builtin_nontemporal_store(*(const u32x4_t*)&lo_p, (u32x4_t*)(out + cpr + c));
    } else {
      out[c] = hi;
      out[cpr + c] = lo_p;
    }
  }
}

// One wavefront per token: dgate[t,j] = <dy_low[t], o_perm[slot]>; do_perm[slot] = w[t,j] * dy_low[t].
// OT: element type of the expert outputs, DT: of the scattered gradient rows.
template <typename OT, typename DT>
__global__ __launch_bounds__(256) void combine_backward_kernel(const float* __restrict__ dy_low, const OT* __restrict__ o_perm,
                                                               const int32_t* __restrict__ slot_of, const float* __restrict__ w,
                                                               float* __restrict__ dgate, DT* __restrict__ do_perm, int T, int k, int width) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  for (int j = 0; j < k; ++j) {
    const int slot_j = slot_of[(size_t)t * k + j];
    if (slot_j < 0) {                           // dropped pair (the same in every lane): no row, no gate gradient
      if (lane == 0) dgate[(size_t)t * k + j] = 0.0f;
      continue;
    }
    const size_t slot = (size_t)slot_j;
    const float wj = w[(size_t)t * k + j];
    float dot = 0.0f;
    for (int c0 = 0; c0 < width; c0 += 256) {
      const int c = c0 + lane * 4;
      if (c < width) {
        const float4 g = *(const float4*)(dy_low + (size_t)t * width + c);
        const OT* o = o_perm + slot * width + c;
        DT* q = do_perm + slot * width + c;
        dot = fmaf(g.x, Elem<OT>::load(o + 0), dot); dot = fmaf(g.y, Elem<OT>::load(o + 1), dot);
        dot = fmaf(g.z, Elem<OT>::load(o + 2), dot); dot = fmaf(g.w, Elem<OT>::load(o + 3), dot);
        Elem<DT>::store(q + 0, wj * g.x); Elem<DT>::store(q + 1, wj * g.y);
        Elem<DT>::store(q + 2, wj * g.z); Elem<DT>::store(q + 3, wj * g.w);
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, 64);
    if (lane == 0) dgate[(size_t)t * k + j] = dot;
  }
}

// The same for bf16 gradient rows at least 512 wide: 16-byte accesses of 8 columns per lane, the
// picks taken KU at a time (KU divides k) with all KU pieces of the expert outputs requested
// before the first multiply-add; the token's dy' piece is read once per group of picks.
template <typename OT, int KU>
__global__ __launch_bounds__(256) void combine_backward_wide_kernel(const float* __restrict__ dy_low, const OT* __restrict__ o_perm,
                                                                    const int32_t* __restrict__ slot_of, const float* __restrict__ w,
                                                                    float* __restrict__ dgate, bf16_t* __restrict__ do_perm, int T, int k, int width) {
  const int lane = threadIdx.x & 63;
  const int t = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  if (t >= T) return;
  for (int j0 = 0; j0 < k; j0 += KU) {
    int slot[KU];
    float wj[KU], dot[KU];
#pragma unroll
    for (int u = 0; u < KU; ++u) {   // one token per wavefront: its slots and weights by scalar loads
      slot[u] = ((const_i32_ptr_t)(unsigned long long)slot_of)[(size_t)t * k + j0 + u];
      wj[u] = ((const_f32_ptr_t)(unsigned long long)w)[(size_t)t * k + j0 + u];
      dot[u] = 0.0f;
    }
    for (int c0 = 0; c0 < width; c0 += 512) {
      const int c = c0 + lane * 8;
      if (c < width) {
        float g[8];
        const float4 g0 = *(const float4*)(dy_low + (size_t)t * width + c), g1 = *(const float4*)(dy_low + (size_t)t * width + c + 4);
        g[0] = g0.x; g[1] = g0.y; g[2] = g0.z; g[3] = g0.w; g[4] = g1.x; g[5] = g1.y; g[6] = g1.z; g[7] = g1.w;
        float o[KU][8];
#pragma unroll
        for (int u = 0; u < KU; ++u) load_row8(o_perm + (size_t)max(slot[u], 0) * width + c, o[u]);
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          if (slot[u] < 0) continue;              // a dropped pair has no row; its dot stays 0
          float q[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            dot[u] = fmaf(g[i], o[u][i], dot[u]);
            q[i] = wj[u] * g[i];
          }
          *(uint4*)(do_perm + (size_t)slot[u] * width + c) = pack_bf16x8(q);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      float d = dot[u];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) d += __shfl_xor(d, off, 64);
      if (lane == 0) dgate[(size_t)t * k + j0 + u] = d;
    }
  }
}

// Column sums over each group's rows (the gradients of the expert biases): part[(g * S + z), c] =
// sum of src[s, c] over the z-th of S equal pieces of group g's row range.  A workgroup takes 64
// columns of one piece: 32 row lanes x 8 column groups of 8 columns (16-byte reads of bf16), the
// row lanes walk the piece 32 rows at a time and are added up through the LDS in lane order, so
// that equal inputs give equal bits.
constexpr int COLSUM_SPLIT = 8;
template <typename ET>
__global__ __launch_bounds__(256) void ragged_colsum_kernel(const ET* __restrict__ src, long ld, int cols, const int32_t* __restrict__ offsets,
                                                            float* __restrict__ part) {
  __shared__ float sums[32][65];
  const int g = blockIdx.y, z = blockIdx.z;
  const int rl = threadIdx.x >> 3, cg = threadIdx.x & 7;
  const int c0 = blockIdx.x * 64 + cg * 8;
  const int beg = offsets[g], end = offsets[g + 1];
  const int piece = ((end - beg + COLSUM_SPLIT - 1) / COLSUM_SPLIT + 31) / 32 * 32;
  const int r0 = beg + z * piece, r1 = min(end, r0 + piece);
  float acc[8] = {};
  if (c0 < cols)
    for (int r = r0 + rl; r < r1; r += 32) {
      float v[8];
      const ET* p = src + (size_t)r * ld + c0;
      if (sizeof(ET) == 2) unpack_bf16x8(*(const uint4*)p, v);
      else {
        const float4 a = *(const float4*)p, b = *((const float4*)p + 1);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += v[i];
    }
#pragma unroll
  for (int i = 0; i < 8; ++i) sums[rl][cg * 8 + i] = acc[i];
  __syncthreads();
  if (threadIdx.x < 64) {
    const int c = blockIdx.x * 64 + threadIdx.x;
    float s = 0.0f;
    for (int l = 0; l < 32; ++l) s += sums[l][threadIdx.x];
    if (c < cols) part[((size_t)g * COLSUM_SPLIT + z) * cols + c] = s;
  }
}
// out[g, c] = (beta ? out : 0) + sum_z part[(g * S + z), c], z ascending
__global__ void colsum_reduce_kernel(const float* __restrict__ part, size_t n, int cols, float* __restrict__ out, int beta) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const size_t g = i / cols, c = i % cols;
  float s = beta ? out[i] : 0.0f;
  for (int z = 0; z < COLSUM_SPLIT; ++z) s += part[(g * COLSUM_SPLIT + z) * cols + c];
  out[i] = s;
}

}  // namespace

size_t ragged_colsum_ws_bytes(int groups, int cols) { return align_up((size_t)groups * COLSUM_SPLIT * cols * sizeof(float)); }

int launch_ragged_colsum(int dtype, const void* src, long ld, int cols, const int32_t* offsets, int groups, float* out, int beta,
                         void* ws, hipStream_t s) {
  if (cols % 8 || ld % 8) return BIGMAC_ERR_INVALID_ARG;
  const dim3 grid((cols + 63) / 64, groups, COLSUM_SPLIT), block(256);
  if (dtype == BIGMAC_BF16)
    hipLaunchKernelGGL(ragged_colsum_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)src, ld, cols, offsets, (float*)ws);
  else
    hipLaunchKernelGGL(ragged_colsum_kernel<float>, grid, block, 0, s, (const float*)src, ld, cols, offsets, (float*)ws);
  BIGMAC_CHECK_LAUNCH();
  const size_t n = (size_t)groups * cols;
  hipLaunchKernelGGL(colsum_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const float*)ws, n, cols, out, beta);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

size_t permutation_ws_bytes(int T, int k, int N) {
  const int chunk = perm_chunk(T * k, N);
  const size_t nchunks = ((size_t)T * k + chunk - 1) / chunk;
  return align_up(nchunks * N * sizeof(int32_t));
}

int launch_build_permutation(int T, int k, int N, int capacity, const int32_t* topk_idx, int32_t* expert_offsets,
                             int32_t* slot_of, int32_t* src_of, void* ws, hipStream_t s, const TileMapJobs* tile_maps) {
  if (N > 1024) return BIGMAC_ERR_UNSUPPORTED;   // one thread of the scan per expert
  const TileMapJobs maps = tile_maps ? *tile_maps : TileMapJobs{};
  {
    const int need = (T * k + 1023) / 1024;
    const int rounds = need <= 1 ? 1 : (need == 2 ? 2 : 4);           // the instantiated round counts
    if (need <= PS_MAX_ROUNDS && rounds * 16 * N <= PS_MAX_COUNTERS) {
      int bits = 0;
      while ((1 << bits) < N) ++bits;
#define BIGMAC_PERM_SMALL(R) \
  hipLaunchKernelGGL(perm_small_kernel<R>, dim3(1), dim3(1024), 0, s, topk_idx, T * k, N, bits, capacity, expert_offsets, slot_of, src_of, maps)
      if (rounds == 1) BIGMAC_PERM_SMALL(1);
      else if (rounds == 2) BIGMAC_PERM_SMALL(2);
      else BIGMAC_PERM_SMALL(4);
#undef BIGMAC_PERM_SMALL
      BIGMAC_CHECK_LAUNCH();
      return BIGMAC_OK;
    }
  }
  const int Tk = T * k;
  const int chunk = perm_chunk(Tk, N);
  const int nchunks = (Tk + chunk - 1) / chunk;
  int nbits = 0;
  while ((1 << nbits) < N) ++nbits;
  int32_t* counts = (int32_t*)ws;
  hipLaunchKernelGGL(perm_count_kernel, dim3(nchunks), dim3(256), N * sizeof(int), s, topk_idx, Tk, N, chunk, counts);
  BIGMAC_CHECK_LAUNCH();
  int NP = 1;
  while (NP < N) NP <<= 1;
  hipLaunchKernelGGL(perm_scan_kernel, dim3(1), dim3(1024), 0, s, counts, nchunks, N, NP, capacity, expert_offsets, maps);
  BIGMAC_CHECK_LAUNCH();
  if (chunk == P_CHUNK_SMALL)
    hipLaunchKernelGGL(perm_rank_kernel<P_CHUNK_SMALL / 64>, dim3(nchunks), dim3(64), 2 * N * sizeof(int), s, topk_idx, Tk, N, nbits, capacity,
                       counts, expert_offsets, slot_of, src_of);
  else
    hipLaunchKernelGGL(perm_rank_kernel<P_CHUNK_LARGE / 64>, dim3(nchunks), dim3(64), 2 * N * sizeof(int), s, topk_idx, Tk, N, nbits, capacity,
                       counts, expert_offsets, slot_of, src_of);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

namespace {
// read-only counterpart of combine_rows_kernel (see bigmac_gather_probe)
template <bool STREAMING>
__global__ __launch_bounds__(256) void gather_probe_kernel(const u32x4_t* __restrict__ table, const int32_t* __restrict__ order, long groups,
                                                           int row16, unsigned* sink) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int per = row16 / 2;
  if (g >= (size_t)groups * per) return;
  const size_t grp = g / per;
  const int c = (int)(g % per);
  u32x4_t v[8][2];
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const u32x4_t* p = table + (size_t)order[grp * 8 + u] * row16 + c * 2;
    if (STREAMING) { v[u][0] = __builtin_nontemporal_load(p); v[u][1] = __builtin_nontemporal_load(p + 1); }
    else { v[u][0] = p[0]; v[u][1] = p[1]; }
  }
  unsigned acc = 0;
#pragma unroll
  for (int u = 0; u < 8; ++u) acc ^= v[u][0].x ^ v[u][1].w;
  if (acc == 0x9e3779b9u && sink[0] == 0x7f4a7c15u) sink[0] = acc;   // (keeps the loads alive; rows of real data never meet both)
}
}  // namespace

int launch_gather_probe(const void* table, const int32_t* order, long rows, long row_bytes, int streaming, unsigned* sink, hipStream_t s) {
  const long groups = rows / 8;
  const int row16 = (int)(row_bytes / 16);
  const size_t n = (size_t)groups * (row16 / 2);
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (streaming) hipLaunchKernelGGL(gather_probe_kernel<true>, grid, block, 0, s, (const u32x4_t*)table, order, groups, row16, sink);
  else hipLaunchKernelGGL(gather_probe_kernel<false>, grid, block, 0, s, (const u32x4_t*)table, order, groups, row16, sink);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

int launch_dispatch_rows(int dtype, int T, int k, int width, const void* x_low, const int32_t* slot_of,
                         void* x_perm, hipStream_t s) {
  const int cpr = width * esize(dtype) / 16;
  const size_t n = (size_t)T * cpr;
  hipLaunchKernelGGL(dispatch_rows_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const uint4*)x_low, slot_of,
                     (uint4*)x_perm, T, k, cpr);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

namespace {
template <typename ROW, int OUT>
void launch_combine_ku(int ku, dim3 grid, hipStream_t s, const ROW* o_perm, const int32_t* slot_of, const float* w, const float* addend,
                       void* y, int T, int k, int width, int stream_out) {
  const dim3 block(256);
  const bool uniform = width % 512 == 0;   // 64 threads x 8 columns: whole wavefronts per token
#define BIGMAC_COMBINE(KU)                                                                                                        \
  if (uniform) hipLaunchKernelGGL((combine_rows_kernel<ROW, OUT, KU, true>), grid, block, 0, s, o_perm, slot_of, w, addend, y, T, k, width, stream_out); \
  else hipLaunchKernelGGL((combine_rows_kernel<ROW, OUT, KU, false>), grid, block, 0, s, o_perm, slot_of, w, addend, y, T, k, width, stream_out)
  switch (ku) {
    case 8: BIGMAC_COMBINE(8); break;
    case 7: BIGMAC_COMBINE(7); break;
    case 6: BIGMAC_COMBINE(6); break;
    case 5: BIGMAC_COMBINE(5); break;
    case 4: BIGMAC_COMBINE(4); break;
    case 3: BIGMAC_COMBINE(3); break;
    case 2: BIGMAC_COMBINE(2); break;
    default: BIGMAC_COMBINE(1); break;
  }
#undef BIGMAC_COMBINE
}
// picks taken at a time: all k up to 8, else the largest divisor of k that is at most 8
inline int combine_unroll(int k) {
  for (int ku = 8; ku > 1; --ku)
    if (k % ku == 0) return ku;
  return 1;
}
}  // namespace

// stream_out (split-bf16 output only): store the result with the non-temporal hint.  Measured at
// zipf_stress: the kernel itself 6-10 % faster either way; the forward combine's y', which the
// ascending product reads several times, is then missing from the caches (that product 0.54 ->
// 0.60 ms), the backward's dx' is not missed by its two readers: on for the latter only.
int launch_combine_rows(int dtype, int T, int k, int width, const void* o_perm, const int32_t* slot_of,
                        const float* topk_w, void* y_low, int out_kind, hipStream_t s, const float* addend, int stream_out) {
  if (width % 8) return BIGMAC_ERR_INVALID_ARG;
  if (out_kind != COMBINE_F32 && out_kind != COMBINE_SPLIT_BF16) return BIGMAC_ERR_INVALID_ARG;
  const size_t n = (size_t)T * (width / 8);
  const dim3 grid((unsigned)((n + 255) / 256));
  const int ku = combine_unroll(k);
  if (dtype == BIGMAC_BF16) {
    if (out_kind == COMBINE_F32) launch_combine_ku<bf16_t, COMBINE_F32>(ku, grid, s, (const bf16_t*)o_perm, slot_of, topk_w, addend, y_low, T, k, width, stream_out);
    else launch_combine_ku<bf16_t, COMBINE_SPLIT_BF16>(ku, grid, s, (const bf16_t*)o_perm, slot_of, topk_w, addend, y_low, T, k, width, stream_out);
  } else {
    if (out_kind == COMBINE_F32) launch_combine_ku<float, COMBINE_F32>(ku, grid, s, (const float*)o_perm, slot_of, topk_w, addend, y_low, T, k, width, stream_out);
    else launch_combine_ku<float, COMBINE_SPLIT_BF16>(ku, grid, s, (const float*)o_perm, slot_of, topk_w, addend, y_low, T, k, width, stream_out);
  }
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

namespace {
template <typename OT>
void launch_combine_backward_wide(int ku, dim3 grid, hipStream_t s, const float* dy_low, const OT* o_perm, const int32_t* slot_of,
                                  const float* w, float* dgate, bf16_t* do_perm, int T, int k, int width) {
  const dim3 block(256);
#define BIGMAC_COMBINE_BWD(KU) \
  hipLaunchKernelGGL((combine_backward_wide_kernel<OT, KU>), grid, block, 0, s, dy_low, o_perm, slot_of, w, dgate, do_perm, T, k, width)
  switch (ku) {
    case 8: BIGMAC_COMBINE_BWD(8); break;
    case 7: BIGMAC_COMBINE_BWD(7); break;
    case 6: BIGMAC_COMBINE_BWD(6); break;
    case 5: BIGMAC_COMBINE_BWD(5); break;
    case 4: BIGMAC_COMBINE_BWD(4); break;
    case 3: BIGMAC_COMBINE_BWD(3); break;
    case 2: BIGMAC_COMBINE_BWD(2); break;
    default: BIGMAC_COMBINE_BWD(1); break;
  }
#undef BIGMAC_COMBINE_BWD
}
}  // namespace

int launch_combine_backward(int dtype, int o_dtype, int T, int k, int width, const float* dy_low, const void* o_perm,
                            const int32_t* slot_of, const float* topk_w, float* dgate, void* do_perm, hipStream_t s) {
  const dim3 grid((T + 3) / 4), block(256);
  if (dtype == BIGMAC_BF16 && width % 8 == 0 && width >= 512) {   // narrower rows would leave lanes idle
    const int ku = combine_unroll(k);
    if (o_dtype == BIGMAC_BF16)
      launch_combine_backward_wide<bf16_t>(ku, grid, s, dy_low, (const bf16_t*)o_perm, slot_of, topk_w, dgate, (bf16_t*)do_perm, T, k, width);
    else
      launch_combine_backward_wide<float>(ku, grid, s, dy_low, (const float*)o_perm, slot_of, topk_w, dgate, (bf16_t*)do_perm, T, k, width);
  } else if (dtype == BIGMAC_BF16 && o_dtype == BIGMAC_BF16) {
    hipLaunchKernelGGL((combine_backward_kernel<bf16_t, bf16_t>), grid, block, 0, s, dy_low, (const bf16_t*)o_perm, slot_of, topk_w, dgate,
                       (bf16_t*)do_perm, T, k, width);
  } else if (dtype == BIGMAC_BF16) {
    hipLaunchKernelGGL((combine_backward_kernel<float, bf16_t>), grid, block, 0, s, dy_low, (const float*)o_perm, slot_of, topk_w, dgate,
                       (bf16_t*)do_perm, T, k, width);
  } else {
    if (o_dtype != BIGMAC_F32) return BIGMAC_ERR_INVALID_ARG;
    hipLaunchKernelGGL((combine_backward_kernel<float, float>), grid, block, 0, s, dy_low, (const float*)o_perm, slot_of, topk_w, dgate,
                       (float*)do_perm, T, k, width);
  }
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

namespace {
// Device address of `scratch` on the current device.  In host code the array's name is only a
// stand-in for the symbol, not a device address: the address is asked for once per device (each
// GPU holds its own copy at its own address) and kept.
constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
std::atomic<void*> g_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES];
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) return BIGMAC_ERR_HIP;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BIGMAC_ERR_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // two first calls racing store the same address
  }
  *out = p;
  return BIGMAC_OK;
}
}  // namespace

}  // namespace bigmac

extern "C" int bigmac_dispatch_static(const bigmac_dims* D, const void* x_low, const int32_t* topk_idx, void* x_perm,
                                      int32_t* expert_offsets, int32_t* slot_of, int32_t* src_of, void* stream) {
  using namespace bigmac;
  int rc = check_dims(D);
  if (rc) return rc;
  if (!topk_idx || !expert_offsets || !slot_of || !src_of) return BIGMAC_ERR_INVALID_ARG;
  if ((x_low == nullptr) != (x_perm == nullptr)) return BIGMAC_ERR_INVALID_ARG;
  if (permutation_ws_bytes(D->T, D->k, D->N) > BIGMAC_STATIC_SCRATCH_BYTES) return BIGMAC_ERR_TOO_LARGE;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)stream;
  // every counter the sort reads is written by its first kernel in the same call: nothing to clear
  rc = launch_build_permutation(D->T, D->k, D->N, D->capacity, topk_idx, expert_offsets, slot_of, src_of, ws, s);
  if (rc || !x_low) return rc;
  return launch_dispatch_rows(D->dtype, D->T, D->k, widths(*D).win, x_low, slot_of, x_perm, s);
}
