// Building blocks of the matrix-product kernels (gemm.hip): tile enumeration
// over the 8 XCDs, operand tiles moved from global memory straight into LDS, swizzled LDS layouts
// and the assembly LDS accesses of the MFMA operand fragments.  gfx950 only.
#pragma once
#include "common.hpp"
#include "tile_map.hpp"

// Block tile of the MFMA kernel (build-time tunables): BM x BN outputs per block, BK-deep LDS
// stages, WM x WN wavefronts each owning a (BM/WM) x (BN/WN) sub-tile of 32x32 MFMA tiles.
#ifndef BIGMAC_TILE_BM
#define BIGMAC_TILE_BM 128
#define BIGMAC_TILE_BN 128
#define BIGMAC_TILE_BK 32
#define BIGMAC_TILE_WM 2
#define BIGMAC_TILE_WN 2
#endif
// Phase time stamps for kernel studies; compiled out unless a harness defines the macro.
#ifndef BIGMAC_TRACE_AT
#define BIGMAC_TRACE_AT(tile, i)
#endif
#ifndef BIGMAC_TILE_STAGES
#define BIGMAC_TILE_STAGES 3     // LDS ring stages: STAGES - 1 k tiles of global loads in flight per block
#endif
// Workgroups resident per CU: what the ring's LDS (16 KB a stage) leaves room for, out of 160 KB.
#ifndef BIGMAC_BLOCKS_PER_CU
#define BIGMAC_BLOCKS_PER_CU (BIGMAC_TILE_STAGES <= 3 ? 3 : 2)
#endif
// The tall tile (GemmDesc::tall_tile): twice the rows per workgroup, each wavefront a 128 x 64
// sub-tile (128 accumulator registers), two workgroups per CU.  A third fewer operand bytes per
// flop: what products with many tiles and a long K are short of.
#define BIGMAC_TALL_BM (2 * BIGMAC_TILE_BM)
#define BIGMAC_TALL_BLOCKS_PER_CU 2

namespace bigmac {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

// The schedule tables (tile map, group offsets) are written before the kernel starts and only
// read by it.  Read through the constant address space they come in by scalar loads, one per
// workgroup; as plain global reads the compiler, which cannot rule out that the kernel's own
// stores change them, would issue vector loads and wait on the vector-memory counter for them.
typedef const int __attribute__((address_space(4))) * table_ptr_t;
__device__ __forceinline__ int table_at(const int* table, int i) { return ((table_ptr_t)(unsigned long long)table)[i]; }

struct TileCoord {
  int m0, n0;        // first row / column of the C tile (absolute)
  int m_end;         // rows of A and C at or beyond this are not touched
  int kbeg, kend;    // contraction range
  const void* B;     // group-resolved operand / output pointers
  void* C;
  const void* bias;  // group-resolved bias vector (NULL: none)
  bool valid;
};

// Tile enumeration.  The launch is one-dimensional.  MI355X hands consecutive workgroup ids to
// its 8 XCDs in turn and every XCD has its own L2, so a workgroup id is first turned into
// (xcd = id % 8, slot = id / 8) and each XCD is given a contiguous run of logical tiles, n tile
// fastest: the blocks that share an A tile, and the M tiles that share one expert's weights, then
// meet in one L2 instead of being fetched eight times.
struct TileSpace {
  int gx, gy, total, per_xcd;
  int first, last;   // this workgroup's XCD owns the logical tiles [first, last)
};
template <int BM, int BN>
__device__ __forceinline__ TileSpace tile_space(const GemmDesc& p) {
  TileSpace ts;
  ts.gx = (p.N + BN - 1) / BN;
  ts.gy = p.mode == GEMM_RAGGED_M ? table_at(p.tile_map, 0) : (p.M + BM - 1) / BM;
  const int gz = p.mode == GEMM_RAGGED_K ? p.groups : (p.mode == GEMM_DENSE ? p.ksplit : 1);
  ts.total = ts.gx * ts.gy * gz;
  ts.per_xcd = (ts.total + 7) >> 3;
  ts.first = (int)(blockIdx.x & 7) * ts.per_xcd;
  ts.last = min(ts.first + ts.per_xcd, ts.total);
  return ts;
}
// logical tile of position `pos` in this workgroup's XCD run, or -1
__device__ __forceinline__ int tile_at(const TileSpace& ts, int pos) {
  const int id = ts.first + pos;
  return id < ts.last ? id : -1;
}
// Tile order in time.  Every XCD owns a run of consecutive tiles, row tile by row tile, so tiles
// that follow each other share an operand panel (the A rows of a row tile, and every gx-th tile the
// B columns).  Those panels are re-read from the XCD's L2 only while the tiles that share them run
// close together in time.  With a fixed stride (workgroup w takes tiles w, w + n, w + 2n, ...)
// nothing keeps them together: a workgroup that got short tiles (ragged groups) runs ahead for
// good, after a few rounds the workgroups of an XCD are whole tiles apart, and each fetches its
// panels from memory again (measured on zipf_stress: 4-5 times the operand bytes came from HBM, and
// the products ran at the speed of that traffic).  So after its first tile a workgroup claims the
// XCD's next unstarted tile from a counter: tiles start in index order whatever each one costs,
// the ones that share a panel start within a fraction of a tile's duration of each other, and a
// panel's lines are touched again before they leave the L2.
// The claim runs one tile ahead of its use: the atomic is requested by one lane as a tile's epilogue
// starts, its result is put into LDS when that epilogue ends (publish), and read by everyone after
// the next tile's k loop (next).  Counter null: the fixed stride.
struct TileClaim {
  unsigned* ctr;
  int stride;
  int* box;
  int got;
  __device__ __forceinline__ TileClaim(unsigned* claim, int stride_, int* box_)
      : ctr(claim ? claim + (blockIdx.x & 7) * 16 : nullptr), stride(stride_), box(box_), got(0) {}
  __device__ __forceinline__ void request() {
    if (ctr && threadIdx.x == 0) got = (int)__hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __device__ __forceinline__ void publish() {
    if (ctr && threadIdx.x == 0) *box = stride + got;
  }
  // position of the next tile in the XCD's run; a barrier of the workgroup lies between this call and the next request()
  __device__ __forceinline__ int next(int pos) {
    if (!ctr) return pos + stride;
    __syncthreads();
    return __builtin_amdgcn_readfirstlane(*box);
  }
};

// Ragged-K problems (one output matrix per group, contraction over that group's rows): a tile of
// a group with many rows costs many k tiles, one of a small group almost none, so equal tile
// counts per XCD can leave one XCD with a multiple of the average work (skewed routing).  The
// tile map therefore carries an order of the groups and nine split points that cut that sequence
// into eight runs of equal cost (cost of a group = its k tiles + a constant for set-up and
// epilogue, see build_tile_map_block), each as position * 65536 + 16-bit fraction of the group at
// that position; every group has the same number of tiles, so a split point turns into a tile
// index for any tile shape.  Under skew the order puts the groups of one XCD next to each other
// (whole groups, dealt out largest first to the least loaded XCD) and the fractions are zero.
static_assert(TILE_MAP_K_ROWS == BIGMAC_TILE_BK, "the tile map prices groups in k tiles of the square tile");
__device__ __forceinline__ void balance_ragged_k(const GemmDesc& p, TileSpace& ts) {
  const int tiles_per_group = ts.gx * ts.gy;
  const int x = (int)(blockIdx.x & 7);
  const int a = table_at(p.tile_map, 1 + x), b = table_at(p.tile_map, 2 + x);
  ts.first = (a >> 16) * tiles_per_group + (((a & 0xFFFF) * tiles_per_group) >> 16);
  ts.last = (b >> 16) * tiles_per_group + (((b & 0xFFFF) * tiles_per_group) >> 16);
}

template <int BM, int BN>
__device__ __forceinline__ TileCoord resolve_tile(const GemmDesc& p, const TileSpace& ts, int id, int esz) {
  TileCoord t;
  t.B = p.B;
  t.C = p.C;
  t.bias = p.bias;
  if (id < 0) {   // no tile: empty ranges everywhere
    t.valid = false;
    t.m0 = t.n0 = t.m_end = t.kbeg = t.kend = 0;
    return t;
  }
  const int bx = id % ts.gx, by = (id / ts.gx) % ts.gy, bz = id / (ts.gx * ts.gy);
  t.valid = true;
  t.n0 = bx * BN;
  if (p.mode == GEMM_RAGGED_M) {
    int g = table_at(p.tile_map, TILE_MAP_HEADER + p.groups + 2 * by);
    t.m0 = table_at(p.tile_map, TILE_MAP_HEADER + p.groups + 1 + 2 * by);
    t.m_end = table_at(p.offsets, g + 1);
    t.kbeg = 0;
    t.kend = p.K;
    t.B = (const char*)p.B + (size_t)g * p.gstride_b * esz;
    if (p.bias) t.bias = (const char*)p.bias + (size_t)g * p.gstride_bias * esz;
  } else if (p.mode == GEMM_RAGGED_K) {
    // with a tile map the groups are walked in the map's order (see balance_ragged_k)
    const int grp = p.tile_map ? table_at(p.tile_map, TILE_MAP_HEADER + bz) : bz;
    t.m0 = by * BM;
    t.m_end = p.M;
    t.kbeg = table_at(p.offsets, grp);
    t.kend = table_at(p.offsets, grp + 1);
    t.C = (char*)p.C + (size_t)grp * p.gstride_c * sizeof(float);
  } else {
    t.m0 = by * BM;
    t.m_end = p.M;
    int per = (p.K + p.ksplit - 1) / p.ksplit;
    per = (per + 63) / 64 * 64;
    t.kbeg = bz * per;
    t.kend = min(p.K, t.kbeg + per);
    if (t.kend < t.kbeg) t.kend = t.kbeg;
    if (p.ksplit > 1) t.C = (char*)p.C + (size_t)bz * p.gstride_c * sizeof(float);
  }
  return t;
}

// ------------------------------------------------------------------------ MFMA kernel ------

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// 16-byte chunk index inside an LDS tile.  "kc" tiles keep k contiguous (CPR = BK/8 chunks per
// row); "tr" tiles keep the m (or n) index contiguous (CPR = BM/8 chunks per k row).  Both are
// XOR-swizzled so that what one pass of a fragment read touches (256 bytes, the span of the 64
// banks) falls on all banks once.
template <int CPR>
__device__ __forceinline__ int lds_chunk_kc(int row, int cc) {
  int L = row * CPR + cc;
  // 16 consecutive rows at one k chunk (what a quarter of a fragment read touches) lie in CPR
  // consecutive windows; the XOR with the window index gives their CPR-chunk groups CPR different
  // rotations, 16 different 16-byte bank groups in all
  int w = L >> 4;   // window of 16 chunks = the 256 bytes the 64 banks span
  return (w << 4) | ((L & 15) ^ (w & (CPR - 1)));
}
// A transposing fragment read takes 64 contiguous bytes from each of 4 consecutive k rows; the
// 64-byte pieces of a row are permuted by (a function of) the row index so that those four land
// on the four quarters of the 256 bytes the banks span, whatever the row pitch.
template <int CPR>
__device__ __forceinline__ int tr_piece_swap(int krow) {
  static_assert(CPR >= 4 && (CPR & (CPR - 1)) == 0, "a power of two of chunks per row");
  constexpr int ROWS_PER_WINDOW = CPR >= 16 ? 1 : 16 / CPR;     // rows that already differ in their position modulo 256 bytes
  constexpr int PIECES = CPR / 4;                                // 64-byte pieces per row
  return (krow / ROWS_PER_WINDOW) & 3 & (PIECES - 1);
}
template <int CPR>
__device__ __forceinline__ int lds_chunk_tr(int krow, int cc) {
  return krow * CPR + ((((cc >> 2) ^ tr_piece_swap<CPR>(krow)) << 2) | (cc & 3));
}

// Inverse of the two swizzles: which (row, 16-byte column chunk) lives at LDS chunk position q.
template <int CPR>
__device__ __forceinline__ void lds_unchunk_kc(int q, int& row, int& cc) {
  const int w = q >> 4;
  const int L = (w << 4) | ((q & 15) ^ (w & (CPR - 1)));
  row = L / CPR;
  cc = L % CPR;
}
template <int CPR>
__device__ __forceinline__ void lds_unchunk_tr(int q, int& krow, int& cc) {
  krow = q / CPR;
  const int pc = q % CPR;
  cc = ((((pc >> 2) ^ tr_piece_swap<CPR>(krow)) << 2) | (pc & 3));
}

// Moves one operand tile (ROWS x COLS elements, COLS contiguous in memory) from global memory
// straight into LDS (buffer load with LDS destination, 16 bytes per lane, no registers in
// between).  The hardware places the 64 lanes of a wavefront at consecutive 16-byte positions,
// so lane q loads whatever the swizzle wants at position q.  Loads are branch-free, and anything
// past the buffer's byte range (rows of a ragged tail, k rows past the end) arrives as zeros.
template <int ROWS, int COLS, int THREADS, bool KC>
struct TileMover {
  static constexpr int CPR = COLS / 8;
  static constexpr int NCH = ROWS * COLS / 8 / THREADS;
  static_assert(ROWS * COLS / 8 % THREADS == 0, "tile does not divide over the block");
  unsigned voff[NCH];   // byte offset of this lane's chunks at k tile 0
  int wave_chunk;       // first LDS chunk of this wavefront within a pass (wave-uniform)
  __device__ __forceinline__ void init(long ld) {
    wave_chunk = __builtin_amdgcn_readfirstlane((int)(threadIdx.x & ~63u));
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int q = i * THREADS + threadIdx.x;
      int row, cc;
      if (KC) lds_unchunk_kc<CPR>(q, row, cc);
      else lds_unchunk_tr<CPR>(q, row, cc);
      voff[i] = (unsigned)(row * ld + cc * 8) * 2u;
    }
  }
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, uint4* lds, unsigned tile_off) const {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass of hipcc cannot parse this builtin inside a template
#pragma unroll
    for (int i = 0; i < NCH; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(lds + i * THREADS + wave_chunk), 16,
                                               voff[i] + tile_off, 0, 0, 0);
#else
    (void)rsrc; (void)lds; (void)tile_off;
#endif
  }
};

// LDS accesses of the epilogue's staging strips, as assembly the compiler does not look into.
// The compiler makes every LDS access it knows of wait for all direct-to-LDS loads in flight
// unless it can pair the access with the loads of one particular LDS object; the strips are
// used while the next tile's prefetch is in flight, and such a wait would undo the overlap.
// Within a wavefront the LDS executes these in issue order, so a read issued after a write sees
// it; lds_wait() makes the data of the reads issued so far available.
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const void*)p;
}
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void lds_write_b64(unsigned addr, u32x2_t v) {
  asm volatile("ds_write_b64 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write_b128(unsigned addr, u32x4_t v) {
  asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_read_b64(unsigned addr, u32x2_t& v) {
  asm volatile("ds_read_b64 %0, %1" : "=v"(v) : "v"(addr) : "memory");
}
__device__ __forceinline__ void lds_read_b128(unsigned addr, u32x4_t& v) {
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
}
template <typename T, int N>
__device__ __forceinline__ void lds_wait(T (&v)[N]) {   // the values become usable behind this point
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int i = 0; i < N; ++i) asm volatile("" : "+v"(v[i]));
}
// The same with a 16-bit instruction offset, for the operand fragments in the ring.
template <int OFFSET>
__device__ __forceinline__ void lds_read_b128(unsigned addr, u32x4_t& v) {
  static_assert(OFFSET >= 0 && OFFSET < 65536, "instruction offset");
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET) : "memory");
}
// Transposing read: in each group of 16 lanes, lane i gives the address of 4 consecutive 16-bit
// elements of row (i/4) and receives column i of the resulting 4 x 16 block.
template <int OFFSET>
__device__ __forceinline__ void lds_read_tr_b64(unsigned addr, u32x2_t& v) {
  static_assert(OFFSET >= 0 && OFFSET < 65536, "instruction offset");
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET) : "memory");
}
template <int STILL_UNDER_WAY>
__device__ __forceinline__ void lds_wait_for() {   // all but the last STILL_UNDER_WAY LDS reads have delivered
  static_assert(STILL_UNDER_WAY >= 0 && STILL_UNDER_WAY < 16, "counter range");
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(STILL_UNDER_WAY) : "memory");
}
// One 32x8 operand fragment of the 32x32x16 MFMA (lane l: k = 8*(l/32) .. +8 of row l%32), read
// either as one 16-byte piece of a k-contiguous tile or as two transposing reads of 4 k rows.
template <bool KCONTIG>
struct Frag;
template <>
struct Frag<true> {
  u32x4_t q;
  __device__ __forceinline__ void settle() { asm volatile("" : "+v"(q)); }   // orders the uses behind the wait in front of this call
  __device__ __forceinline__ bf16x8_t value() const { return __builtin_bit_cast(bf16x8_t, q); }
};
template <>
struct Frag<false> {
  u32x2_t h[2];
  __device__ __forceinline__ void settle() {
    asm volatile("" : "+v"(h[0]));
    asm volatile("" : "+v"(h[1]));
  }
  __device__ __forceinline__ bf16x8_t value() const { return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(h[0], h[1], 0, 1, 2, 3)); }
};
template <int I>
struct StaticIndex { static constexpr int value = I; };
template <int BEGIN, int END, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (BEGIN < END) {
    f(StaticIndex<BEGIN>{});
    static_for<BEGIN + 1, END>(f);
  }
}

// s_waitcnt that only waits for the vector-memory counter to drop to n (gfx9 encoding)
#define BIGMAC_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

// Bias of the columns an accumulator sub-tile holds, added in place (bf16 bias vector of one group).
// Plain layout: lane l holds column col0 + l % 32 in all 16 values.  Transposed layout (bf16
// results): per quad vq the 4 consecutive columns col0 + 8 vq + 4 (l / 32) .. + 3.  Columns at or
// past n read the vector's first elements instead (their results are never stored).
__device__ __forceinline__ void add_bias_plain(f32x16_t& acc, const bf16_t* bias, int col0, int n, int lane) {
  const int col = col0 + (lane & 31);
  const float b = bf2f(bias[col < n ? col : 0]);
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] += b;
}
__device__ __forceinline__ void add_bias_transposed(f32x16_t& acc, const bf16_t* bias, int col0, int n, int lane) {
#pragma unroll
  for (int vq = 0; vq < 4; ++vq) {
    const int col = col0 + vq * 8 + (lane >> 5) * 4;
    const uint2 w = *(const uint2*)(bias + (col < n ? col : 0));
    acc[vq * 4 + 0] += __uint_as_float(w.x << 16);
    acc[vq * 4 + 1] += __uint_as_float(w.x & 0xFFFF0000u);
    acc[vq * 4 + 2] += __uint_as_float(w.y << 16);
    acc[vq * 4 + 3] += __uint_as_float(w.y & 0xFFFF0000u);
  }
}

// One tile's operands as the movers need them.
struct TileOperands {
  TileCoord t;
  __amdgpu_buffer_rsrc_t ra, rb;
  unsigned step_a, step_b;   // byte advance per k tile
  int nk;                    // k tiles
  int wrap_first;            // with a wrapped B: k tile index (within the wrap period) of this tile's first k tile
};

}  // namespace bigmac
