// The matrix products of the layer at shapes where they are bound by the matrix cores (long K,
// many tiles): 256 x 256 output tiles, one workgroup of four wavefronts per CU, each wavefront a
// 128 x 128 sub-tile whose 256 accumulator registers fill half of a lane's register file.
//
// Why this shape.  A CU has to be fed (BM + BN) * BK * 2 bytes of operands per 2 * BM * BN * BK flops;
// with 128 x 128 tiles the matrix cores at full rate would ask the L2 for 39 TB/s, with 256 x 128
// tiles for 29 TB/s, with 256 x 256 tiles for 19.6 TB/s, and per XCD the 32 resident tiles (a block
// of 32 / gx row tiles x gx column tiles of the tile order) share their operand tiles 4 to 8 ways
// in the L2.  Operand tiles are 32 deep (32 KB per k tile for A and B together) in a ring of four
// stages: three k tiles in flight per CU.  The k loop is software-pipelined at the level of the
// 16-deep MFMA steps: while the 16 MFMAs of one step run, the LDS reads of the next step's
// fragments (and the global requests of the k tile three ahead) are issued, so that neither LDS
// latency nor the once-per-k-tile barrier leaves the matrix pipe idle for long.
#include "gemm_core.hpp"

namespace bigmac {

namespace {

constexpr int BIG_BM = 256, BIG_BN = 256, BIG_BK = 32, BIG_NS = 4;

template <bool AK, bool BKC, int EPI, bool OUTF32>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void mfma_big_kernel(GemmDesc p) {
  constexpr int BM = BIG_BM, BN = BIG_BN, BK = BIG_BK, NS = BIG_NS;
  constexpr int THREADS = 256, WAVES_N = 2;
  constexpr int WM = 128, WN = 128, TM = 4, TN = 4, KS = BK / 16;
  constexpr int A_CHUNKS = BM * BK / 8, B_CHUNKS = BN * BK / 8;
  constexpr int STAGE_CHUNKS = A_CHUNKS + B_CHUNKS, STAGE_BYTES = STAGE_CHUNKS * 16;   // 32 KB
  constexpr bool SWAP = !(EPI == EPI_ACCUM || OUTF32);   // bf16 results accumulate the transposed tile (see gemm.hip)
  static_assert(KS == 2 && NS == 4, "the k loop below is written for two MFMA steps per k tile and four ring stages");
  static_assert(EPI == EPI_STORE || EPI == EPI_ACCUM || EPI == EPI_GELU, "epilogues of this kernel");
  __shared__ uint4 ring[NS * STAGE_CHUNKS];   // 128 KB
  const unsigned ring_at = lds_address(ring);
  constexpr unsigned OUT_OF_RANGE = 0x80000000u;
  constexpr int NON_TEMPORAL = 2;
  constexpr int STREAMING = (EPI == EPI_GELU) ? NON_TEMPORAL : 0;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave / WAVES_N) * WM, wn = (wave % WAVES_N) * WN;

  using MoveA = TileMover<AK ? BM : BK, AK ? BK : BM, THREADS, AK>;
  using MoveB = TileMover<BKC ? BN : BK, BKC ? BK : BN, THREADS, BKC>;
  constexpr int LOADS_PER_TILE = MoveA::NCH + MoveB::NCH;   // 8
  MoveA ma;
  MoveB mb;
  ma.init(p.lda);
  mb.init(p.ldb);
  const int wrap_tiles = p.kwrap_b ? p.kwrap_b / BK : 0x7FFFFFFF;

  TileSpace ts = tile_space<BM, BN>(p);
  if (p.mode == GEMM_RAGGED_K && p.tile_map) balance_ragged_k(p, ts);
  // buffers of one tile (id < 0: no tile, empty ranges); ranges end at the last valid row so that
  // tails read as zeros
  auto operands = [&](int id) {
    TileOperands o;
    o.t = resolve_tile<BM, BN>(p, ts, id, 2);
    const TileCoord& t = o.t;
    const int klen = t.kend - t.kbeg;
    o.nk = (klen + BK - 1) / BK;
    o.wrap_first = p.kwrap_b ? (t.kbeg / BK) % (p.kwrap_b / BK) : 0;
    const bf16_t* A = (const bf16_t*)p.A;
    if (AK) {
      const int rows = min(t.m_end - t.m0, BM);
      o.ra = __builtin_amdgcn_make_buffer_rsrc((void*)(A + (size_t)t.m0 * p.lda + t.kbeg), 0,
                                               rows > 0 && klen > 0 ? (int)(((size_t)(rows - 1) * p.lda + klen) * 2) : 0, 0x00020000);
      o.step_a = BK * 2u;
    } else {
      const int cols = t.valid ? min(p.M - t.m0, BM) : 0;
      o.ra = __builtin_amdgcn_make_buffer_rsrc((void*)(A + (size_t)t.kbeg * p.lda + t.m0), 0,
                                               klen > 0 && cols > 0 ? (int)(((size_t)(klen - 1) * p.lda + cols) * 2) : 0, 0x00020000);
      o.step_a = (unsigned)(BK * p.lda * 2);
    }
    const bf16_t* B = (const bf16_t*)t.B;
    const int kb0 = p.kwrap_b ? 0 : t.kbeg;
    const int kblen = !t.valid ? 0 : (p.kwrap_b ? p.kwrap_b : klen);
    if (BKC) {
      const int rows = min(p.N - t.n0, BN);
      o.rb = __builtin_amdgcn_make_buffer_rsrc((void*)(B + (size_t)t.n0 * p.ldb + kb0), 0,
                                               rows > 0 && kblen > 0 ? (int)(((size_t)(rows - 1) * p.ldb + kblen) * 2) : 0, 0x00020000);
      o.step_b = BK * 2u;
    } else {
      const int cols = min(p.N - t.n0, BN);
      o.rb = __builtin_amdgcn_make_buffer_rsrc((void*)(B + (size_t)kb0 * p.ldb + t.n0), 0,
                                               kblen > 0 && cols > 0 ? (int)(((size_t)(kblen - 1) * p.ldb + cols) * 2) : 0, 0x00020000);
      o.step_b = (unsigned)(BK * p.ldb * 2);
    }
    return o;
  };
  // k tile `tile` of tile `o` -> ring stage `stage` (k tiles past the end are requested out of
  // range: zeros, no memory traffic)
  auto fetch = [&](const TileOperands& o, int tile, int stage) {
    const bool live = tile < o.nk;
    const unsigned off_a = live ? (unsigned)tile * o.step_a : OUT_OF_RANGE;
    const unsigned off_b = live ? (unsigned)((tile + o.wrap_first) % wrap_tiles) * o.step_b : OUT_OF_RANGE;
    uint4* dst = ring + stage * STAGE_CHUNKS;
    ma.load(o.ra, dst, off_a);
    mb.load(o.rb, dst + A_CHUNKS, off_b);
  };

  // Per-lane fragment addresses (bytes, stage 0).  k-contiguous tiles (4 chunks per row): one
  // address per MFMA step, sub-tile i is 32 rows = 2048 bytes further.  Transposed tiles (32
  // chunks per k row): the piece permutation of the layout depends on the k row only through
  // krow % 4, which the lane fixes, so one address per sub-tile serves both steps and both 4-row
  // reads through instruction offsets (16 k rows = 8192 bytes, 4 k rows = 2048 bytes).
  constexpr int NA = AK ? KS : TM, NB = BKC ? KS : TN;
  unsigned pa[NA], pb[NB];
  if (AK) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) pa[ks] = ring_at + lds_chunk_kc<BK / 8>(wm + (lane & 31), ks * 2 + (lane >> 5)) * 16;
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int c = wm + i * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
      pa[i] = ring_at + lds_chunk_tr<BM / 8>((lane >> 5) * 8 + ((lane & 15) >> 2), c >> 3) * 16 + (c & 7) * 2;
    }
  }
  if (BKC) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) pb[ks] = ring_at + A_CHUNKS * 16 + lds_chunk_kc<BK / 8>(wn + (lane & 31), ks * 2 + (lane >> 5)) * 16;
  } else {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int c = wn + j * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
      pb[j] = ring_at + A_CHUNKS * 16 + lds_chunk_tr<BN / 8>((lane >> 5) * 8 + ((lane & 15) >> 2), c >> 3) * 16 + (c & 7) * 2;
    }
  }
  // The ring spans 128 KB and an LDS instruction's offset field 64 KB: stages 2 and 3 are reached
  // through addresses 64 KB on.
  struct FragSet {
    Frag<AK> a[TM];
    Frag<BKC> b[TN];
  };
  constexpr int READS_PER_STEP = (AK ? TM : 2 * TM) + (BKC ? TN : 2 * TN);
  // the LDS reads of sub-tile `sub` (0 .. TM - 1: A, TM .. TM + TN - 1: B) of one MFMA step
  auto read_sub = [&](auto stage_c, auto ks_c, auto sub_c, FragSet& f) {
    constexpr int s = decltype(stage_c)::value, ks = decltype(ks_c)::value, sub = decltype(sub_c)::value;
    constexpr int OFF = (s & 1) * STAGE_BYTES;
    const unsigned hi = (s >> 1) * 65536u;
    if constexpr (sub < TM) {
      constexpr int i = sub;
      if constexpr (AK) lds_read_b128<OFF + i * 2048>(pa[ks] + hi, f.a[i].q);
      else {
        lds_read_tr_b64<OFF + ks * 8192>(pa[i] + hi, f.a[i].h[0]);
        lds_read_tr_b64<OFF + ks * 8192 + 2048>(pa[i] + hi, f.a[i].h[1]);
      }
    } else {
      constexpr int j = sub - TM;
      if constexpr (BKC) lds_read_b128<OFF + j * 2048>(pb[ks] + hi, f.b[j].q);
      else {
        lds_read_tr_b64<OFF + ks * 8192>(pb[j] + hi, f.b[j].h[0]);
        lds_read_tr_b64<OFF + ks * 8192 + 2048>(pb[j] + hi, f.b[j].h[1]);
      }
    }
  };
  auto read_frags = [&](auto stage_c, auto ks_c, FragSet& f) {
    static_for<0, TM + TN>([&](auto sub) { read_sub(stage_c, ks_c, sub, f); });
  };

  auto rows_of = [&](const TileCoord& t, const void* base, int esz_out) {
    const int c_rows = min(t.m_end - t.m0, BM);
    const size_t first = (size_t)base + (size_t)t.m0 * p.ldc * esz_out;
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)first);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(first >> 32));
    const int bytes = __builtin_amdgcn_readfirstlane(c_rows > 0 ? (int)(((size_t)(c_rows - 1) * p.ldc + p.N) * esz_out) : 0);
    return __builtin_amdgcn_make_buffer_rsrc((void*)(((size_t)hi << 32) | lo), 0, bytes, 0x00020000);
  };

  const int stride = (int)(gridDim.x >> 3);
  int pos = (int)(blockIdx.x >> 3);
  int id = tile_at(ts, pos);
  if (id < 0) return;
  TileOperands cur = operands(id);
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) fetch(cur, s, s);

  while (true) {
    const TileCoord t = cur.t;
    const int nk = cur.nk;
    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    FragSet f0, f1;
    auto mfma_one = [&](FragSet& f, auto q_c) {
      constexpr int q = decltype(q_c)::value, i = q / TN, j = q % TN;
      acc[i][j] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[j].value(), f.a[i].value(), acc[i][j], 0, 0, 0)
                       : __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i].value(), f.b[j].value(), acc[i][j], 0, 0, 0);
    };
    auto settle = [&](FragSet& f) {
#pragma unroll
      for (int i = 0; i < TM; ++i) f.a[i].settle();
#pragma unroll
      for (int j = 0; j < TN; ++j) f.b[j].settle();
    };
    // Every k tile requests exactly LOADS_PER_TILE loads (out of range, i.e. zeros without memory
    // traffic, past the last k tile), so the loads in flight behind any k tile are a constant.
    // In front of this point, oldest first: this tile's k tiles 0, 1, 2 (requested before the
    // previous tile's epilogue) and that epilogue's stores, which are younger: the count below is
    // reached once k tile 0 and nearly all of those stores are done.
    BIGMAC_WAIT_VMCNT(2 * LOADS_PER_TILE);
    __builtin_amdgcn_s_barrier();                       // every wave's part of k tile 0 is there; stage 3 is free
    fetch(cur, 3, 3);
    if (nk > 0) read_frags(StaticIndex<0>{}, StaticIndex<0>{}, f0);
    for (int it0 = 0; it0 < nk; it0 += NS) {
      static_for<0, NS>([&](auto stage) {
        constexpr int s = decltype(stage)::value;
        const int it = it0 + s;
        if (it >= nk) return;
        // first MFMA step: its fragments (f0) were requested during the previous step; the second
        // step's (f1) go out now and arrive while the 16 products of the first run
        read_frags(stage, StaticIndex<1>{}, f1);
        lds_wait_for<(READS_PER_STEP < 15 ? READS_PER_STEP : 15)>();
        settle(f0);
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, TM * TN>([&](auto q) { mfma_one(f0, q); });
        __builtin_amdgcn_sched_barrier(0);              // the products are issued before the waits below
        lds_wait_for<0>();                              // this wave has read all it needs of stage s
        settle(f1);
        if (it + 1 < nk) {
          // behind k tile it + 1 the loads of k tiles it + 2 and it + 3 may stay in flight
          BIGMAC_WAIT_VMCNT(2 * LOADS_PER_TILE);
          __builtin_amdgcn_s_barrier();                 // k tile it + 1 has landed for everyone; stage s is free
          // Second MFMA step, with the requests of k tile it + NS (into the stage just freed) and
          // the LDS reads of the next k tile's first step dealt out between its 16 products: each
          // is issued in the shadow of a product the matrix pipe is still working on.
          const int tile = it + NS;
          const bool live = tile < nk;
          const unsigned off_a = live ? (unsigned)tile * cur.step_a : OUT_OF_RANGE;
          const unsigned off_b = live ? (unsigned)((tile + cur.wrap_first) % wrap_tiles) * cur.step_b : OUT_OF_RANGE;
          uint4* dst = ring + s * STAGE_CHUNKS;
          static_for<0, TM * TN>([&](auto q_c) {
            constexpr int q = decltype(q_c)::value;
            mfma_one(f1, q_c);
            if constexpr (q < MoveA::NCH) ma.template load_one<q>(cur.ra, dst, off_a);
            else if constexpr (q < LOADS_PER_TILE) mb.template load_one<q - MoveA::NCH>(cur.rb, dst + A_CHUNKS, off_b);
            else read_sub(StaticIndex<(s + 1) % NS>{}, StaticIndex<0>{}, StaticIndex<q - LOADS_PER_TILE>{}, f0);
            __builtin_amdgcn_sched_barrier(0);
          });
        } else {
          __builtin_amdgcn_sched_barrier(0);
          static_for<0, TM * TN>([&](auto q) { mfma_one(f1, q); });
        }
      });
    }

    pos += stride;
    id = tile_at(ts, pos);
    const TileOperands nxt = operands(id);
    __builtin_amdgcn_s_barrier();                       // every wave has left the k loop: the ring is free
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) fetch(nxt, s, s);

    if ((EPI == EPI_GELU || EPI == EPI_STORE) && t.bias) {   // optional bias of the product's columns
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if (SWAP) add_bias_transposed(acc[i][j], (const bf16_t*)t.bias, t.n0 + wn + j * 32, p.N, lane);
          else add_bias_plain(acc[i][j], (const bf16_t*)t.bias, t.n0 + wn + j * 32, p.N, lane);
          __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (EPI == EPI_ACCUM || OUTF32) {
      // fp32 results straight from the accumulators: lane l of a 32 x 32 sub-tile holds column
      // l % 32 and rows 8 (v / 4) + 4 (l / 32) + v % 4; a store covers 128 contiguous bytes of two rows
      const __amdgpu_buffer_rsrc_t rc = rows_of(t, t.C, 4);
      const unsigned row_step = (unsigned)(p.ldc * 4);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = t.n0 + wn + j * 32 + (lane & 31);
          unsigned off[4];
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            const int row = wm + i * 32 + vq * 8 + (lane >> 5) * 4;
            off[vq] = (unsigned)(((size_t)row * p.ldc + col) * 4) | ((unsigned)(p.N - 1 - col) >> 31) * OUT_OF_RANGE;
          }
          if (EPI == EPI_ACCUM && p.beta) {
            float old[16];
#pragma unroll
            for (int v = 0; v < 16; ++v)
              old[v] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rc, off[v >> 2] + (v & 3) * row_step, 0, 0));
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] += old[v];
          }
#pragma unroll
          for (int v = 0; v < 16; ++v)
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][v]), rc, off[v >> 2] + (v & 3) * row_step, 0, NON_TEMPORAL);
          __builtin_amdgcn_sched_barrier(0);   // one sub-tile at a time: its 16 accumulators leave the accumulator file, no more
        }
    } else {
      // bf16 results (transposed accumulation: lane l owns row l % 32 of each 32-row sub-tile and,
      // per accumulator quad, 4 consecutive columns): packed quads pass through a wave-private
      // strip of 32 rows x 128 bytes in the ring's last stage (free until the next k loop's first
      // barrier) and leave as whole 128-byte row segments, 64 columns at a time.
      constexpr int SROW = 128;
      // (the k loop's last requests into stage 3, if any, were out of range: they only write zeros,
      // but must have done so before the strips are used; they are older than the prefetch)
      BIGMAC_WAIT_VMCNT((NS - 1) * LOADS_PER_TILE);
      const unsigned strip = ring_at + 65536u + STAGE_BYTES + wave * (32 * SROW);   // stage 3
      const unsigned quad_row = strip + (lane & 31) * SROW + (lane >> 5) * 8;
      const unsigned quad_swz = (lane >> 1) & 7;
      auto quad_at = [&](int jj, int vq) { return quad_row + ((((unsigned)(jj * 4 + vq)) ^ quad_swz) << 4); };
      const unsigned row_even = strip + (lane >> 3) * SROW + (((lane & 7) ^ (lane >> 4)) << 4);
      const unsigned row_odd = strip + (lane >> 3) * SROW + (((lane & 7) ^ (lane >> 4) ^ 4) << 4);
      auto row_at = [&](int q) { return (q & 1 ? row_odd : row_even) + q * 8 * SROW; };
      const __amdgpu_buffer_rsrc_t rc = rows_of(t, t.C, 2);
      const __amdgpu_buffer_rsrc_t rx = rows_of(t, EPI == EPI_GELU && p.aux_out ? p.aux_out : t.C, 2);
      const unsigned pass_step = (unsigned)(8 * p.ldc * 2);
      auto flush_rows = [&](const __amdgpu_buffer_rsrc_t& dst, int i, unsigned out_off) {
        u32x4_t v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) lds_read_b128(row_at(q), v[q]);
        lds_wait(v);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          __builtin_amdgcn_raw_buffer_store_b128(v[q], dst, out_off + (unsigned)(i * 4 + q) * pass_step, 0, STREAMING);
      };
#pragma unroll
      for (int half = 0; half < TN / 2; ++half) {
        const int out_col = t.n0 + wn + half * 64 + (lane & 7) * 8;
        const unsigned out_off = (unsigned)(((size_t)(wm + (lane >> 3)) * p.ldc + out_col) * 2) | ((unsigned)(p.N - 1 - out_col) >> 31) * OUT_OF_RANGE;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          if (EPI == EPI_GELU && p.aux_out) {   // the pre-activation itself, for the backward pass
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
              for (int vq = 0; vq < 4; ++vq) {
                const f32x16_t& a = acc[i][half * 2 + jj];
                u32x2_t w;
                w.x = f2bf_pair(a[vq * 4 + 0], a[vq * 4 + 1]);
                w.y = f2bf_pair(a[vq * 4 + 2], a[vq * 4 + 3]);
                lds_write_b64(quad_at(jj, vq), w);
              }
            flush_rows(rx, i, out_off);
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
              const f32x16_t& a = acc[i][half * 2 + jj];
              float v[4];
#pragma unroll
              for (int vr = 0; vr < 4; ++vr) v[vr] = a[vq * 4 + vr];
              if (EPI == EPI_GELU) {
#pragma unroll
                for (int vr = 0; vr < 4; ++vr) v[vr] = gelu_bf16_f(v[vr]);
              }
              u32x2_t w;
              w.x = f2bf_pair(v[0], v[1]);
              w.y = f2bf_pair(v[2], v[3]);
              lds_write_b64(quad_at(jj, vq), w);
            }
          flush_rows(rc, i, out_off);
          __builtin_amdgcn_sched_barrier(0);   // one 32-row strip at a time
        }
      }
    }
    if (id < 0) break;
    cur = nxt;
  }
}

template <bool AK, bool BKC>
int launch_big_combo(const GemmDesc& g, hipStream_t s) {
  // one workgroup per CU (256 CUs), a multiple of the 8 XCDs; fewer when there are fewer tiles
  long gx = (g.N + BIG_BN - 1) / BIG_BN, gy, gz = 1;
  if (g.mode == GEMM_RAGGED_M) gy = g.max_rows / BIG_BM + g.groups + 1;
  else gy = (g.M + BIG_BM - 1) / BIG_BM;
  if (g.mode == GEMM_RAGGED_K) gz = g.groups;
  if (g.mode == GEMM_DENSE) gz = g.ksplit;
  long blocks = (gx * gy * gz + 7) / 8 * 8;
  if (blocks > 256) blocks = 256;
  const dim3 grid((unsigned)blocks), block(256);
#define BIGMAC_BIG(EPI, OUTF32) hipLaunchKernelGGL((mfma_big_kernel<AK, BKC, EPI, OUTF32>), grid, block, 0, s, g)
  switch (g.epilogue) {
    case EPI_STORE:
      if (g.out_f32) BIGMAC_BIG(EPI_STORE, true);
      else BIGMAC_BIG(EPI_STORE, false);
      break;
    case EPI_GELU: BIGMAC_BIG(EPI_GELU, false); break;
    case EPI_ACCUM: BIGMAC_BIG(EPI_ACCUM, true); break;
    default: return BIGMAC_ERR_UNSUPPORTED;
  }
#undef BIGMAC_BIG
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

}  // namespace

static_assert(BIG_BM == BIGMAC_TALL_BM, "ragged-M products on this tile use the tile map of the tall tile");

// Shapes this kernel takes (the caller decides whether it pays): bf16, the three operand layouts
// of the layer, store / GELU / accumulate epilogues; the same alignment rules as launch_gemm.
bool gemm_big_supported(const GemmDesc& g) {
  if (g.dtype != BIGMAC_BF16 || g.epilogue == EPI_DGELU || g.touch_bytes) return false;
  if (g.lda % 8 || g.ldb % 8 || g.N % 8 || ((g.a_kcontig || g.b_kcontig) && g.K % BIG_BK)) return false;
  if (g.mode != GEMM_RAGGED_M && !g.a_kcontig && g.M % 8) return false;
  if ((g.a_kcontig || g.b_kcontig) && g.mode == GEMM_RAGGED_K) return false;
  const int combo = g.a_kcontig * 2 + g.b_kcontig;
  return combo == 2 || combo == 3 || combo == 0;
}

int launch_gemm_big(const GemmDesc& g, hipStream_t s) {
  if (!gemm_big_supported(g)) return BIGMAC_ERR_UNSUPPORTED;
  if (g.N <= 0 || (g.mode != GEMM_RAGGED_M && g.M <= 0) || (g.mode != GEMM_RAGGED_K && g.K <= 0)) return BIGMAC_ERR_INVALID_ARG;
  if (g.mode != GEMM_DENSE && (!g.offsets || g.groups <= 0)) return BIGMAC_ERR_INVALID_ARG;
  if (g.mode == GEMM_RAGGED_M && !g.tile_map) return BIGMAC_ERR_INVALID_ARG;
  if (g.mode == GEMM_DENSE && g.ksplit < 1) return BIGMAC_ERR_INVALID_ARG;
  switch (g.a_kcontig * 2 + g.b_kcontig) {
    case 2: return launch_big_combo<true, false>(g, s);
    case 3: return launch_big_combo<true, true>(g, s);
    default: return launch_big_combo<false, false>(g, s);
  }
}

}  // namespace bigmac
