// Matrix products of the BigMac layer on gfx950: the shared projections of Eq. 2, the expert
// matrices of Eq. 4 / Eq. 3 over ragged per-expert row ranges, and their backward products.
//
// bf16 storage: MFMA 32x32x16 bf16 tiles with fp32 accumulation.  Operand tiles are staged in LDS
// in the same orientation they have in memory (so global reads are row-contiguous for every
// transposition) with XOR swizzles against bank conflicts; operands whose contraction index is
// not the fast one in memory are fetched with the gfx950 LDS transpose read (ds_read_b64_tr_b16).
// Workgroup tiles: 128 x 128; 256 x 128 for products with many tiles and a long K, and the same on
// its side (128 x 256) where only A is k-contiguous; 256 x 256 (eight wavefronts, one workgroup per
// CU, 64-deep k tiles) for the per-expert row products with a long K; 128 x 64 and 128 x 128 with
// 64-deep k tiles for products with few tiles.
// fp32 storage: a plain tiled FMA kernel (only the tiny fp32 workload uses it).
#include "gemm_core.hpp"

namespace bigmac {

// Persistent kernel: a workgroup walks the tiles of its XCD run (stride = workgroups per XCD).
// Per tile: a ring of NS LDS stages, NS - 1 k tiles in flight while one is consumed, one barrier
// per k tile.  When a tile's k loop ends, the first NS - 1 k tiles of the workgroup's next tile
// are requested before the epilogue starts, so the epilogue's arithmetic and stores overlap that
// latency.  Every vector memory instruction is issued unconditionally (accesses that must not
// happen are pushed out of their buffer's range instead of being branched around): the number of
// instructions in flight behind any load is then a compile-time constant, which is what the
// counter waits below and the compiler's own ones are derived from.
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool AK, bool BKC, int EPI, bool OUTF32, int NS = BIGMAC_TILE_STAGES, bool GATHER = false,
          bool SCATTER = false>
__global__ __launch_bounds__(64 * WAVES_M* WAVES_N)
    __attribute__((amdgpu_waves_per_eu(BM * BN > BIGMAC_TILE_BM * BIGMAC_TILE_BN || BK > BIGMAC_TILE_BK ? BIGMAC_TALL_BLOCKS_PER_CU : BIGMAC_BLOCKS_PER_CU)))   // (eight wavefronts, one block per CU: also 2)
void mfma_gemm_kernel(GemmDesc p) {
  constexpr int THREADS = 64 * WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int KS = BK / 16;
  constexpr int A_CHUNKS = BM * BK / 8, B_CHUNKS = BN * BK / 8;
  // NS: stages of the LDS ring, NS - 1 k tiles in flight while one is consumed
  // bf16 results accumulate the transposed tile (operands swapped in the MFMA): a lane then owns
  // one output row and groups of 4 consecutive columns, which pack into 8-byte pieces
  constexpr bool SWAP = !(EPI == EPI_ACCUM || OUTF32);
  static_assert(NS >= 2 && NS <= 4, "ring of 2 to 4 stages");
  // The ring.  All reads of it are assembly (see lds_read_*), so the only waits on its loads are
  // the counter waits written out below.
  constexpr int STAGE_CHUNKS = A_CHUNKS + B_CHUNKS;
  constexpr int STAGE_BYTES = STAGE_CHUNKS * 16;
  // Fragment reads address a stage through the 16-bit instruction offset where the whole ring is
  // within its reach; in a larger ring the stage's start is added to the address register instead.
  constexpr bool NEAR_RING = (NS - 1) * STAGE_BYTES + 8192 <= 65536;
  static_assert(NEAR_RING || (TM > TN ? TM : TN) * 32 * (BK / 8) * 16 <= 65536, "a wave tile's sub-tiles must be within reach of the instruction offset");
  __shared__ uint4 ring[NS * STAGE_CHUNKS];
  const unsigned ring_at = lds_address(ring);
  constexpr unsigned OUT_OF_RANGE = 0x80000000u;
  // Cache policy of the layer's big one-pass streams: non-temporal.  These are the results of
  // the two activation epilogues and the saved pre-activation read back by the second (the
  // [rows, hidden] tensors), and all fp32 results (weight gradients, y, dx).  Left at the default
  // they fill the XCD's L2 (4 MB, about what its workgroups write per round of tiles) and push out
  // the operand tiles that neighbouring workgroups share.  Narrow bf16 results, which the next
  // kernel reads back, keep the default; so do all operand loads (measured: slower otherwise).
  constexpr int NON_TEMPORAL = 2;
  constexpr int STREAMING = (EPI == EPI_GELU || EPI == EPI_DGELU) ? NON_TEMPORAL : 0;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave / WAVES_N) * WM, wn = (wave % WAVES_N) * WN;

  using MoveA = TileMover<AK ? BM : BK, AK ? BK : BM, THREADS, AK>;
  using MoveB = TileMover<BKC ? BN : BK, BKC ? BK : BN, THREADS, BKC>;
  constexpr int LOADS_PER_TILE = MoveA::NCH + MoveB::NCH;
  MoveA ma;
  MoveB mb;
  ma.init(p.lda);
  mb.init(p.ldb);
  // GATHER (ragged-M, k-contiguous A): row m of the product is row gather[m] / gather_div of A
  // (the index holds flat (token, pick) pairs, gather_div picks per token), so the rows an
  // expert works on are read where they lie instead of from a permuted copy (the dispatch step
  // folded into this product's operand loads).  A lane's chunks keep their place in the tile;
  // what changes from tile to tile is the memory row behind each of them: its index is read one
  // tile ahead (gather_request) and turned into the mover's offsets once the k loop of the tile
  // before is over (gather_apply).  Tile rows past the group's end read row gather[..] = 0 of A
  // (an index beyond the table's range arrives as zero): finite values that only reach output rows
  // the epilogue does not store.
  static_assert(!GATHER || AK, "gathered rows are k-contiguous rows of A");
  // SCATTER (dense product, plain bf16 store): row m of the result goes to the rows
  // scatter[m * scatter_k + j] of C instead of row m: the shared descending projection writes
  // each token's narrow row straight into the places of its (token, pick) pairs in the permuted
  // copy, and the dispatch step (a read of x' and the same writes) is gone.
  static_assert(!SCATTER || (EPI == EPI_STORE && !OUTF32), "scattered rows leave through the bf16 store epilogue");
  int gather_row[GATHER ? MoveA::NCH : 1];
  unsigned gather_col[GATHER ? MoveA::NCH : 1], gather_idx[GATHER ? MoveA::NCH : 1];
  if (GATHER) {
#pragma unroll
    for (int i = 0; i < MoveA::NCH; ++i) {
      int row, cc;
      lds_unchunk_kc<MoveA::CPR>(i * THREADS + (int)threadIdx.x, row, cc);
      gather_row[i] = row;
      gather_col[i] = (unsigned)cc * 16u;
    }
  }
  auto gather_request = [&](const TileCoord& t) {
    if (GATHER) {
      const __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc((void*)p.gather, 0, t.valid ? t.m_end * 4 : 0, 0x00020000);
#pragma unroll
      for (int i = 0; i < MoveA::NCH; ++i) gather_idx[i] = __builtin_amdgcn_raw_buffer_load_b32(rg, (unsigned)(t.m0 + gather_row[i]) * 4u, 0, 0);
    }
  };
  auto gather_apply = [&]() {
    if (GATHER) {
#pragma unroll
      for (int i = 0; i < MoveA::NCH; ++i) ma.voff[i] = (gather_idx[i] / (unsigned)p.gather_div) * (unsigned)(p.lda * 2) + gather_col[i];
    }
  };
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
    if (GATHER) {   // all of A: the rows come through the index
      o.ra = __builtin_amdgcn_make_buffer_rsrc((void*)A, 0, t.valid && klen > 0 ? (int)(((size_t)(p.gather_rows - 1) * p.lda + klen) * 2) : 0, 0x00020000);
      o.step_a = BK * 2u;
    } else if (AK) {
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
    const int kb0 = p.kwrap_b ? 0 : t.kbeg;                  // with a wrap the whole B is one k period
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
  // k tile `tile` of tile `o` -> one ring stage.  (The prefetch requests k tiles past the end of a
  // very short K too, out of range: zeros, no memory traffic.)
  auto fetch = [&](const TileOperands& o, int tile, uint4* dst) {
    const bool live = tile < o.nk;
    const unsigned off_a = live ? (unsigned)tile * o.step_a : OUT_OF_RANGE;
    const unsigned off_b = live ? (unsigned)((tile + o.wrap_first) % wrap_tiles) * o.step_b : OUT_OF_RANGE;
    ma.load(o.ra, dst, off_a);
    mb.load(o.rb, dst + A_CHUNKS, off_b);
  };
  auto prefetch = [&](const TileOperands& o) {   // the first NS - 1 k tiles into stages 0 .. NS - 2
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) fetch(o, s, ring + s * STAGE_CHUNKS);
  };

  // Per-lane fragment positions for every k step of a tile.  k-contiguous tiles: chunk index of
  // sub-tile 0 (sub-tile i is 32 rows = a whole number of swizzle periods further).  Transposed
  // tiles: byte addresses of the two 4-row reads of every sub-tile (the piece permutation moves
  // sub-tiles by lane-dependent amounts).
  unsigned pa[KS][2][AK ? 1 : TM], pb[KS][2][BKC ? 1 : TN];   // LDS byte addresses within stage 0
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    if (AK) {
      pa[ks][0][0] = ring_at + lds_chunk_kc<BK / 8>(wm + (lane & 31), ks * 2 + (lane >> 5)) * 16;
    } else {
#pragma unroll
      for (int i = 0; i < (AK ? 1 : TM); ++i) {
        const int c = wm + i * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
          pa[ks][jj][i] = ring_at + lds_chunk_tr<BM / 8>(ks * 16 + (lane >> 5) * 8 + jj * 4 + ((lane & 15) >> 2), c >> 3) * 16 + (c & 7) * 2;
      }
    }
    if (BKC) {
      pb[ks][0][0] = ring_at + A_CHUNKS * 16 + lds_chunk_kc<BK / 8>(wn + (lane & 31), ks * 2 + (lane >> 5)) * 16;
    } else {
#pragma unroll
      for (int j = 0; j < (BKC ? 1 : TN); ++j) {
        const int c = wn + j * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
          pb[ks][jj][j] = ring_at + A_CHUNKS * 16 + lds_chunk_tr<BN / 8>(ks * 16 + (lane >> 5) * 8 + jj * 4 + ((lane & 15) >> 2), c >> 3) * 16 + (c & 7) * 2;
      }
    }
  }

  // Output rows as buffers: the range ends with the last valid row, so rows of the next group
  // (or past M) fall outside it and their stores are dropped and their loads read as zero
  // without a branch; columns at or beyond N get an offset that is out of range by itself.
  // (Tile coordinates are the same in every lane; saying so keeps the descriptor in scalar
  // registers where the compiler has lost track of it: a descriptor in vector registers costs
  // a loop over its distinct values around every access.)
  auto rows_of = [&](const TileCoord& t, const void* base, int esz_out) {
    const int c_rows = min(t.m_end - t.m0, BM);
    const size_t first = (size_t)base + (size_t)t.m0 * p.ldc * esz_out;
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)first);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(first >> 32));
    const int bytes = __builtin_amdgcn_readfirstlane(c_rows > 0 ? (int)(((size_t)(c_rows - 1) * p.ldc + p.N) * esz_out) : 0);
    return __builtin_amdgcn_make_buffer_rsrc((void*)(((size_t)hi << 32) | lo), 0, bytes, 0x00020000);
  };
  // EPI_DGELU multiplies by act'(saved pre-activation): that tile is requested one tile ahead
  // (row layout: 8 lanes per 64-column row, 8 rows per pass) and used in the epilogue
  // On the tall tile (TM = 4) the saved tile passes through in two halves of TMH sub-tiles: its
  // registers and those of its quad form would not fit beside 128 accumulators otherwise.
  constexpr int HALVES = (EPI == EPI_DGELU && TM > 2) ? 2 : 1;
  constexpr int TMH = TM / HALVES;
  uint4 aux[EPI == EPI_DGELU ? TMH * 4 : 1];
  auto request_aux = [&](const TileCoord& t, int half) {
    if (EPI == EPI_DGELU) {
      const __amdgpu_buffer_rsrc_t ra = rows_of(t, p.aux_in, 2);
      const int col = t.n0 + wn + (lane & 7) * 8;
      // columns past N get the out-of-range bit by arithmetic: written as a selection, the
      // compiler turns it into two guarded loads per access, and waits between them
      const unsigned past_n = ((unsigned)(p.N - 1 - col) >> 31) * OUT_OF_RANGE;
      // One offset register, the passes 8 rows apart added per load: the empty statement keeps
      // the compiler from carrying all the per-pass offsets across tiles in registers of their own.
      unsigned first = (unsigned)(((size_t)(wm + half * TMH * 32 + (lane >> 3)) * p.ldc + col) * 2) | past_n;
      asm volatile("" : "+v"(first));
      const unsigned pass_step = (unsigned)(8 * p.ldc * 2);
#pragma unroll
      for (int c = 0; c < TMH * 4; ++c)
        aux[c] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(ra, first + (unsigned)c * pass_step, 0, NON_TEMPORAL));
    }
  };
  // While k tile `it` is awaited, the NS - 2 k tiles requested after it may stay in flight.  (At
  // the start of a tile the previous epilogue's stores are in flight as well; they are younger
  // than the whole prefetch, so this count then also waits for the rest of the prefetch, which
  // had the length of an epilogue to arrive.)
  constexpr int RING_AHEAD = (NS - 2) * LOADS_PER_TILE;

  // Warm-up of a region the k loops will read for the first time (the expert weights): one
  // 4-byte read per 128-byte line, the lines dealt out evenly over the launch.  A k loop that
  // meets a new expert's weights in memory waits a full miss latency at every k step; after
  // this they come from the memory-side cache.  (Giving every XCD the part its own tiles use,
  // for its L2, measured no better than this even split, which does not depend on the group sizes.)
  if (p.touch_bytes) {
    const size_t lines = p.touch_bytes >> 7, step = (size_t)gridDim.x * THREADS;
    const unsigned* src = (const unsigned*)p.touch;
    unsigned seen = 0;
    for (size_t l = (size_t)blockIdx.x * THREADS + threadIdx.x; l < lines; l += 4 * step) {
      unsigned v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = l + u * step < lines ? src[(l + u * step) * 32] : 0u;
      seen |= v[0] | v[1] | v[2] | v[3];
    }
    asm volatile("" ::"v"(seen));   // the reads have to happen; their values are of no interest
  }

  const int stride = (int)(gridDim.x >> 3);
  int pos = (int)(blockIdx.x >> 3);
  int id = tile_at(ts, pos);
  if (id < 0) return;
  TileOperands cur = operands(id);
  gather_request(cur.t);
  gather_apply();
  prefetch(cur);
  request_aux(cur.t, 0);
  // Tile order (see TileClaim): the first tile is this workgroup's slot, every later one is claimed.
  __shared__ int claim_box;
  TileClaim claim(p.claim, stride, &claim_box);
  claim.request();
  claim.publish();
  // the tile after this one is resolved (its table entries read) a whole k loop ahead of its use
  pos = claim.next(pos);
  int nid = tile_at(ts, pos);
  TileOperands nxt = operands(nid);
  gather_request(nxt.t);

  while (true) {
    const TileCoord t = cur.t;
    const int nk = cur.nk;
    const int cur_id = id;
    (void)cur_id;
    BIGMAC_TRACE_AT(cur_id, 0);

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // optional: waves in a k loop issue ahead of the CU's waves that are in an epilogue, so that the
    // next operand request and the matrix instructions do not queue behind epilogue arithmetic
    if (p.kloop_priority) __builtin_amdgcn_s_setprio(3);
    for (int it0 = 0; it0 < nk; it0 += NS) {
      static_for<0, NS>([&](auto stage) {
        constexpr int s = decltype(stage)::value;
        const int it = it0 + s;
        if (it >= nk) return;
        // This wave's part of k tile `it` has landed once only the k tiles requested after it are
        // in flight: NS - 2 of them, fewer over the last steps (nothing is requested past the end).
        const int younger = min(NS - 2, max(nk, NS - 1) - 1 - it);
        if (younger == NS - 2) BIGMAC_WAIT_VMCNT(RING_AHEAD);
        else if (NS > 3 && younger > 0) BIGMAC_WAIT_VMCNT(LOADS_PER_TILE);
        else BIGMAC_WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();                    // ... and so has everyone's; stage (s - 1) is free
        if (it == 0) BIGMAC_TRACE_AT(cur_id, 1);
        if (it + NS - 1 < nk) fetch(cur, it + NS - 1, ring + ((s + NS - 1) % NS) * STAGE_CHUNKS);
        // The fragments of two k steps are requested at once; the products of the first start as
        // soon as its fragments are there, while those of the second are still arriving.  (A
        // 64-deep k tile takes two such rounds: its fragments would not fit the registers at once.)
        constexpr int KG = KS < 2 ? KS : 2;
        constexpr int S_IMM = NEAR_RING ? s * STAGE_BYTES : 0;
        constexpr unsigned S_REG = NEAR_RING ? 0u : (unsigned)(s * STAGE_BYTES);
        constexpr int READS_PER_STEP = (AK ? TM : 2 * TM) + (BKC ? TN : 2 * TN);
        static_for<0, KS / KG>([&](auto round) {
          constexpr int k0 = decltype(round)::value * KG;
          Frag<AK> fa[KG][TM];
          Frag<BKC> fb[KG][TN];
          static_for<0, KG>([&](auto kstep) {
            constexpr int kk = decltype(kstep)::value, ks = k0 + kk;
            static_for<0, TM>([&](auto sub) {
              constexpr int i = decltype(sub)::value;
              if constexpr (AK) lds_read_b128<S_IMM + i * 32 * (BK / 8) * 16>(pa[ks][0][0] + S_REG, fa[kk][i].q);
              else {
                lds_read_tr_b64<S_IMM>(pa[ks][0][i] + S_REG, fa[kk][i].h[0]);
                lds_read_tr_b64<S_IMM>(pa[ks][1][i] + S_REG, fa[kk][i].h[1]);
              }
            });
            static_for<0, TN>([&](auto sub) {
              constexpr int j = decltype(sub)::value;
              if constexpr (BKC) lds_read_b128<S_IMM + j * 32 * (BK / 8) * 16>(pb[ks][0][0] + S_REG, fb[kk][j].q);
              else {
                lds_read_tr_b64<S_IMM>(pb[ks][0][j] + S_REG, fb[kk][j].h[0]);
                lds_read_tr_b64<S_IMM>(pb[ks][1][j] + S_REG, fb[kk][j].h[1]);
              }
            });
          });
          static_for<0, KG>([&](auto kstep) {
            constexpr int kk = decltype(kstep)::value;
            // the reads of the later k step may still be under way (the counter saturates at 15:
            // asking for fewer in flight than allowed only waits a little longer)
            constexpr int LATER_READS = (KG - 1 - kk) * READS_PER_STEP;
            lds_wait_for<(LATER_READS < 15 ? LATER_READS : 15)>();
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[kk][i].settle();
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[kk][j].settle();
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
              for (int j = 0; j < TN; ++j)
                acc[i][j] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk][j].value(), fa[kk][i].value(), acc[i][j], 0, 0, 0)
                                 : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk][i].value(), fb[kk][j].value(), acc[i][j], 0, 0, 0);
          });
        });
      });
    }
    BIGMAC_TRACE_AT(cur_id, 2);
    if (p.kloop_priority) __builtin_amdgcn_s_setprio(0);

    // Once every wave has left the k loop the ring is free, and nothing is in flight into its
    // last stage (the last k step waited for everything that was requested into it).
    __builtin_amdgcn_s_barrier();
    claim.request();                                     // (everyone has read the box)
    gather_apply();                                      // the mover's rows are now those of the next tile
    // bf16 epilogue staging, in the ring's last stage: the prefetch below fills stages
    // 0 .. NS - 2, and the last stage is requested again only behind the first barrier of the next
    // k loop.  A staged row is 128 bytes = 8 chunks of 16; chunk c of row r sits at position
    // c ^ ((r / 2) % 8).  The 64 banks span two rows, so the 16 rows of one parity share 8 chunk
    // positions: a column-wise quad access (32 lanes, one row each, 8 bytes) meets every position
    // twice, the least this form allows while a chunk keeps its two quads in order; a row-wise
    // access takes whole rows.  One strip (32 rows x 64 columns) per wave.
    constexpr int SROW = 128;
    static_assert(!SWAP || WN == 64, "the strip holds 64-column wave tiles");
    static_assert(WAVES_M * WAVES_N * 32 * SROW <= (A_CHUNKS + B_CHUNKS) * 16, "staging strips do not fit a ring stage");
    const unsigned strip = ring_at + (NS - 1) * STAGE_BYTES + wave * (32 * SROW);
    const unsigned quad_row = strip + (lane & 31) * SROW + (lane >> 5) * 8;
    const unsigned quad_swz = (lane >> 1) & 7;                              // (row / 2) % 8 of the quads' row
    auto quad_at = [&](int j, int vq) { return quad_row + ((((unsigned)(j * 4 + vq)) ^ quad_swz) << 4); };
    // row-wise: pass q takes row lane / 8 + 8 q, whose swizzle is lane / 16 + 4 (q % 2)
    const unsigned row_even = strip + (lane >> 3) * SROW + (((lane & 7) ^ (lane >> 4)) << 4);
    const unsigned row_odd = strip + (lane >> 3) * SROW + (((lane & 7) ^ (lane >> 4) ^ 4) << 4);
    auto row_at = [&](int q) { return (q & 1 ? row_odd : row_even) + q * 8 * SROW; };
    // EPI_DGELU: turn the saved pre-activation from its row layout into the accumulators' quad
    // layout now; its registers are then free for the next tile's request, which goes out ahead
    // of the prefetch and is therefore complete whenever a k tile of that prefetch is.
    // (Tall tile: the first half now, with the second half requested in its place; the second half
    // is turned, and the next tile's first half requested, between the two halves of the epilogue.)
    u32x2_t pre[EPI == EPI_DGELU ? TMH * TN * 4 : 1];
    auto turn_aux = [&]() {
#pragma unroll
      for (int i = 0; i < TMH; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) lds_write_b128(row_at(q), __builtin_bit_cast(u32x4_t, aux[i * 4 + q]));
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) lds_read_b64(quad_at(j, vq), pre[(i * TN + j) * 4 + vq]);
      }
      lds_wait(pre);
    };
    if (EPI == EPI_DGELU) {
      turn_aux();
      if (HALVES == 2) request_aux(t, 1);
      else request_aux(nxt.t, 0);
    }
    prefetch(nxt);

    // optional bias of the product's columns (expert biases), before the epilogue's own work
    if ((EPI == EPI_GELU || EPI == EPI_STORE) && t.bias) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if (SWAP) add_bias_transposed(acc[i][j], (const bf16_t*)t.bias, t.n0 + wn + j * 32, p.N, lane);
          else add_bias_plain(acc[i][j], (const bf16_t*)t.bias, t.n0 + wn + j * 32, p.N, lane);
        }
    }
    // epilogue: lane l of a 32x32 tile holds column l%32, rows 8*(v/4) + 4*(l/32) + v%4
    if (EPI == EPI_ACCUM || OUTF32) {
      // fp32 results: a lane group already writes 128 contiguous bytes per row.  Accumulation into
      // C requests 32 rows of the old tile before the first add: one memory round trip, not one
      // per element.
      const __amdgpu_buffer_rsrc_t rc = rows_of(t, t.C, 4);
      const unsigned row_step = (unsigned)(p.ldc * 4);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = t.n0 + wn + j * 32 + (lane & 31);
          unsigned off[4];   // offset of each quad's first row; the 4 rows of a quad are ldc apart
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
        }
    } else {
      // bf16 results.  With the transposed accumulation lane l owns row l%32 of each 32-row sub-tile
      // and, per accumulator quad, 4 consecutive columns: the epilogue math runs on the accumulators,
      // quads are packed to 8 bytes and pass through the wave's LDS strip to come out as whole
      // rows: 16-byte stores, 128 contiguous bytes per row.
      const int out_col = t.n0 + wn + (lane & 7) * 8;
      const __amdgpu_buffer_rsrc_t rc = rows_of(t, t.C, 2);
      const __amdgpu_buffer_rsrc_t rx = rows_of(t, EPI == EPI_GELU && p.aux_out ? p.aux_out : t.C, 2);
      const unsigned out_off = (unsigned)(((size_t)(wm + (lane >> 3)) * p.ldc + out_col) * 2) | ((unsigned)(p.N - 1 - out_col) >> 31) * OUT_OF_RANGE;
      const unsigned pass_step = (unsigned)(8 * p.ldc * 2);
      auto flush_rows = [&](const __amdgpu_buffer_rsrc_t& dst, int i) {
        u32x4_t v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) lds_read_b128(row_at(q), v[q]);
        lds_wait(v);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          __builtin_amdgcn_raw_buffer_store_b128(v[q], dst, out_off + (unsigned)(i * 4 + q) * pass_step, 0, STREAMING);
      };
      // SCATTER: the staged rows of a sub-tile leave once per pick.  The slots of the lane's four rows
      // are read eight picks at a time (the loads are younger than the next tile's prefetch: by the
      // time they answer, that has landed); a row past M, a pick past scatter_k and a negative slot
      // (a dropped pair) turn the store's offset out of range by arithmetic, not by a branch.
      auto flush_scattered = [&](int i) {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)p.scatter, 0, p.M * p.scatter_k * 4, 0x00020000);
        const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(p.C, 0, (int)((size_t)p.scatter_rows * p.ldc * 2), 0x00020000);
        const unsigned col_off = (unsigned)out_col * 2u | ((unsigned)(p.N - 1 - out_col) >> 31) * OUT_OF_RANGE;
        const unsigned row_bytes = (unsigned)(p.ldc * 2);
        u32x4_t v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) lds_read_b128(row_at(q), v[q]);
        lds_wait(v);
        for (int j0 = 0; j0 < p.scatter_k; j0 += 8) {
          int slot[4][8];
          unsigned dead[4][8];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int row = t.m0 + wm + i * 32 + q * 8 + (lane >> 3);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              dead[q][j] = ((unsigned)(t.m_end - 1 - row) >> 31) | ((unsigned)(p.scatter_k - 1 - (j0 + j)) >> 31);
              slot[q][j] = (int)__builtin_amdgcn_raw_buffer_load_b32(rs, (unsigned)((row * p.scatter_k + j0 + j) * 4) | dead[q][j] * OUT_OF_RANGE, 0, 0);
            }
          }
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              const unsigned gone = dead[q][j] | ((unsigned)slot[q][j] >> 31);
              __builtin_amdgcn_raw_buffer_store_b128(v[q], rd, ((unsigned)slot[q][j] * row_bytes + col_off) | gone * OUT_OF_RANGE, 0, 0);
            }
        }
      };
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        if (EPI == EPI_DGELU && HALVES == 2 && i == TMH) {
          turn_aux();
          request_aux(nxt.t, 0);
        }
        if (EPI == EPI_GELU && p.aux_out) {   // the pre-activation itself, for the backward pass
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
              u32x2_t w;
              w.x = f2bf_pair(acc[i][j][vq * 4 + 0], acc[i][j][vq * 4 + 1]);
              w.y = f2bf_pair(acc[i][j][vq * 4 + 2], acc[i][j][vq * 4 + 3]);
              lds_write_b64(quad_at(j, vq), w);
            }
          flush_rows(rx, i);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            float v[4];
#pragma unroll
            for (int vr = 0; vr < 4; ++vr) v[vr] = acc[i][j][vq * 4 + vr];
            if (EPI == EPI_GELU) {
#pragma unroll
              for (int vr = 0; vr < 4; ++vr) v[vr] = gelu_bf16_f(v[vr]);
            } else if (EPI == EPI_DGELU) {
              const u32x2_t sv = pre[((i % TMH) * TN + j) * 4 + vq];
              v[0] *= gelu_grad_bf16_f(__uint_as_float(sv.x << 16));
              v[1] *= gelu_grad_bf16_f(__uint_as_float(sv.x & 0xFFFF0000u));
              v[2] *= gelu_grad_bf16_f(__uint_as_float(sv.y << 16));
              v[3] *= gelu_grad_bf16_f(__uint_as_float(sv.y & 0xFFFF0000u));
            }
            u32x2_t w;
            w.x = f2bf_pair(v[0], v[1]);
            w.y = f2bf_pair(v[2], v[3]);
            lds_write_b64(quad_at(j, vq), w);
          }
        if (SCATTER) flush_scattered(i);
        else flush_rows(rc, i);
      }
    }
    BIGMAC_TRACE_AT(cur_id, 3);
    BIGMAC_TRACE_AT(cur_id, 4);
    if (nid < 0) break;
    claim.publish();
    cur = nxt;
    id = nid;
    pos = claim.next(pos);
    nid = tile_at(ts, pos);
    nxt = operands(nid);
    gather_request(nxt.t);
  }
}

// ------------------------------------------------------------------------ fp32 kernel ------

template <bool AK, bool BKC, int EPI>
__global__ __launch_bounds__(256) void fma_gemm_kernel(GemmDesc p) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float sa[BK][BM + 1];
  __shared__ float sb[BK][BN + 1];
  const TileSpace ts = tile_space<BM, BN>(p);
  const int id = tile_at(ts, (int)(blockIdx.x >> 3));
  if (id < 0) return;
  TileCoord t = resolve_tile<BM, BN>(p, ts, id, 4);
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
      const float a = acc[i][j] + ((EPI == EPI_STORE || EPI == EPI_GELU) && t.bias ? ((const float*)t.bias)[col] : 0.0f);
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

__global__ __launch_bounds__(1024) void build_tile_map_kernel(const int* __restrict__ offsets, int groups, int tile_rows, int* __restrict__ tile_map) {
  build_tile_map_block(offsets, groups, tile_rows, tile_map);
}

// out[i .. i+4) = (beta ? out : 0) + sum_z part[z*n + i ..]: one float4 of the output per thread;
// slices are summed in ascending order, eight loads in flight
__device__ __forceinline__ void reduce_slices(const float* __restrict__ part, int nslices, size_t n, float* __restrict__ out, int beta, size_t i) {
  if (i >= n) return;
  if ((n & 3) == 0) {   // then every slice keeps the 16-byte alignment
    float4 s = beta ? *(const float4*)(out + i) : make_float4(0.f, 0.f, 0.f, 0.f);
    int z = 0;
    for (; z + 8 <= nslices; z += 8) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *(const float4*)(part + (size_t)(z + u) * n + i);
#pragma unroll
      for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
    for (; z < nslices; ++z) {
      const float4 v = *(const float4*)(part + (size_t)z * n + i);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *(float4*)(out + i) = s;
  } else {
    for (size_t e = i; e < n && e < i + 4; ++e) {
      float s = beta ? out[e] : 0.0f;
      for (int z = 0; z < nslices; ++z) s += part[(size_t)z * n + e];
      out[e] = s;
    }
  }
}
__global__ void reduce_partials_kernel(const float* __restrict__ part, int nslices, size_t n, float* __restrict__ out, int beta) {
  reduce_slices(part, nslices, n, out, beta, ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4);
}
struct ReduceJobs {
  ReduceJob job[3];
};
__global__ void reduce_partials_multi_kernel(ReduceJobs jobs, int beta) {
  const ReduceJob j = jobs.job[blockIdx.y];
  reduce_slices(j.part, j.nslices, j.n, j.out, beta, ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4);
}

int gemm_ragged_tile_rows(int dtype, int tall_tile) { return dtype == BIGMAC_BF16 ? (tall_tile ? BIGMAC_TALL_BM : BIGMAC_TILE_BM) : 64; }

int launch_build_tile_map(const int* offsets, int groups, int tile_rows, int* tile_map, hipStream_t s) {
  if (groups > 1024) return BIGMAC_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(build_tile_map_kernel, dim3(1), dim3(1024), 0, s, offsets, groups, tile_rows, tile_map);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

// out[i] = bf16(sum_z part[z*n + i]), slices summed in ascending order; n a multiple of 8
__global__ void reduce_partials_bf16_kernel(const float* __restrict__ part, int nslices, size_t n, bf16_t* __restrict__ out) {
  const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (i >= n) return;
  float acc[8] = {};
  for (int z = 0; z < nslices; ++z) {
    const float4 a = *(const float4*)(part + (size_t)z * n + i), b = *(const float4*)(part + (size_t)z * n + i + 4);
    acc[0] += a.x; acc[1] += a.y; acc[2] += a.z; acc[3] += a.w;
    acc[4] += b.x; acc[5] += b.y; acc[6] += b.z; acc[7] += b.w;
  }
  *(uint4*)(out + i) = pack_bf16x8(acc);
}

int launch_reduce_partials_bf16(const float* part, int nslices, size_t n, void* out, hipStream_t s) {
  if (n % 8) return BIGMAC_ERR_INVALID_ARG;
  hipLaunchKernelGGL(reduce_partials_bf16_kernel, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, s, part, nslices, n, (bf16_t*)out);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

int launch_reduce_partials(const float* part, int nslices, size_t n, float* out, int beta, hipStream_t s) {
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, s, part, nslices, n, out, beta);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

int launch_reduce_partials_multi(const ReduceJob* jobs, int count, int beta, hipStream_t s) {
  if (count < 1 || count > 3) return BIGMAC_ERR_INVALID_ARG;
  ReduceJobs all = {};
  size_t longest = 0;
  for (int i = 0; i < count; ++i) {
    all.job[i] = jobs[i];
    if (jobs[i].n > longest) longest = jobs[i].n;
  }
  hipLaunchKernelGGL(reduce_partials_multi_kernel, dim3((unsigned)((longest + 1023) / 1024), count), dim3(256), 0, s, all, beta);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

namespace {

// One-dimensional launch, a multiple of the 8 XCDs.  `persistent`: at most two workgroups per CU
// (256 CUs), each walking several tiles; otherwise one workgroup per tile (surplus ones exit).
template <int BM, int BN>
dim3 grid_for(const GemmDesc& g, bool persistent, int blocks_per_cu = 0) {
  long gx = (g.N + BN - 1) / BN, gy, gz = 1;
  if (g.mode == GEMM_RAGGED_M) gy = g.max_rows / BM + g.groups + 1;
  else gy = (g.M + BM - 1) / BM;
  if (g.mode == GEMM_RAGGED_K) gz = g.groups;
  if (g.mode == GEMM_DENSE) gz = g.ksplit;
  long blocks = (gx * gy * gz + 7) / 8 * 8;
  const long resident = 256 * (blocks_per_cu ? blocks_per_cu : BM > BIGMAC_TILE_BM ? BIGMAC_TALL_BLOCKS_PER_CU : BIGMAC_BLOCKS_PER_CU);
  if (persistent && blocks > resident) blocks = resident;
  return dim3((unsigned)blocks, 1, 1);
}

template <int BM, bool AK, bool BKC>
int launch_mfma(const GemmDesc& g, hipStream_t s) {
  constexpr int BN = BIGMAC_TILE_BN, BK = BIGMAC_TILE_BK, WMs = BIGMAC_TILE_WM, WNs = BIGMAC_TILE_WN;
  dim3 grid = grid_for<BM, BN>(g, true), block(64 * WMs * WNs);
#define BIGMAC_MFMA(EPI, OUTF32) \
  hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, WMs, WNs, AK, BKC, EPI, OUTF32>), grid, block, 0, s, g)
  if constexpr (AK && !BKC) {
    if (g.scatter) {  // scattered rows: the descending projection's plain bf16 store
      hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, WMs, WNs, AK, BKC, EPI_STORE, false, BIGMAC_TILE_STAGES, false, true>), grid, block, 0, s, g);
      BIGMAC_CHECK_LAUNCH();
      return BIGMAC_OK;
    }
    if (g.gather) {   // gathered rows: the two epilogues of the expert-up product
      if (g.epilogue == EPI_GELU)
        hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, WMs, WNs, AK, BKC, EPI_GELU, false, BIGMAC_TILE_STAGES, true>), grid, block, 0, s, g);
      else if (g.epilogue == EPI_STORE && !g.out_f32)
        hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, WMs, WNs, AK, BKC, EPI_STORE, false, BIGMAC_TILE_STAGES, true>), grid, block, 0, s, g);
      else
        return BIGMAC_ERR_UNSUPPORTED;
      BIGMAC_CHECK_LAUNCH();
      return BIGMAC_OK;
    }
  }
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

// 256 x 256 outputs by eight wavefronts (each 128 x 64, as in the tall tile), one workgroup per
// CU, 32-deep k tiles in a ring of four 32 KB stages.  Per flop it asks the L2 for two thirds of
// the operand bytes the tall tile does (see the comment at launch_gemm).
template <bool AK, bool BKC>
int launch_mfma_wide(const GemmDesc& g, hipStream_t s) {
  constexpr int BM = 256, BN = 256, BK = 32;
  dim3 grid = grid_for<BM, BN>(g, true, 1), block(512);
#define BIGMAC_MFMA_WIDE(EPI, OUTF32) \
  hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 2, 4, AK, BKC, EPI, OUTF32, 4>), grid, block, 0, s, g)
  if constexpr (AK && !BKC) {
    if (g.gather) {
      if (g.epilogue == EPI_GELU) hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 2, 4, AK, BKC, EPI_GELU, false, 4, true>), grid, block, 0, s, g);
      else if (g.epilogue == EPI_STORE && !g.out_f32)
        hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 2, 4, AK, BKC, EPI_STORE, false, 4, true>), grid, block, 0, s, g);
      else return BIGMAC_ERR_UNSUPPORTED;
      BIGMAC_CHECK_LAUNCH();
      return BIGMAC_OK;
    }
  }
  switch (g.epilogue) {
    case EPI_STORE:
      if (g.out_f32) BIGMAC_MFMA_WIDE(EPI_STORE, true);
      else BIGMAC_MFMA_WIDE(EPI_STORE, false);
      break;
    case EPI_GELU: BIGMAC_MFMA_WIDE(EPI_GELU, false); break;
    case EPI_DGELU: BIGMAC_MFMA_WIDE(EPI_DGELU, false); break;
    case EPI_ACCUM: BIGMAC_MFMA_WIDE(EPI_ACCUM, true); break;
    default: return BIGMAC_ERR_INVALID_ARG;
  }
#undef BIGMAC_MFMA_WIDE
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

// 128 x 256 outputs: the tall tile turned on its side (four wavefronts side by side, each 128 x 64;
// the same ring and registers).  For the expert-up product, whose A rows are k-contiguous (64
// bytes of a row per k tile, half a cache line) while its B rows are whole lines: half the A rows
// and twice the B columns per tile mean fewer of the half-line requests per flop, and an expert's
// last tile pads half as many rows.  Measured against the tall tile: expert-up -5.5 % at
// zipf_stress, -7 % at gpt_xl and gpt_6p7b; the two shared projections of the forward pass, which
// have the same operand layouts, -6 % and -9 % at zipf_stress.  (Products whose B is k-contiguous
// too gain nothing.)
int launch_mfma_long(const GemmDesc& g, hipStream_t s) {
  constexpr int BM = 128, BN = 256, BK = BIGMAC_TILE_BK;
  dim3 grid = grid_for<BM, BN>(g, true, BIGMAC_TALL_BLOCKS_PER_CU), block(256);
  if (g.epilogue == EPI_ACCUM) hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 1, 4, true, false, EPI_ACCUM, true>), grid, block, 0, s, g);
  else if (g.epilogue == EPI_STORE) {   // the dense projections
    if (g.scatter) hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 1, 4, true, false, EPI_STORE, false, BIGMAC_TILE_STAGES, false, true>), grid, block, 0, s, g);
    else if (g.out_f32) hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 1, 4, true, false, EPI_STORE, true>), grid, block, 0, s, g);
    else hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 1, 4, true, false, EPI_STORE, false>), grid, block, 0, s, g);
  } else if (g.gather) hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 1, 4, true, false, EPI_GELU, false, BIGMAC_TILE_STAGES, true>), grid, block, 0, s, g);
  else hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 1, 4, true, false, EPI_GELU, false>), grid, block, 0, s, g);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

// The 256 x 256 tile with 64-deep k tiles in a ring of two 64 KB stages: k-contiguous operands
// arrive as whole 128-byte lines, half the requests to the L2.  Plain stores and the GELU' epilogue.
template <bool AK, bool BKC>
int launch_mfma_wide64(const GemmDesc& g, hipStream_t s) {
  constexpr int BM = 256, BN = 256, BK = 64;
  dim3 grid = grid_for<BM, BN>(g, true, 1), block(512);
  if (g.gather || g.scatter) return BIGMAC_ERR_UNSUPPORTED;
  if (g.epilogue == EPI_DGELU) hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 2, 4, AK, BKC, EPI_DGELU, false, 2>), grid, block, 0, s, g);
  else if (g.epilogue != EPI_STORE) return BIGMAC_ERR_UNSUPPORTED;
  else if (g.out_f32) hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 2, 4, AK, BKC, EPI_STORE, true, 2>), grid, block, 0, s, g);
  else hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 2, 4, AK, BKC, EPI_STORE, false, 2>), grid, block, 0, s, g);
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

// Few output tiles under a long K (the shared projections onto the narrow width): twice the
// tiles and half the k steps.  128 x 64 outputs, 64-deep k tiles, four wavefronts stacked in M
// (each 32 x 64: the bf16 epilogue's strip), 72 KB of ring: two workgroups per CU.
// The square tile with 64-deep k tiles in a ring of two stages (64 KB, two workgroups per CU).  A
// k-contiguous operand then arrives as whole 128-byte lines; with 32-deep k tiles each of its
// lines is requested from the L2 twice, half a line per k tile.
template <bool AK, bool BKC>
int launch_mfma_widek(const GemmDesc& g, hipStream_t s) {
  constexpr int BM = 128, BN = 128, BK = 64;
  dim3 grid = grid_for<BM, BN>(g, false), block(256);
  if (grid.x > 512) grid.x = 512;
#define BIGMAC_MFMA_WIDEK(EPI, OUTF32) \
  hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 2, 2, AK, BKC, EPI, OUTF32, 2>), grid, block, 0, s, g)
  switch (g.epilogue) {
    case EPI_STORE:
      if (g.out_f32) BIGMAC_MFMA_WIDEK(EPI_STORE, true);
      else BIGMAC_MFMA_WIDEK(EPI_STORE, false);
      break;
    case EPI_GELU: BIGMAC_MFMA_WIDEK(EPI_GELU, false); break;
    case EPI_DGELU: BIGMAC_MFMA_WIDEK(EPI_DGELU, false); break;
    case EPI_ACCUM: BIGMAC_MFMA_WIDEK(EPI_ACCUM, true); break;
    default: return BIGMAC_ERR_INVALID_ARG;
  }
#undef BIGMAC_MFMA_WIDEK
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

template <bool AK, bool BKC>
int launch_mfma_deep(const GemmDesc& g, hipStream_t s) {
  constexpr int BM = 128, BN = 64, BK = 64;
  dim3 grid = grid_for<BM, BN>(g, false), block(256);
  if (grid.x > 512) grid.x = 512;
#define BIGMAC_MFMA_DEEP(EPI, OUTF32) \
  hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 4, 1, AK, BKC, EPI, OUTF32>), grid, block, 0, s, g)
  if (g.scatter) {   // the descending projection writing the dispatched rows (k-contiguous A, whole-line B only)
    if constexpr (AK && !BKC) hipLaunchKernelGGL((mfma_gemm_kernel<BM, BN, BK, 4, 1, AK, BKC, EPI_STORE, false, BIGMAC_TILE_STAGES, false, true>), grid, block, 0, s, g);
    else return BIGMAC_ERR_UNSUPPORTED;
  } else if (g.epilogue == EPI_ACCUM) BIGMAC_MFMA_DEEP(EPI_ACCUM, true);
  else if (g.out_f32) BIGMAC_MFMA_DEEP(EPI_STORE, true);
  else BIGMAC_MFMA_DEEP(EPI_STORE, false);
#undef BIGMAC_MFMA_DEEP
  BIGMAC_CHECK_LAUNCH();
  return BIGMAC_OK;
}

template <bool AK, bool BKC>
int launch_fma(const GemmDesc& g, hipStream_t s) {
  dim3 grid = grid_for<64, 64>(g, false), block(256);
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

// Matrix-core rate probe: every wavefront issues 32x32x16 bf16 MFMAs back to back on four
// independent accumulators held in registers; no memory traffic inside the loop.  What this
// reaches is the achievable dense bf16 peak that the products' rates are set against.
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, float* __restrict__ sink) {
  bf16x8_t a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(float)((threadIdx.x + i) & 3);
    b[i] = (__bf16)(float)((threadIdx.x * 3 + i) & 1);
  }
  f32x16_t acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  float total = 0.0f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) total += acc[j][v];
  if (total == -1.0f) sink[0] = total;   // never true (the sums are non-negative): keeps the loop alive
}

// flops issued by one launch of the probe
double launch_mfma_probe(int blocks, int iters, float* sink, hipStream_t s) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, s, iters, sink);
  if (hipGetLastError() != hipSuccess) return -1.0;
  return (double)blocks * 4 * iters * 16 * (2.0 * 32 * 32 * 16);
}

namespace {
struct ClaimPool { unsigned* base; int next; };
thread_local ClaimPool claim_pool = {nullptr, 0};
__global__ void clear_claims_kernel(unsigned* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}
}  // namespace
ClaimScope::ClaimScope(void* region, hipStream_t s) {
  const int n = CLAIM_SLOTS * CLAIM_SLOT_INTS;
  hipLaunchKernelGGL(clear_claims_kernel, dim3((n + 255) / 256), dim3(256), 0, s, (unsigned*)region, n);
  status = hipGetLastError() == hipSuccess ? BIGMAC_OK : BIGMAC_ERR_HIP;
  claim_pool = {status == BIGMAC_OK ? (unsigned*)region : nullptr, 0};
}
ClaimScope::~ClaimScope() { claim_pool = {nullptr, 0}; }

int launch_gemm(const GemmDesc& desc, hipStream_t s) {
  GemmDesc g = desc;
  // The claimed order for the ragged-M products only.  Measured on zipf_stress: the four per-expert
  // row products 13-19 % faster with it; the ragged-K weight gradients 40 % slower (the tiles of a
  // group all cost the same, and with the fixed stride every workgroup of an XCD is on the same
  // group and k range at once, which the claimed order breaks up); dense products level or 1-3 % slower.
  if (!g.claim && g.dtype == BIGMAC_BF16 && g.mode == GEMM_RAGGED_M && claim_pool.base && claim_pool.next < CLAIM_SLOTS)
    g.claim = claim_pool.base + (size_t)CLAIM_SLOT_INTS * claim_pool.next++;
  // host-side shape checks: the kernels move 16-byte chunks and 64-wide k tiles
  if (g.N <= 0 || (g.mode != GEMM_RAGGED_M && g.M <= 0) || (g.mode != GEMM_RAGGED_K && g.K <= 0)) return BIGMAC_ERR_INVALID_ARG;
  if (g.mode != GEMM_DENSE && (!g.offsets || g.groups <= 0)) return BIGMAC_ERR_INVALID_ARG;
  if (g.mode == GEMM_RAGGED_M && !g.tile_map) return BIGMAC_ERR_INVALID_ARG;
  if (g.dtype == BIGMAC_BF16) {
    // (a k-contiguous operand is moved in whole k tiles: past a K that is no multiple of the
    // tile the next row's elements would follow, not zeros)
    if (g.lda % 8 || g.ldb % 8 || g.N % 8 || ((g.a_kcontig || g.b_kcontig) && g.K % BIGMAC_TILE_BK) ||
        (g.mode != GEMM_RAGGED_M && !g.a_kcontig && g.M % 8) || g.kwrap_b % 64)
      return BIGMAC_ERR_INVALID_ARG;
    if ((g.a_kcontig || g.b_kcontig) && g.mode == GEMM_RAGGED_K) return BIGMAC_ERR_UNSUPPORTED;  // k ranges start anywhere
  }
  if (g.mode == GEMM_DENSE && g.ksplit < 1) return BIGMAC_ERR_INVALID_ARG;
  if (g.dtype == BIGMAC_BF16) {
    // A tile's operand is one buffer addressed by 32-bit byte offsets whose top bit marks "out of
    // range".  Operands whose rows are the k index span (k range) x pitch bytes per tile: the whole
    // K of a dense product, at most all rows of a ragged-K one (max_rows, when the caller gives it).
    const size_t krows = g.mode == GEMM_RAGGED_K ? (size_t)(g.max_rows > 0 ? g.max_rows : 0) : (size_t)g.K;
    const size_t limit = 1ull << 31;
    if ((!g.a_kcontig && krows * (size_t)g.lda * 2 >= limit) || (!g.b_kcontig && krows * (size_t)g.ldb * 2 >= limit) ||
        (g.a_kcontig && 256ull * (size_t)g.lda * 2 >= limit) || (g.b_kcontig && 256ull * (size_t)g.ldb * 2 >= limit))
      return BIGMAC_ERR_TOO_LARGE;
  }
  const int combo = g.a_kcontig * 2 + g.b_kcontig;
  if (g.gather) {   // see the kernel: ragged-M rows of a k-contiguous A through an index, B not k-contiguous
    if (g.dtype != BIGMAC_BF16 || g.mode != GEMM_RAGGED_M || combo != 2 || g.wide_k || g.deep_tile || g.gather_rows <= 0 || g.gather_div <= 0 ||
        (size_t)g.gather_rows * (size_t)g.lda * 2 >= (1ull << 31))
      return BIGMAC_ERR_UNSUPPORTED;
  }
  if (g.scatter) {  // see the kernel: a dense bf16 product's rows written through an index, the same operand layout as above
    if (g.dtype != BIGMAC_BF16 || g.mode != GEMM_DENSE || combo != 2 || g.epilogue != EPI_STORE || g.out_f32 || g.ksplit != 1 || g.wide_k ||
        g.big_tile || g.gather || g.bias || g.scatter_k <= 0 || g.scatter_rows <= 0 ||
        (size_t)g.M * (size_t)g.scatter_k * 4 >= (1ull << 31) || (size_t)g.scatter_rows * (size_t)g.ldc * 2 >= (1ull << 31))
      return BIGMAC_ERR_UNSUPPORTED;
  }
  if (g.long_tile) {   // the expert-up product and the forward pass's shared projections
    const bool expert_up = g.mode == GEMM_RAGGED_M && g.epilogue == EPI_GELU && !g.scatter;
    const bool projection = g.mode == GEMM_DENSE && (g.epilogue == EPI_STORE || g.epilogue == EPI_ACCUM) && g.ksplit == 1 && !g.gather &&
                            (!g.scatter || g.epilogue == EPI_STORE);
    if (g.dtype != BIGMAC_BF16 || combo != 2 || !(expert_up || projection) || g.tall_tile || g.big_tile || g.wide_k || g.deep_tile)
      return BIGMAC_ERR_INVALID_ARG;
    return launch_mfma_long(g, s);
  }
  if (g.big_tile) {
    if (g.dtype != BIGMAC_BF16 || g.tall_tile || g.wide_k || g.deep_tile || g.touch_bytes) return BIGMAC_ERR_INVALID_ARG;
    // k-contiguous A and a K of whole 64-deep k tiles: the 64-deep form (whole-line requests).  Measured at
    // zipf_stress against the 32-deep ring of four: expert-down -3.5 %, the first matrix's data gradient
    // (both operands k-contiguous) -8.3 %, the GELU' product -1.3 %; expert-up +6 %, which keeps its own tile.
    if (g.a_kcontig && g.K % 64 == 0 && !g.gather && (g.epilogue == EPI_STORE || g.epilogue == EPI_DGELU))
      return g.b_kcontig ? launch_mfma_wide64<true, true>(g, s) : launch_mfma_wide64<true, false>(g, s);
    switch (combo) {
      case 2: return launch_mfma_wide<true, false>(g, s);
      case 3: return launch_mfma_wide<true, true>(g, s);
      case 0: return launch_mfma_wide<false, false>(g, s);
      default: return BIGMAC_ERR_UNSUPPORTED;
    }
  }
  if (g.dtype == BIGMAC_BF16) {
    if (g.wide_k) {
      if (g.mode == GEMM_RAGGED_K || g.tall_tile || g.deep_tile || !g.a_kcontig || g.K % 64) return BIGMAC_ERR_INVALID_ARG;
      return g.b_kcontig ? launch_mfma_widek<true, true>(g, s) : launch_mfma_widek<true, false>(g, s);
    }
    if (g.deep_tile) {
      if (g.mode != GEMM_DENSE || (g.epilogue != EPI_STORE && g.epilogue != EPI_ACCUM) || g.tall_tile ||
          ((g.a_kcontig || g.b_kcontig) && g.K % 64))
        return BIGMAC_ERR_INVALID_ARG;
      switch (combo) {
        case 2: return launch_mfma_deep<true, false>(g, s);
        case 3: return launch_mfma_deep<true, true>(g, s);
        case 0: return launch_mfma_deep<false, false>(g, s);
        default: return BIGMAC_ERR_UNSUPPORTED;
      }
    }
    if (g.tall_tile) {
      switch (combo) {
        case 2: return launch_mfma<BIGMAC_TALL_BM, true, false>(g, s);
        case 3: return launch_mfma<BIGMAC_TALL_BM, true, true>(g, s);
        case 0: return launch_mfma<BIGMAC_TALL_BM, false, false>(g, s);
        default: return BIGMAC_ERR_UNSUPPORTED;
      }
    }
    switch (combo) {
      case 2: return launch_mfma<BIGMAC_TILE_BM, true, false>(g, s);
      case 3: return launch_mfma<BIGMAC_TILE_BM, true, true>(g, s);
      case 0: return launch_mfma<BIGMAC_TILE_BM, false, false>(g, s);
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
