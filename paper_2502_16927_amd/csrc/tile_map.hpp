// Tile map of a ragged-M problem (rows grouped by expert) and the cost-balanced schedule of the
// ragged-K one, built by one workgroup of 1024 threads: by the kernel of its own in gemm.hip, or at
// the end of the counting sort's scan, which has the group offsets at hand.
#pragma once
#include <hip/hip_runtime.h>

namespace bigmac {

constexpr int TILE_MAP_HEADER = 16;   // ints in front of the group order: [0] tile count, [1..9] split points of the ragged-K schedule;
                                      // then `groups` ints of group order (positions -> groups), then the (group, first row) pairs
constexpr int TILE_MAP_K_ROWS = 32;   // rows per k tile in the cost of a group (the square tile's depth)

struct TileMapJobs {   // up to two maps (different tile heights) from one set of offsets; map == NULL: none
  int tile_rows[2];
  int* map[2];
};

// The map for at most 64 groups by one wavefront (lane = group): shuffles take the place of the
// LDS arrays of the general form below, which it follows step by step.
__device__ __forceinline__ void build_tile_map_wave(const int* offsets, int groups, int tile_rows, int* __restrict__ tile_map) {
  const int g = threadIdx.x & 63;
  int beg = 0, rows = 0, cnt = 0;
  if (g < groups) {
    beg = offsets[g];
    rows = offsets[g + 1] - beg;
    cnt = (rows + tile_rows - 1) / tile_rows;
  }
  auto inclusive_scan = [&](int v) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int o = __shfl_up(v, d, 64);
      if (g >= d) v += o;
    }
    return v;
  };
  const int last_tile = inclusive_scan(cnt);
  const int first = last_tile - cnt;
  for (int i = 0; i < cnt; ++i) {
    tile_map[TILE_MAP_HEADER + groups + 2 * (first + i)] = g;
    tile_map[TILE_MAP_HEADER + groups + 1 + 2 * (first + i)] = beg + i * tile_rows;
  }
  if (g < groups) tile_map[TILE_MAP_HEADER + g] = g;   // ragged-K schedule: the groups in their own order
  if (g == 63) tile_map[0] = last_tile;
  const int cost = g < groups ? (rows + TILE_MAP_K_ROWS - 1) / TILE_MAP_K_ROWS + 8 : 0;
  const int upto = inclusive_scan(cost);
  const long long total = __shfl(upto, 63, 64);
  // cost in front of position q = group * 65536 + fraction (every lane takes part in the shuffles)
  auto cost_before = [&](long long q) {
    const int gi = (int)(q >> 16);
    const int src = gi < 64 ? gi : 63;
    const int incl_gi = __shfl(upto, src, 64), cost_gi = __shfl(cost, src, 64);
    if (gi >= groups) return total;
    return (long long)(incl_gi - cost_gi) + (((q & 0xFFFF) * cost_gi) >> 16);
  };
  const int x8 = g < 8 ? g : 7;
  const long long q0 = ((long long)groups * x8 << 16) / 8, q1 = ((long long)groups * (x8 + 1) << 16) / 8;
  long long worst_run = cost_before(q1) - cost_before(q0);
#pragma unroll
  for (int off = 1; off < 8; off <<= 1) {
    const long long o = __shfl_xor(worst_run, off, 64);
    worst_run = o > worst_run ? o : worst_run;
  }
  worst_run = __shfl(worst_run, 0, 64);
  const bool balanced = worst_run * 64 > total * 9;
#pragma unroll 1
  for (int x = 0; x <= 8; ++x) {
    if (!balanced) {
      if (g == 0) tile_map[1 + x] = (int)(((long long)groups * x << 16) / 8);
      continue;
    }
    const long long target = total * x / 8;
    if (x == 8) {
      if (g == 0) tile_map[1 + x] = groups << 16;
    } else if (cost > 0 && target >= upto - cost && target < upto) {
      tile_map[1 + x] = (g << 16) | (int)(((target - (upto - cost)) << 16) / cost);
    }
  }
}

// tile_map[0] = number of M tiles, [1..9] = the split points of the cost-balanced ragged-K
// schedule (see balance_ragged_k), then from TILE_MAP_HEADER on (group, first row) per M tile,
// groups in order.  Called by all 1024 threads of a workgroup, one thread per group; offsets may
// lie in the LDS.
// schedule_from: a map built before this one by the same workgroup from the same offsets; its
// ragged-K schedule (split points and group order do not depend on the tile height) is copied
// instead of being worked out again.
// Forced inline, like every device function of this library: left to the compiler, the second
// call site turned this into a real call (stack pointer, scratch, LDS of the callee in a
// module-wide block), and the one-workgroup counting sort that calls it then lost the counters
// of whole wavefronts from run to run; inlined, the same source is deterministic.
__device__ __forceinline__ void build_tile_map_block(const int* offsets, int groups, int tile_rows, int* __restrict__ tile_map,
                                            const int* schedule_from = nullptr) {
  if (groups <= 64) {                // one wavefront holds every group: the same steps without LDS or barriers
    if (threadIdx.x < 64) build_tile_map_wave(offsets, groups, tile_rows, tile_map);
    return;
  }
  __shared__ int scan[16];
  __syncthreads();                   // a previous call in the same kernel may still read the shared arrays
  const int g = threadIdx.x;
  int beg = 0, rows = 0, cnt = 0;
  if (g < groups) {
    beg = offsets[g];
    rows = offsets[g + 1] - beg;
    cnt = (rows + tile_rows - 1) / tile_rows;
  }
  // inclusive scan over the 1024 threads: shuffles inside each wavefront, the 16 wavefront totals through LDS
  auto inclusive_scan = [&](int v) {
    const int lane = g & 63, wave = g >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int o = __shfl_up(v, d, 64);
      if (lane >= d) v += o;
    }
    __syncthreads();
    if (lane == 63) scan[wave] = v;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += scan[w];
    return v + before;
  };
  const int last_tile = inclusive_scan(cnt);
  const int first = last_tile - cnt;
  for (int i = 0; i < cnt; ++i) {
    tile_map[TILE_MAP_HEADER + groups + 2 * (first + i)] = g;
    tile_map[TILE_MAP_HEADER + groups + 1 + 2 * (first + i)] = beg + i * tile_rows;
  }
  if (g == 1023) tile_map[0] = last_tile;
  if (schedule_from) {
    __syncthreads();                 // the other map's entries were written by this workgroup
    if (g < 9) tile_map[1 + g] = schedule_from[1 + g];
    if (g < groups) tile_map[TILE_MAP_HEADER + g] = schedule_from[TILE_MAP_HEADER + g];
    return;
  }
  // split points: cost of a group = its k tiles + 8 (set-up and epilogue of a tile, in k tiles)
  __shared__ int cost_of[1024];
  __shared__ int incl[1024];
  __shared__ long long worst_run;
  const int cost = g < groups ? (rows + TILE_MAP_K_ROWS - 1) / TILE_MAP_K_ROWS + 8 : 0;
  const int upto = inclusive_scan(cost);
  cost_of[g] = cost;
  incl[g] = upto;
  if (g == 0) worst_run = 0;
  __syncthreads();
  const long long total = incl[1023];
  // cost in front of position q = group * 65536 + fraction
  auto cost_before = [&](long long q) {
    const int gi = (int)(q >> 16);
    if (gi >= groups) return total;
    return (long long)(incl[gi] - cost_of[gi]) + (((q & 0xFFFF) * cost_of[gi]) >> 16);
  };
  // Near-uniform routing: runs of equal tile counts are as good and keep whole groups together,
  // and the workgroups of an XCD then get equal numbers of tiles.  Use the cost-balanced cut
  // only where the equal cut would leave an XCD more than 1/8 over its share.
  if (g < 8) {
    const long long q0 = ((long long)groups * g << 16) / 8, q1 = ((long long)groups * (g + 1) << 16) / 8;
    atomicMax((unsigned long long*)&worst_run, (unsigned long long)(cost_before(q1) - cost_before(q0)));
  }
  __syncthreads();
  const bool balanced = worst_run * 64 > total * 9;
  // Skewed routing.  Runs of *whole* groups are preferred to runs of equal cost: all tiles of a
  // group cost the same, so with whole groups the workgroups of an XCD move from group to group
  // together and read the group's operand panels through the L2 once, while a run that starts
  // inside a group puts two groups of different cost into every round of the stride, the
  // workgroups drift apart for the rest of the launch and re-read the panels from memory
  // (measured on zipf_stress: the two weight-gradient products 1.31 -> 1.07 ms and 1.30 -> 1.12
  // ms).  The groups are dealt out largest first, each to the XCD with the least cost so
  // far; the map's group order lists the groups XCD by XCD, each XCD's largest first, and the
  // split points are the XCDs' first positions.  Used when the fullest XCD stays within 1.2
  // times the even share (one group that outweighs an eighth of the work does not); else the
  // groups keep their own order and the cut of equal cost.
  // (16-bit entries: the counting sort's one-workgroup kernels call this with 40 KB of LDS of
  // their own, and a kernel's static LDS ends at 64 KB)
  __shared__ unsigned short by_cost[1024];      // groups, largest cost first (ties: lower index first)
  __shared__ unsigned short xcd_of[1024], place_in_xcd[1024];
  __shared__ int xcd_first[9];
  __shared__ int whole_ok;
  if (g < groups) {
    int rank = 0;
    for (int o = 0; o < groups; ++o) {
      const int co = cost_of[o];
      rank += (co > cost || (co == cost && o < g)) ? 1 : 0;
    }
    by_cost[rank] = (unsigned short)g;
  }
  if (g == 0) whole_ok = 0;
  __syncthreads();
  if (balanced && g < 64) {
    // the first wavefront: lane x < 8 keeps XCD x's cost and count; a step finds the least loaded
    // XCD by a minimum over (cost * 8 + x) across the eight lanes
    unsigned load = 0;
    int count = 0;
    const int lane8 = g & 7;
    for (int r0 = 0; r0 < groups; r0 += 8) {
      int grp[8], c[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {                   // eight independent reads, then eight dependent steps
        grp[u] = by_cost[r0 + u < groups ? r0 + u : groups - 1];
        c[u] = cost_of[grp[u]];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (r0 + u >= groups) break;
        unsigned key = (load << 3) | (unsigned)lane8;
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) {
          const unsigned o = (unsigned)__shfl_xor((int)key, off, 64);
          key = o < key ? o : key;
        }
        const int best = (int)(key & 7u);
        if (lane8 == best) {
          if (g < 8) {
            xcd_of[grp[u]] = (unsigned short)best;
            place_in_xcd[grp[u]] = (unsigned short)count;
          }
          load += (unsigned)c[u];
          ++count;
        }
      }
    }
    // fullest XCD and the first position of each
    unsigned fullest = load;
    int before = count;
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) {
      const unsigned o = (unsigned)__shfl_xor((int)fullest, off, 64);
      fullest = o > fullest ? o : fullest;
      const int b = __shfl_up(before, off, 64);       // inclusive scan of the counts over lanes 0..7
      if (lane8 >= off) before += b;
    }
    if (g < 8) xcd_first[g] = before - count;
    if (g == 0) {
      xcd_first[8] = groups;
      whole_ok = (long long)fullest * 40 <= total * 6;   // <= 1.2 x total / 8
    }
  }
  __syncthreads();
  if (g < groups) tile_map[TILE_MAP_HEADER + (whole_ok ? xcd_first[xcd_of[g]] + place_in_xcd[g] : g)] = g;
#pragma unroll 1
  for (int x = 0; x <= 8; ++x) {
    if (whole_ok) {
      if (g == 0) tile_map[1 + x] = xcd_first[x] << 16;
      continue;
    }
    if (!balanced) {
      if (g == 0) tile_map[1 + x] = (int)(((long long)groups * x << 16) / 8);
      continue;
    }
    const long long target = total * x / 8;
    if (x == 8) {
      if (g == 0) tile_map[1 + x] = groups << 16;
    } else if (cost > 0 && target >= upto - cost && target < upto) {
      tile_map[1 + x] = (g << 16) | (int)(((target - (upto - cost)) << 16) / cost);
    }
  }
}

}  // namespace bigmac
