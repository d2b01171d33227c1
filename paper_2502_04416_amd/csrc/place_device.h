// Slot assignment of one 64-token tile (shared by the permute kernel and the decode front end).
#pragma once
#include "cmoe_internal.h"
#include "device_utils.h"

namespace cmoe {

constexpr int N_XCD = 8;              // dies with an L2 of their own; workgroup b runs on die b % 8
constexpr int TILE_FIXED_COST = 4;    // prologue + epilogue of a tile, in units of one 64-deep K step

struct PlaceArgs {
  const int32_t* sel_group;    // [T][S_dyn]
  const float* sel_weight;     // [T][S_dyn]
  const int32_t* tile_counts;  // [n_tiles][G]
  const GroupDev* groups;
  int32_t* seg_off;            // [G+1]
  int32_t* counts;             // [G]
  int32_t* work1;              // [G+1] prefix of work items, then [N_XCD+1] first item of each die's share
  int32_t* work2;              // same for the down contraction
  int64_t* h_off;              // [G+1]
  int32_t* slot2tok;           // [n_slots]
  int32_t* tok2slot;           // [T][S_all]
  float* slot_w;               // [T][S_all]
  float* w_by_slot;            // [n_slots] the same weights indexed by slot
  int32_t* counts_out;         // optional user output: counts of the routed groups [G - n_always]
  int64_t T;
  int G, n_always, S_dyn, n_tiles;
  int bm1, bn1, bm2, bn2, d;   // tile sizes of the grouped GEMMs (bn1 in packed gate/up rows)
  int dyn1, dyn2;              // > 0: that contraction runs tiles of dynamic height, in steps of this many rows (a
                               // ragged last tile costs its rows)
  int decode;                  // 1: the work lists count decode units (dec_unit1 neurons / 16 output columns per unit)
  int dec_unit1;               // neurons per gate/up unit of the decode kernels (16 or 8)
  int skip_always;             // 1: no gate/up work items for the always-on groups (another launch ran them)
};

// All 64 callers are one wave: the LDS operations of a wave are carried out in the order it issued them, so
// waiting for its outstanding ones (and keeping the compiler from moving LDS accesses across this point) is
// enough to hand data between its lanes.  Deliberately not a fence: a workgroup-scope fence also waits for
// every global store the wave has in flight, which nothing here needs.
__device__ __forceinline__ void wave_lds_sync() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_wave_barrier();
}

// Padded widths of the (at most two) groups a lane looks after in place_tile; a caller with other work to
// do first requests them early so that their latency is hidden.
struct LaneWidths { int w[MAX_GROUPS / 64]; };
__device__ __forceinline__ LaneWidths load_lane_widths(const PlaceArgs& p, int lane) {
  LaneWidths lw;
#pragma unroll
  for (int k = 0; k < MAX_GROUPS / 64; ++k) {
    const int g = lane + 64 * k;
    lw.w[k] = (g < p.G) ? p.groups[g].width_pad : 0;
  }
  return lw;
}

// One wave places one 64-token tile.  `counts` is the per-tile histogram table [n_tiles][G] (global memory, or
// LDS when the caller is the single-tile decode front end); sel_g / sel_w are the routed entries
// [T][S_dyn] (the workspace arrays, or an LDS copy of the caller).  Must be called by exactly 64 threads
// (lane = id).  Cost is O(S_dyn + G/64) per lane: the prefix over groups is a wave scan (two groups per
// lane), and the rank of a token inside its group comes from a 64-bit presence mask per group that the
// lanes build with LDS atomics, not from a pass over all groups.
__device__ __forceinline__ void place_tile(const PlaceArgs& p, int tile, const int32_t* counts, int lane,
                                           const int32_t* sel_g, const float* sel_w, const LaneWidths& lw) {
  constexpr int GPL = MAX_GROUPS / 64;      // groups per lane
  __shared__ int32_t base[MAX_GROUPS];      // first slot of each group for this tile
  __shared__ uint32_t present[MAX_GROUPS][2];   // which lanes (tokens of the tile) have an entry for the group
  const int S_all = p.n_always + p.S_dyn;
  const int64_t t = (int64_t)tile * TOK_TILE + lane;
  const bool valid = t < p.T;
  // this token's routed entries, requested first: nothing below depends on them until the marking pass
  // (S_dyn and G are the same for every lane: the unrolled loops below leave at the first unused entry
  // through a scalar branch instead of running all MAX_DYN predicated bodies; one wave pays four cycles
  // for every vector instruction, used or not)
  int my_g[MAX_DYN];
  float my_w[MAX_DYN];
#pragma unroll
  for (int i = 0; i < MAX_DYN; ++i) {
    if (i >= p.S_dyn) break;
    my_g[i] = valid ? sel_g[t * p.S_dyn + i] : -1;
    my_w[i] = valid ? sel_w[t * p.S_dyn + i] : 0.0f;
  }
#pragma unroll
  for (int k = 0; k < GPL; ++k) {
    present[lane + 64 * k][0] = 0u;
    present[lane + 64 * k][1] = 0u;
  }
  // totals and the count of all preceding tiles for this lane's groups
  int tot[GPL], prev[GPL];
#pragma unroll
  for (int k = 0; k < GPL; ++k) {
    const int g = lane + 64 * k;
    tot[k] = 0;
    prev[k] = 0;
    if (64 * k >= p.G) continue;            // no lane has a group in this half
    if (g < p.G) {
      if (g < p.n_always) {
        tot[k] = (int)p.T;
      } else {
        // independent loads, sixteen in flight at a time (the compiler does not batch them by itself)
        int i = 0;
        for (; i + 16 <= p.n_tiles; i += 16) {
          int c[16];
#pragma unroll
          for (int q = 0; q < 16; ++q) c[q] = counts[(int64_t)(i + q) * p.G + g];
#pragma unroll
          for (int q = 0; q < 16; ++q) {
            tot[k] += c[q];
            prev[k] += (i + q < tile) ? c[q] : 0;
          }
        }
        for (; i < p.n_tiles; ++i) {
          const int c = counts[(int64_t)i * p.G + g];
          tot[k] += c;
          prev[k] += (i < tile) ? c : 0;
        }
      }
    }
  }
  wave_lds_sync();                          // the cleared masks are visible to every lane
#pragma unroll
  for (int i = 0; i < MAX_DYN; ++i) {
    if (i >= p.S_dyn) break;
    if (my_g[i] >= 0) atomicOr(&present[my_g[i]][lane >> 5], 1u << (lane & 31));
  }
  // exclusive prefix over groups of: slots, work items of the two contractions, hidden-buffer elements
  int run0 = 0, w1_0 = 0, w2_0 = 0;
  long long h0 = 0;
  int n1[GPL], n2[GPL], w1x[GPL], w2x[GPL];     // work items of this lane's groups and their exclusive prefix
#pragma unroll
  for (int k = 0; k < GPL; ++k) {
    const int g = lane + 64 * k;
    if (k > 0 && 64 * k >= p.G) {           // nothing to add: skip this half's four scans
      n1[k] = 0; n2[k] = 0; w1x[k] = w1_0; w2x[k] = w2_0;
      continue;
    }
    const int cnt = tot[k], wp = lw.w[k];
    int a1, a2;
    if (p.decode) {
      a1 = cnt > 0 ? wp / p.dec_unit1 : 0;
      a2 = cnt > 0 ? p.d / 16 : 0;
    } else {
      a1 = cdiv(cnt, p.bm1) * cdiv(2 * wp, p.bn1);
      a2 = cdiv(cnt, p.bm2) * cdiv(p.d, p.bn2);
    }
    if (g >= p.G) { a1 = 0; a2 = 0; }
    if (p.skip_always && g < p.n_always) a1 = 0;
    const long long ah = (long long)cnt * wp;
    const int run_i = wave_incl_scan(cnt, lane), w1_i = wave_incl_scan(a1, lane), w2_i = wave_incl_scan(a2, lane);
    const long long h_i = wave_incl_scan(ah, lane);
    const int run = run0 + run_i - cnt, w1 = w1_0 + w1_i - a1, w2 = w2_0 + w2_i - a2;
    const long long h = h0 + h_i - ah;
    n1[k] = a1; n2[k] = a2; w1x[k] = w1; w2x[k] = w2;
    if (g < p.G) {
      base[g] = run + prev[k];
      if (tile == 0) {
        p.seg_off[g] = run;
        p.counts[g] = cnt;
        p.work1[g] = w1;
        p.work2[g] = w2;
        p.h_off[g] = h;
        if (p.counts_out && g >= p.n_always) p.counts_out[g - p.n_always] = cnt;
      }
    }
    run0 += __shfl(run_i, 63, 64);
    w1_0 += __shfl(w1_i, 63, 64);
    w2_0 += __shfl(w2_i, 63, 64);
    h0 += __shfl(h_i, 63, 64);
  }
  if (tile == 0) {
    if (lane == 0) {
      p.seg_off[p.G] = run0;
      p.work1[p.G] = w1_0;
      p.work2[p.G] = w2_0;
      p.h_off[p.G] = h0;
    }
  }
  if (tile == 0 && !p.decode) {            // (the decode kernels take their units in list order: no shares)
    // Where each XCD's share of a work list starts (entries G+1 .. G+9 of the list): contiguous ranges of
    // equal estimated cost, so that the tiles sharing operands stay in one L2 while the eight dies finish
    // together.  A tile costs its depth (K steps of 64, plus a fixed part for prologue and epilogue: the shared
    // group's down tiles are N_s times as deep as a routed expert's) times its height in 32-row blocks; with
    // tiles of dynamic height the ragged last row tile of a group costs its own blocks (at least three: below
    // that a tile is bound by fetching its weights), otherwise as much as a full one.  Inside a group the
    // boundary falls in proportion to the cost.
    __shared__ int32_t xs[2][N_XCD + 1];
    if (lane <= N_XCD) {
      xs[0][lane] = lane == N_XCD ? w1_0 : 0;
      xs[1][lane] = lane == N_XCD ? w2_0 : 0;
    }
    wave_lds_sync();
#pragma unroll
    for (int list = 0; list < 2; ++list) {
      const int bm = list == 0 ? p.bm1 : p.bm2, dyn = list == 0 ? p.dyn1 : p.dyn2;
      const int blocks_full = bm / 32 > 0 ? bm / 32 : 1;
      // (Which group a boundary falls into is decided in exact integers, so that every item lands in exactly
      // one share; where inside the group, in single precision: the shares need to be about equal, not exact,
      // and this wave is on the critical path of the whole forward: 64-bit divisions here doubled the
      // kernel's duration.)
      long long gc[GPL], gx[GPL];             // cost of this lane's groups and their exclusive prefix
      long long c0 = 0;
#pragma unroll
      for (int k = 0; k < GPL; ++k) {
        gc[k] = 0;
        gx[k] = c0;
        if (k > 0 && 64 * k >= p.G) continue;
        const int n_items = list == 0 ? n1[k] : n2[k];
        const int cnt = tot[k], wp = lw.w[k];
        if (n_items > 0) {
          const int row_tiles = cdiv(cnt, bm), col_tiles = n_items / row_tiles;
          const int depth = (list == 0 ? cdiv(p.d, 64) : cdiv(wp, 64)) + TILE_FIXED_COST;
          const int full = cnt / bm, rem = cnt - full * bm;
          int last = 0;
          if (rem > 0) {
            last = blocks_full;
            if (dyn) {
              last = cdiv(rem, dyn) * (dyn / 32);           // dyn = rows per height step
              const int floor_blocks = blocks_full < 3 ? blocks_full : 3;
              if (last < floor_blocks) last = floor_blocks;
            }
          }
          gc[k] = (long long)col_tiles * depth * (full * blocks_full + last);
        }
        const long long ci = wave_incl_scan(gc[k], lane);
        gx[k] = c0 + ci - gc[k];
        c0 += __shfl(ci, 63, 64);
      }
#pragma unroll
      for (int k = 0; k < GPL; ++k) {
        if (k > 0 && 64 * k >= p.G) continue;
        const int n_items = list == 0 ? n1[k] : n2[k];
        if (n_items <= 0) continue;
        const float per_item = (float)n_items / (float)gc[k];
        static_assert(N_XCD == 8, "the share boundaries divide by a shift");
#pragma unroll
        for (int x = 1; x < N_XCD; ++x) {
          const long long t = (x * c0) >> 3;
          if (gx[k] <= t && t < gx[k] + gc[k]) {
            int local = (int)((float)(t - gx[k]) * per_item);
            if (local > n_items - 1) local = n_items - 1;
            xs[list][x] = (list == 0 ? w1x[k] : w2x[k]) + local;
          }
        }
      }
    }
    wave_lds_sync();
    if (lane <= N_XCD) {
      p.work1[p.G + 1 + lane] = xs[0][lane];
      p.work2[p.G + 1 + lane] = xs[1][lane];
    }
  }
  wave_lds_sync();                          // base[] and present[] are complete
  // always-on groups: identity segments
  if (valid)
    for (int a = 0; a < p.n_always; ++a) {
      const int slot = a * (int)p.T + (int)t;
      p.slot2tok[slot] = (int)t;
      p.tok2slot[t * S_all + a] = slot;
      p.slot_w[t * S_all + a] = 1.0f;
      p.w_by_slot[slot] = 1.0f;
    }
  // routed entries: stable (token-ascending) rank inside the group = lower lanes present in its mask
  const uint32_t lt_lo = lane >= 32 ? 0xffffffffu : ((1u << lane) - 1u);
  const uint32_t lt_hi = lane > 32 ? ((1u << (lane - 32)) - 1u) : 0u;
#pragma unroll
  for (int i = 0; i < MAX_DYN; ++i) {
    if (i >= p.S_dyn) break;
    const int g = my_g[i];
    if (g < 0) continue;
    const int slot = base[g] + __popc(present[g][0] & lt_lo) + __popc(present[g][1] & lt_hi);
    p.slot2tok[slot] = (int)t;
    p.tok2slot[t * S_all + p.n_always + i] = slot;
    p.slot_w[t * S_all + p.n_always + i] = my_w[i];
    p.w_by_slot[slot] = my_w[i];
  }
}


}  // namespace cmoe
