// Slot assignment of one 64-token tile (shared by the permute kernel and the decode front end).
#pragma once
#include "cmoe_internal.h"
#include "device_utils.h"

namespace cmoe {

struct PlaceArgs {
  const int32_t* sel_group;    // [T][S_dyn]
  const float* sel_weight;     // [T][S_dyn]
  const int32_t* tile_counts;  // [n_tiles][G]
  const GroupDev* groups;
  int32_t* seg_off;            // [G+1]
  int32_t* counts;             // [G]
  int32_t* work1;              // [G+1]
  int32_t* work2;              // [G+1]
  int64_t* h_off;              // [G+1]
  int32_t* slot2tok;           // [n_slots]
  int32_t* tok2slot;           // [T][S_all]
  float* slot_w;               // [T][S_all]
  int32_t* counts_out;         // optional user output: counts of the routed groups [G - n_always]
  int64_t T;
  int G, n_always, S_dyn, n_tiles;
  int bm1, bn1, bm2, bn2, d;   // tile sizes of the grouped GEMMs (bn1 in packed gate/up rows)
  int decode;                  // 1: the work lists count decode units (16 neurons / 16 output columns per unit)
};

// All 64 callers are one wave: LDS traffic of a wave completes in order, so a workgroup-scope fence (which
// waits for this wave's outstanding LDS operations) is enough to hand data between its lanes.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
  __builtin_amdgcn_wave_barrier();
}

// One wave places one 64-token tile.  `counts` is the per-tile histogram table [n_tiles][G] (global memory, or
// LDS when the caller is the single-tile decode front end).  Must be called by exactly 64 threads (lane = id).
__device__ __forceinline__ void place_tile(const PlaceArgs& p, int tile, const int32_t* counts, int lane) {
  __shared__ int32_t base[MAX_GROUPS];      // next free slot of each group for this tile
  __shared__ int32_t total[MAX_GROUPS];
  __shared__ int32_t wpad[MAX_GROUPS];      // padded widths (read once, in parallel)
  const int S_all = p.n_always + p.S_dyn;
  const int64_t t = (int64_t)tile * TOK_TILE + lane;
  const bool valid = t < p.T;
  // this token's routed entries, requested first: nothing below depends on them until the group loop
  int my_g[MAX_DYN];
  float my_w[MAX_DYN];
#pragma unroll
  for (int i = 0; i < MAX_DYN; ++i) {
    const bool ok = valid && i < p.S_dyn;
    my_g[i] = ok ? p.sel_group[t * p.S_dyn + i] : -1;
    my_w[i] = ok ? p.sel_weight[t * p.S_dyn + i] : 0.0f;
  }
  // totals and the count of all preceding tiles, two groups per lane at most
  for (int g = lane; g < MAX_GROUPS; g += 64) {
    int tot = 0, prev = 0;
    if (g < p.G) {
      if (g < p.n_always) {
        tot = (int)p.T;
        prev = 0;
      } else {
        // independent loads, sixteen in flight at a time (the compiler does not batch them by itself)
        int i = 0;
        for (; i + 16 <= p.n_tiles; i += 16) {
          int c[16];
#pragma unroll
          for (int k = 0; k < 16; ++k) c[k] = counts[(int64_t)(i + k) * p.G + g];
#pragma unroll
          for (int k = 0; k < 16; ++k) {
            tot += c[k];
            prev += (i + k < tile) ? c[k] : 0;
          }
        }
        for (; i < p.n_tiles; ++i) {
          const int c = counts[(int64_t)i * p.G + g];
          tot += c;
          prev += (i < tile) ? c : 0;
        }
      }
    }
    total[g] = tot;
    base[g] = prev;
    wpad[g] = (g < p.G) ? p.groups[g].width_pad : 0;
  }
  wave_lds_sync();
  // exclusive scan over groups (G <= 128: a serial pass by lane 0 is a few hundred cycles)
  if (lane == 0) {
    int run = 0, w1 = 0, w2 = 0;
    int64_t h = 0;
    for (int g = 0; g < p.G; ++g) {
      const int cnt = total[g];
      const int wp = wpad[g];
      base[g] += run;
      if (tile == 0) {
        p.seg_off[g] = run;
        p.counts[g] = cnt;
        p.work1[g] = w1;
        p.work2[g] = w2;
        p.h_off[g] = h;
        if (p.counts_out && g >= p.n_always) p.counts_out[g - p.n_always] = cnt;
      }
      run += cnt;
      if (p.decode) {
        w1 += cnt > 0 ? wp / 16 : 0;
        w2 += cnt > 0 ? p.d / 16 : 0;
      } else {
        w1 += cdiv(cnt, p.bm1) * cdiv(2 * wp, p.bn1);
        w2 += cdiv(cnt, p.bm2) * cdiv(p.d, p.bn2);
      }
      h += (int64_t)cnt * wp;
    }
    if (tile == 0) {
      p.seg_off[p.G] = run;
      p.work1[p.G] = w1;
      p.work2[p.G] = w2;
      p.h_off[p.G] = h;
    }
  }
  wave_lds_sync();
  // always-on groups: identity segments
  if (valid)
    for (int a = 0; a < p.n_always; ++a) {
      const int slot = a * (int)p.T + (int)t;
      p.slot2tok[slot] = (int)t;
      p.tok2slot[t * S_all + a] = slot;
      p.slot_w[t * S_all + a] = 1.0f;
    }
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int g = p.n_always; g < p.G; ++g) {
    int hit = -1;
    float hit_w = 0.0f;
#pragma unroll
    for (int i = 0; i < MAX_DYN; ++i) {
      const bool m = my_g[i] == g;
      hit = m ? i : hit;
      hit_w = m ? my_w[i] : hit_w;
    }
    const uint64_t mask = __ballot(hit >= 0);
    if (mask == 0ull) continue;
    const int b = base[g];
    if (hit >= 0) {
      const int slot = b + __popcll(mask & lt_mask);
      p.slot2tok[slot] = (int)t;
      p.tok2slot[t * S_all + p.n_always + hit] = slot;
      p.slot_w[t * S_all + p.n_always + hit] = hit_w;
    }
  }
}


}  // namespace cmoe
