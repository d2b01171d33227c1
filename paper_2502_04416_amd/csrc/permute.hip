// Token -> expert permutation and the gate-weighted combine.
//
// place_kernel: from the routed (group, weight) entries of every token and the per-tile histograms,
// one wave per 64-token tile computes, with an exclusive prefix scan over groups and over preceding
// tiles, the slot of each entry.  Segments are contiguous per group and token-ascending inside a
// group, so the layout is a pure function of the routing decisions.  Tile 0 also publishes the segment
// offsets, counts, the work lists of the two grouped GEMMs and each group's offset in the ragged
// hidden-activation buffer.  Nothing is copied back to the host.
//
// combine_kernel: y[t] = sum over the token's slots of weight * Y[slot]  (Eq. 4 / Eq. 10), a gather,
// so there are no floating-point atomics and the result does not depend on scheduling.
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

__global__ __launch_bounds__(64) void place_kernel(PlaceArgs p) {
  __shared__ int32_t base[MAX_GROUPS];      // next free slot of each group for this tile
  __shared__ int32_t total[MAX_GROUPS];
  __shared__ int32_t wpad[MAX_GROUPS];      // padded widths (read once, in parallel)
  const int lane = threadIdx.x;
  const int tile = blockIdx.x;
  const int S_all = p.n_always + p.S_dyn;
  // totals and the count of all preceding tiles, two groups per lane at most
  for (int g = lane; g < MAX_GROUPS; g += 64) {
    int tot = 0, prev = 0;
    if (g < p.G) {
      if (g < p.n_always) {
        tot = (int)p.T;
        prev = 0;
      } else {
        // independent loads, eight in flight at a time (the compiler does not batch them by itself)
        int i = 0;
        for (; i + 8 <= p.n_tiles; i += 8) {
          int c[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) c[k] = p.tile_counts[(int64_t)(i + k) * p.G + g];
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            tot += c[k];
            prev += (i + k < tile) ? c[k] : 0;
          }
        }
        for (; i < p.n_tiles; ++i) {
          const int c = p.tile_counts[(int64_t)i * p.G + g];
          tot += c;
          prev += (i < tile) ? c : 0;
        }
      }
    }
    total[g] = tot;
    base[g] = prev;
    wpad[g] = (g < p.G) ? p.groups[g].width_pad : 0;
  }
  __syncthreads();
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
  __syncthreads();
  const int64_t t = (int64_t)tile * TOK_TILE + lane;
  const bool valid = t < p.T;
  // always-on groups: identity segments
  if (valid)
    for (int a = 0; a < p.n_always; ++a) {
      const int slot = a * (int)p.T + (int)t;
      p.slot2tok[slot] = (int)t;
      p.tok2slot[t * S_all + a] = slot;
      p.slot_w[t * S_all + a] = 1.0f;
    }
  // this token's routed entries, loaded up front so that no load sits inside the group loop below
  int my_g[MAX_DYN];
  float my_w[MAX_DYN];
#pragma unroll
  for (int i = 0; i < MAX_DYN; ++i) {
    const bool ok = valid && i < p.S_dyn;
    my_g[i] = ok ? p.sel_group[t * p.S_dyn + i] : -1;
    my_w[i] = ok ? p.sel_weight[t * p.S_dyn + i] : 0.0f;
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

hipError_t launch_permute(const Engine& e, int64_t T, char* ws, const WsLayout& L, int32_t* counts_out,
                          hipStream_t s) {
  if (T == 0) return hipSuccess;
  PlaceArgs p;
  p.sel_group = reinterpret_cast<const int32_t*>(ws + L.sel_group);
  p.sel_weight = reinterpret_cast<const float*>(ws + L.sel_weight);
  p.tile_counts = reinterpret_cast<const int32_t*>(ws + L.tile_counts);
  p.groups = e.groups;
  p.seg_off = reinterpret_cast<int32_t*>(ws + L.seg_off);
  p.counts = reinterpret_cast<int32_t*>(ws + L.counts);
  p.work1 = reinterpret_cast<int32_t*>(ws + L.work1);
  p.work2 = reinterpret_cast<int32_t*>(ws + L.work2);
  p.h_off = reinterpret_cast<int64_t*>(ws + L.h_off);
  p.slot2tok = reinterpret_cast<int32_t*>(ws + L.slot2tok);
  p.tok2slot = reinterpret_cast<int32_t*>(ws + L.tok2slot);
  p.slot_w = reinterpret_cast<float*>(ws + L.slot_w);
  p.counts_out = counts_out;
  p.T = T;
  p.G = e.G;
  p.n_always = e.n_always;
  p.S_dyn = e.S_dyn;
  p.n_tiles = L.n_tok_tiles;
  p.bm1 = gemm_tile(e.dtype, 1);
  p.bn1 = gemm_tile(e.dtype, 3);
  p.bm2 = gemm_tile(e.dtype, 2);
  p.bn2 = gemm_tile(e.dtype, 4);
  p.d = e.d;
  p.decode = (!use_simt_experts(e.dtype) && decode_path_ok(e, T)) ? 1 : 0;
  hipLaunchKernelGGL(place_kernel, dim3(L.n_tok_tiles), dim3(64), 0, s, p);
  return hipGetLastError();
}

// ---- combine --------------------------------------------------------------------------------
// One workgroup per token; threads stride over the d columns in vectors of VEC elements.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ y_slots, const int32_t* __restrict__ tok2slot,
                                                      const float* __restrict__ slot_w, T* __restrict__ y, int d,
                                                      int S_all) {
  const int64_t t = blockIdx.x;
  __shared__ int32_t slots[MAX_DYN + MAX_TOPK];
  __shared__ float wts[MAX_DYN + MAX_TOPK];
  if (threadIdx.x < S_all) {
    slots[threadIdx.x] = tok2slot[t * S_all + threadIdx.x];
    wts[threadIdx.x] = slot_w[t * S_all + threadIdx.x];
  }
  __syncthreads();
  for (int c = threadIdx.x * VEC; c < d; c += 256 * VEC) {
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.0f;
    for (int i = 0; i < S_all; ++i) {
      const T* src = y_slots + (int64_t)slots[i] * d + c;
      const float w = wts[i];
      if (VEC == 1) {
        acc[0] = fmaf(w, Elem<T>::ld(src), acc[0]);
      } else {
        T tmp[VEC];
        *reinterpret_cast<uint4*>(tmp) = *reinterpret_cast<const uint4*>(src);
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = fmaf(w, Elem<T>::ld(&tmp[v]), acc[v]);
      }
    }
    if (VEC == 1) {
      Elem<T>::st(y + t * d + c, acc[0]);
    } else {
      T out[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) Elem<T>::st(&out[v], acc[v]);
      *reinterpret_cast<uint4*>(y + t * d + c) = *reinterpret_cast<uint4*>(out);
    }
  }
}

hipError_t launch_combine(const Engine& e, int64_t T, char* ws, const WsLayout& L, void* y, hipStream_t s) {
  if (T == 0 || e.S_all() == 1) return hipSuccess;      // a single slot per token is written straight to y
  const int32_t* tok2slot = reinterpret_cast<const int32_t*>(ws + L.tok2slot);
  const float* slot_w = reinterpret_cast<const float*>(ws + L.slot_w);
  dim3 grid((unsigned)T), block(256);
  if (e.dtype == 1) {
    const bf16_t* ys = reinterpret_cast<const bf16_t*>(ws + L.y_slots);
    if (e.d % 8 == 0)
      hipLaunchKernelGGL((combine_kernel<bf16_t, 8>), grid, block, 0, s, ys, tok2slot, slot_w,
                         static_cast<bf16_t*>(y), e.d, e.S_all());
    else
      hipLaunchKernelGGL((combine_kernel<bf16_t, 1>), grid, block, 0, s, ys, tok2slot, slot_w,
                         static_cast<bf16_t*>(y), e.d, e.S_all());
  } else {
    const float* ys = reinterpret_cast<const float*>(ws + L.y_slots);
    if (e.d % 4 == 0)
      hipLaunchKernelGGL((combine_kernel<float, 4>), grid, block, 0, s, ys, tok2slot, slot_w,
                         static_cast<float*>(y), e.d, e.S_all());
    else
      hipLaunchKernelGGL((combine_kernel<float, 1>), grid, block, 0, s, ys, tok2slot, slot_w,
                         static_cast<float*>(y), e.d, e.S_all());
  }
  return hipGetLastError();
}

}  // namespace cmoe
