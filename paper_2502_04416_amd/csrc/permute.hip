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
#include "decode_device.h"
#include "device_utils.h"
#include "place_device.h"

namespace cmoe {

__global__ __launch_bounds__(64) void place_kernel(PlaceArgs p) {
  const LaneWidths lw = load_lane_widths(p, threadIdx.x);
  place_tile(p, blockIdx.x, p.tile_counts, threadIdx.x, p.sel_group, p.sel_weight, lw);
}

PlaceArgs make_place_args(const Engine& e, int64_t T, char* ws, const WsLayout& L, int32_t* counts_out) {
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
  p.w_by_slot = reinterpret_cast<float*>(ws + L.w_by_slot);
  p.counts_out = counts_out;
  p.T = T;
  p.G = e.G;
  p.n_always = e.n_always;
  p.S_dyn = e.S_dyn;
  p.n_tiles = L.n_tok_tiles;
  p.bm1 = gemm_tile(e, T, 1);
  p.bn1 = gemm_tile(e, T, 3);
  p.bm2 = gemm_tile(e, T, 2);
  p.bn2 = gemm_tile(e, T, 4);
  p.d = e.d;
  p.dyn1 = gemm_tile(e, T, 5);
  p.dyn2 = gemm_tile(e, T, 6);
  p.decode = (!use_simt_experts(e.dtype) && decode_path_ok(e, T)) ? 1 : 0;
  p.skip_always = L.skip_always;
  p.dec_unit1 = p.decode ? decode_unit_neurons(e, T) : 16;
  return p;
}

hipError_t launch_permute(const Engine& e, int64_t T, char* ws, const WsLayout& L, int32_t* counts_out,
                          hipStream_t s) {
  if (T == 0) return hipSuccess;
  const PlaceArgs p = make_place_args(e, T, ws, L, counts_out);
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
  if (T == 0 || e.direct_output()) return hipSuccess;   // the down contraction has written y itself
  if (decode_fuses_combine(e, T)) return hipSuccess;    // the decode down kernel has already summed the slots
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
