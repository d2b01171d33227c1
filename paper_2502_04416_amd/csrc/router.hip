// Router scoring (Eq. 8), wavefront-level top-N_k selection and the gate of Eq. 9, for flat layers
// and for the two-level hierarchy of Sec. 4.4.  Two scoring kernels feed the same selection code:
//   router_simt_kernel  one token per workgroup, fp32 FMA dot products (fp32 layers, decode batches)
//   router_mfma_kernel  a 64-token tile per workgroup, bf16 MFMA with the K range split over the
//                       four waves (prefill batches); also emits the tile's per-group histogram
#include "cmoe_internal.h"
#include "device_utils.h"

namespace cmoe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

struct RouteIO {
  int32_t* sel_group;     // [T][S_dyn]
  float* sel_weight;      // [T][S_dyn]
  int32_t* topk_out;      // flat: [T][N_k]; hierarchy: [T][outer_top_k][N_k]; may be null
  int32_t* outer_out;     // [T][outer_top_k] or null
  float* scores_out;      // [T][n_scored] or null
  const float* gate_u;    // [n_scored] or null
  const float* gate_b;    // [n_scored] or null
  const float* lin_off;   // [n_lin] or null
  int32_t S_dyn;
};

// Top-N_k among the routed experts held by lanes [lo, lo + n) (one lane per expert), Eq. 9:
// key = s (binary gate) or Softmax(s) + b; gate = 1 + Softmax(s) * u.  Emits N_k (group, weight)
// entries in descending key order, ties to the lowest expert id.  Executed by a full wave.
__device__ __forceinline__ void select_routed(const RouterDev& r, const RouteIO& io, float skey, int lo, int n,
                                              float scale, int group_base, int64_t t, int& n_entries,
                                              int32_t* topk_ptr, int32_t* hist) {
  const int lane = threadIdx.x & 63;
  const bool in_range = lane >= lo && lane < lo + n;
  float key = skey, sp = 0.0f;
  if (r.use_gate) {
    const float mx = wave_max(in_range ? skey : -INFINITY);
    const float ex = in_range ? expf(skey - mx) : 0.0f;
    const float sum = wave_sum(ex);
    sp = ex / sum;
    key = sp + ((io.gate_b && in_range) ? io.gate_b[lane] : 0.0f);
  }
  bool active = in_range;
  for (int k = 0; k < r.top_k; ++k) {
    const int w = wave_argmax(key, active);          // uniform
    float gate = 1.0f;
    if (r.use_gate && io.gate_u) gate = 1.0f + __shfl(sp, w, 64) * io.gate_u[w];
    if (lane == 0) {
      const int g = group_base + (w - lo);
      io.sel_group[t * io.S_dyn + n_entries] = g;
      io.sel_weight[t * io.S_dyn + n_entries] = scale * gate;
      if (topk_ptr) topk_ptr[k] = w - lo;
      if (hist) atomicAdd(&hist[g], 1);
    }
    ++n_entries;
    if (lane == w) active = false;
  }
}

// Route one token from its pre-activations `pre` (LDS: n_sw_rows SwiGLU rows in blocks of IL gate /
// IL up rows, then n_lin_rows linear logits).  Executed by a full wave; all control flow is uniform.
__device__ __forceinline__ void route_token(const RouterDev& r, const RouteIO& io, const float* pre, int64_t t,
                                            int32_t* hist) {
  const int lane = threadIdx.x & 63;
  float s = 0.0f;
  if (lane < r.n_scored) {
    const int blk = lane / IL, c = lane % IL;
    const float g = pre[blk * 2 * IL + c], u = pre[blk * 2 * IL + IL + c];
    s = silu_f32(g) * u;                                                     // Eq. 8
    if (io.scores_out) io.scores_out[t * r.n_scored + lane] = s;
  }
  const float skey = r.score_abs ? fabsf(s) : s;
  int n_entries = 0;
  if (r.outer_top_k == 0) {
    select_routed(r, io, skey, 0, r.n_scored, 1.0f, r.n_always, t, n_entries,
                  io.topk_out ? io.topk_out + t * r.top_k : nullptr, hist);
    return;
  }
  // two-level: outer linear logits -> top outer_top_k -> softmax over the selected logits
  float logit = -INFINITY;
  bool active = lane < r.n_lin;
  if (active) logit = pre[r.n_sw_rows + lane] + (io.lin_off ? io.lin_off[lane] : 0.0f);
  int oe[MAX_TOPK];
  float ol[MAX_TOPK];
  for (int i = 0; i < r.outer_top_k; ++i) {
    const int w = wave_argmax(logit, active);
    oe[i] = w;
    ol[i] = __shfl(logit, w, 64);
    if (lane == w) active = false;
  }
  float den = 0.0f;
  for (int i = 0; i < r.outer_top_k; ++i) den += expf(ol[i] - ol[0]);
  for (int i = 0; i < r.outer_top_k; ++i) {
    const int e = oe[i];
    const float w_e = expf(ol[i] - ol[0]) / den;
    const int gbase = e * r.groups_per_outer;
    if (lane == 0 && io.outer_out) io.outer_out[t * r.outer_top_k + i] = e;
    if (r.sub_has_shared) {
      if (lane == 0) {
        io.sel_group[t * io.S_dyn + n_entries] = gbase;
        io.sel_weight[t * io.S_dyn + n_entries] = w_e;
        if (hist) atomicAdd(&hist[gbase], 1);
      }
      ++n_entries;
    }
    if (r.top_k > 0)
      select_routed(r, io, skey, e * r.n_r_sub, r.n_r_sub, w_e, gbase + r.sub_has_shared, t, n_entries,
                    io.topk_out ? io.topk_out + (t * r.outer_top_k + i) * r.top_k : nullptr, hist);
  }
}

// Is router row `rr` one that some scored expert (or linear logit) uses?
__device__ __forceinline__ bool router_row_used(const RouterDev& r, int rr) {
  if (rr < r.n_sw_rows) return (rr / (2 * IL)) * IL + (rr % IL) < r.n_scored;
  return rr - r.n_sw_rows < r.n_lin;
}

// ---- one token per workgroup ---------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void router_simt_kernel(RouterDev r, RouteIO io, const T* __restrict__ x,
                                                          const T* __restrict__ wr, int d) {
  extern __shared__ float smem[];
  float* xs = smem;                      // [d]
  float* pre = smem + d;                 // [n_sw_rows + n_lin_rows]
  const int64_t t = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < d; i += 256) xs[i] = Elem<T>::ld(x + t * d + i);
  const int n_rows = r.n_sw_rows + r.n_lin_rows;
  for (int i = tid; i < n_rows; i += 256) pre[i] = 0.0f;
  __syncthreads();
  for (int rr = wave; rr < n_rows; rr += 4) {
    if (!router_row_used(r, rr)) continue;
    const T* w = wr + (int64_t)rr * d;
    float acc = 0.0f;
    for (int i = lane; i < d; i += 64) acc = fmaf(xs[i], Elem<T>::ld(w + i), acc);
    acc = wave_sum(acc);
    if (lane == 0) pre[rr] = acc;
  }
  __syncthreads();
  if (wave == 0) route_token(r, io, pre, t, nullptr);
}

// ---- 64-token tile per workgroup, bf16 MFMA -------------------------------------------------
// C[64 tokens][n_rows] = X_tile [64][d] * Wr[n_rows][d]^T.  Each of the four waves takes every fourth
// 64-wide K chunk and multiplies straight out of global memory (no operand is shared between waves),
// then the four partial sums are added in a fixed order through LDS.  NT = n_rows / 32 <= 5.
template <int NT>
__global__ __launch_bounds__(256) void router_mfma_kernel(RouterDev r, RouteIO io, const bf16_t* __restrict__ x,
                                                          const bf16_t* __restrict__ wr, int d, int64_t T,
                                                          int32_t* __restrict__ tile_counts, int G) {
  __shared__ float pre[TOK_TILE][NT * 32 + 1];
  __shared__ int32_t hist[MAX_GROUPS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t t0 = (int64_t)blockIdx.x * TOK_TILE;
  const int l32 = lane & 31, lh = lane >> 5;
  floatx16_t acc[2][NT];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < NT; ++ni)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.0f;
  const bf16_t* arow[2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
    int64_t t = t0 + mi * 32 + l32;
    if (t >= T) t = T - 1;                                   // duplicate the last token; never stored
    arow[mi] = x + t * d + lh * 8;
  }
  const bf16_t* brow = wr + (int64_t)l32 * d + lh * 8;
  const int n_chunks = d / 64;                               // host guarantees d % 64 == 0
  for (int kc = wave; kc < n_chunks; kc += 4) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int k = kc * 64 + ks * 16;
      bf16x8_t a[2], b[NT];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) a[mi] = *reinterpret_cast<const bf16x8_t*>(arow[mi] + k);
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) b[ni] = *reinterpret_cast<const bf16x8_t*>(brow + (int64_t)ni * 32 * d + k);
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < NT; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
    }
  }
  // fixed-order reduction of the four K partials: wave 0 stores, waves 1..3 add in turn
  for (int wsel = 0; wsel < 4; ++wsel) {
    if (wave == wsel) {
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < NT; ++ni)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int row = mi * 32 + (i / 4) * 8 + lh * 4 + (i % 4);
            const int col = ni * 32 + l32;
            if (wsel == 0) pre[row][col] = acc[mi][ni][i];
            else pre[row][col] += acc[mi][ni][i];
          }
    }
    __syncthreads();
  }
  for (int i = tid; i < MAX_GROUPS; i += 256) hist[i] = 0;
  __syncthreads();
  for (int i = wave; i < TOK_TILE; i += 4) {
    const int64_t t = t0 + i;
    if (t < T) route_token(r, io, &pre[i][0], t, hist);
  }
  __syncthreads();
  for (int g = tid; g < G; g += 256) tile_counts[(int64_t)blockIdx.x * G + g] = hist[g];
}

// Per-tile histogram of the routed entries (used when the scoring kernel did not produce one).
__global__ __launch_bounds__(64) void tile_count_kernel(const int32_t* __restrict__ sel_group, int64_t T, int S_dyn,
                                                        int G, int32_t* __restrict__ tile_counts) {
  __shared__ int32_t hist[MAX_GROUPS];
  const int lane = threadIdx.x;
  for (int i = lane; i < MAX_GROUPS; i += 64) hist[i] = 0;
  __syncthreads();
  const int64_t t = (int64_t)blockIdx.x * TOK_TILE + lane;
  if (t < T)
    for (int i = 0; i < S_dyn; ++i) atomicAdd(&hist[sel_group[t * S_dyn + i]], 1);
  __syncthreads();
  for (int g = lane; g < G; g += 64) tile_counts[(int64_t)blockIdx.x * G + g] = hist[g];
}

hipError_t launch_router(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L,
                         int32_t* topk_out, int32_t* outer_out, float* scores_out, hipStream_t s) {
  if (e.S_dyn == 0 || T == 0) return hipSuccess;
  RouteIO io;
  io.sel_group = reinterpret_cast<int32_t*>(ws + L.sel_group);
  io.sel_weight = reinterpret_cast<float*>(ws + L.sel_weight);
  io.topk_out = topk_out;
  io.outer_out = outer_out;
  io.scores_out = scores_out;
  io.gate_u = e.gate_u;
  io.gate_b = e.gate_b;
  io.lin_off = e.lin_off;
  io.S_dyn = e.S_dyn;
  int32_t* tile_counts = reinterpret_cast<int32_t*>(ws + L.tile_counts);
  const int n_rows = e.r.n_sw_rows + e.r.n_lin_rows;
  const bool mfma = e.dtype == 1 && T >= 64 && e.d % 64 == 0 && n_rows % 32 == 0 && n_rows / 32 <= 5;
  if (mfma) {
    dim3 grid(L.n_tok_tiles), block(256);
    const bf16_t* xx = static_cast<const bf16_t*>(x);
    const bf16_t* ww = static_cast<const bf16_t*>(e.wr);
    switch (n_rows / 32) {
      case 1: hipLaunchKernelGGL(router_mfma_kernel<1>, grid, block, 0, s, e.r, io, xx, ww, e.d, T, tile_counts, e.G); break;
      case 2: hipLaunchKernelGGL(router_mfma_kernel<2>, grid, block, 0, s, e.r, io, xx, ww, e.d, T, tile_counts, e.G); break;
      case 3: hipLaunchKernelGGL(router_mfma_kernel<3>, grid, block, 0, s, e.r, io, xx, ww, e.d, T, tile_counts, e.G); break;
      case 4: hipLaunchKernelGGL(router_mfma_kernel<4>, grid, block, 0, s, e.r, io, xx, ww, e.d, T, tile_counts, e.G); break;
      default: hipLaunchKernelGGL(router_mfma_kernel<5>, grid, block, 0, s, e.r, io, xx, ww, e.d, T, tile_counts, e.G); break;
    }
    return hipGetLastError();
  }
  const size_t smem = sizeof(float) * (size_t)(e.d + n_rows);
  if (e.dtype == 1)
    hipLaunchKernelGGL(router_simt_kernel<bf16_t>, dim3((unsigned)T), dim3(256), smem, s, e.r, io,
                       static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(e.wr), e.d);
  else
    hipLaunchKernelGGL(router_simt_kernel<float>, dim3((unsigned)T), dim3(256), smem, s, e.r, io,
                       static_cast<const float*>(x), static_cast<const float*>(e.wr), e.d);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(tile_count_kernel, dim3(L.n_tok_tiles), dim3(64), 0, s, io.sel_group, T, e.S_dyn, e.G,
                     tile_counts);
  return hipGetLastError();
}

}  // namespace cmoe
