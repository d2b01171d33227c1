// Router scoring (Eq. 8), wavefront-level top-N_k selection and the gate of Eq. 9, for flat layers
// and for the two-level hierarchy of Sec. 4.4.  Two scoring kernels feed the same selection code:
//   router_simt_kernel  one token per workgroup, fp32 FMA dot products (fp32 layers, decode batches)
//   router_gemm_kernel  bf16 MFMA partial products over (32-token tile, K slice) workgroups, followed by
//                       route_tile_kernel, which sums the slices in order, selects, and emits each
//                       64-token tile's per-group histogram (prefill batches)
#include <cstdlib>
#include "cmoe_internal.h"
#include "decode_device.h"
#include "device_utils.h"
#include "place_device.h"

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
  int oe[MAX_OUTER_TOPK];
  float ol[MAX_OUTER_TOPK];
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

// ---- team-per-token routing (tiles of tokens) -------------------------------------------------------
// The cross-lane arg-max above costs a chain of dependent lane exchanges per token, which is fine for one
// token per workgroup but slow when a wave has to route many tokens in turn.  Here four consecutive lanes
// (a team) route one token: lane q of the team keeps the scores of experts q, q+4, q+8, ... of the
// token's row in registers (at most 16), finds its best candidate with straight-line compares, and two
// lane exchanges pick the team's winner.  Same semantics: descending key, ties to the lowest expert id.
constexpr int TEAM = 4;
constexpr int TEAM_SLOTS = MAX_SCORED / TEAM;

struct TeamSel {
  int n;                   // entries written so far
};

// Gate parameters (Eq. 9) of the experts a team lane looks after, experts lo + q + 4u: requested in one go,
// as early as the caller knows `lo`, so that one memory latency covers them all (a load of u_j for each
// winner inside the selection rounds would add a dependent round trip per round).
struct GateRegs { float u[TEAM_SLOTS], b[TEAM_SLOTS]; };
__device__ __forceinline__ GateRegs load_gate_regs(const RouterDev& r, const RouteIO& io, int lo, int n, int q) {
  GateRegs gr;
#pragma unroll
  for (int k = 0; k < TEAM_SLOTS; ++k) {
    if (k * TEAM >= n) break;               // uniform: slots past the last expert are never read
    const int j = q + TEAM * k;
    const bool ok = r.use_gate && j < n;
    gr.u[k] = (ok && io.gate_u) ? io.gate_u[lo + j] : 1.0f;
    gr.b[k] = (ok && io.gate_b) ? io.gate_b[lo + j] : 0.0f;
  }
  return gr;
}

__device__ __forceinline__ void team_select_routed(const RouterDev& r, const RouteIO& io, const float* sc, int lo,
                                                   int n, float scale, int group_base, int64_t t, TeamSel& st,
                                                   int32_t* topk_ptr, int32_t* hist, int q, const GateRegs& gr) {
  // slots in use: the same for every lane, so each unrolled loop leaves at the first unused slot through a
  // scalar branch (a wave pays for every predicated vector instruction, and n is often a quarter of the cap)
  const int n_used = (n + TEAM - 1) / TEAM;
  float key[TEAM_SLOTS], sp[TEAM_SLOTS];
  float mx = -INFINITY;
#pragma unroll
  for (int u = 0; u < TEAM_SLOTS; ++u) {
    if (u >= n_used) break;
    const int j = q + TEAM * u;
    const float s = j < n ? (r.score_abs ? fabsf(sc[lo + j]) : sc[lo + j]) : -INFINITY;
    key[u] = s;
    sp[u] = 0.0f;
    mx = fmaxf(mx, s);
  }
  if (r.use_gate) {
    mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
    float sum = 0.0f;
#pragma unroll
    for (int u = 0; u < TEAM_SLOTS; ++u) {
      if (u >= n_used) break;
      sp[u] = (q + TEAM * u < n) ? expf(key[u] - mx) : 0.0f;
      sum += sp[u];
    }
    sum += __shfl_xor(sum, 1, 64);
    sum += __shfl_xor(sum, 2, 64);
#pragma unroll
    for (int u = 0; u < TEAM_SLOTS; ++u) {
      if (u >= n_used) break;
      const int j = q + TEAM * u;
      sp[u] = sp[u] / sum;
      key[u] = j < n ? sp[u] + gr.b[u] : -INFINITY;
    }
  }
  uint32_t taken = 0u;
  for (int k = 0; k < r.top_k; ++k) {
    float best = -INFINITY, best_sp = 0.0f, best_u = 1.0f;
    int bj = 0x7fffffff;
#pragma unroll
    for (int u = 0; u < TEAM_SLOTS; ++u) {
      if (u >= n_used) break;
      const int j = q + TEAM * u;
      const bool cand = j < n && ((taken >> u) & 1u) == 0u;
      if (cand && (bj == 0x7fffffff || key[u] > best)) {
        best = key[u];
        best_sp = sp[u];
        best_u = gr.u[u];
        bj = j;
      }
    }
#pragma unroll
    for (int o = 1; o < TEAM; o <<= 1) {
      const float ob = __shfl_xor(best, o, 64), osp = __shfl_xor(best_sp, o, 64), ou = __shfl_xor(best_u, o, 64);
      const int oj = __shfl_xor(bj, o, 64);
      const bool take = oj != 0x7fffffff && (bj == 0x7fffffff || ob > best || (ob == best && oj < bj));
      best = take ? ob : best;
      best_sp = take ? osp : best_sp;
      best_u = take ? ou : best_u;
      bj = take ? oj : bj;
    }
    if ((bj & (TEAM - 1)) == q) taken |= 1u << (bj / TEAM);
    if (q == 0) {
      float gate = 1.0f;
      if (r.use_gate && io.gate_u) gate = 1.0f + best_sp * best_u;
      const int g = group_base + bj;
      io.sel_group[t * io.S_dyn + st.n] = g;
      io.sel_weight[t * io.S_dyn + st.n] = scale * gate;
      if (topk_ptr) topk_ptr[k] = bj;
      atomicAdd(&hist[g], 1);
    }
    ++st.n;
  }
}

// Selection for one token by one team: `sc` holds the token's n_scored scores (Eq. 8), `lin` its linear
// outer logits (hierarchy only; every lane of the team evaluates the few outer logits itself).
// `flat_gr`: gate parameters of a flat layer's experts, which the caller requested before it had the scores
// (ignored for a hierarchy, whose expert range depends on the outer selection).
__device__ __forceinline__ void route_select_team(const RouterDev& r, const RouteIO& io, const float* sc,
                                                  const float* lin, int64_t t, int32_t* hist, int q,
                                                  const GateRegs& flat_gr) {
  TeamSel st{0};
  if (r.outer_top_k == 0) {
    team_select_routed(r, io, sc, 0, r.n_scored, 1.0f, r.n_always, t, st,
                       io.topk_out ? io.topk_out + t * r.top_k : nullptr, hist, q, flat_gr);
    return;
  }
  int oe[MAX_OUTER_TOPK];
  float ol[MAX_OUTER_TOPK];
  uint32_t taken = 0u;
  for (int i = 0; i < r.outer_top_k; ++i) {
    float best = -INFINITY;
    int be = -1;
    for (int e = 0; e < r.n_lin; ++e) {
      const float l = lin[e] + (io.lin_off ? io.lin_off[e] : 0.0f);
      if (((taken >> e) & 1u) == 0u && (be < 0 || l > best)) {
        best = l;
        be = e;
      }
    }
    taken |= 1u << be;
    oe[i] = be;
    ol[i] = best;
  }
  float den = 0.0f;
  for (int i = 0; i < r.outer_top_k; ++i) den += expf(ol[i] - ol[0]);
  for (int i = 0; i < r.outer_top_k; ++i) {
    const int e = oe[i];
    const float w_e = expf(ol[i] - ol[0]) / den;
    const int gbase = e * r.groups_per_outer;
    if (q == 0 && io.outer_out) io.outer_out[t * r.outer_top_k + i] = e;
    if (r.sub_has_shared) {
      if (q == 0) {
        io.sel_group[t * io.S_dyn + st.n] = gbase;
        io.sel_weight[t * io.S_dyn + st.n] = w_e;
        atomicAdd(&hist[gbase], 1);
      }
      ++st.n;
    }
    if (r.top_k > 0) {
      const GateRegs gr = load_gate_regs(r, io, e * r.n_r_sub, r.n_r_sub, q);
      team_select_routed(r, io, sc, e * r.n_r_sub, r.n_r_sub, w_e, gbase + r.sub_has_shared, t, st,
                         io.topk_out ? io.topk_out + (t * r.outer_top_k + i) * r.top_k : nullptr, hist, q, gr);
    }
  }
}

// Scores of a tile of tokens, all threads of the workgroup in parallel (the exponentials are the
// expensive part of routing): sc[tok][j] = Swish(gate_j) * up_j from pre[tok][...] (Eq. 8).
__device__ __forceinline__ void score_tile(const RouterDev& r, const RouteIO& io, const float* pre, int ld_pre,
                                           float* sc, int ld_sc, int n_tok, int64_t t0, int tid, int n_threads) {
  for (int idx = tid; idx < n_tok * r.n_scored; idx += n_threads) {
    const int tok = idx / r.n_scored, j = idx - tok * r.n_scored;
    const int blk = j / IL, c = j % IL;
    const float g = pre[tok * ld_pre + blk * 2 * IL + c], u = pre[tok * ld_pre + blk * 2 * IL + IL + c];
    const float s = silu_f32(g) * u;
    sc[tok * ld_sc + j] = s;
    if (io.scores_out) io.scores_out[(t0 + tok) * r.n_scored + j] = s;
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

// ---- prefill scoring: bf16 MFMA, split over tokens and over K ----------------------------------
// P[ks][t][row] = X[t][K slice ks] * Wr[row][K slice ks]^T for a 32-token tile.  The grid is
// (token tiles, K slices) so that even a 2048-token batch fills the chip; inside a workgroup each of
// the four waves takes every fourth 64-wide chunk of the slice and multiplies straight out of global
// memory, then the four partial sums are added in a fixed order through LDS.  NT = n_rows / 32 <= 5.
constexpr int RT_TOK = 32;

template <int NT>
__global__ __launch_bounds__(256) void router_gemm_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wr,
                                                          int d, int64_t T, int k_slice, float* __restrict__ partial) {
  __shared__ float red[RT_TOK][NT * 32 + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t t0 = (int64_t)blockIdx.x * RT_TOK;
  const int ks = blockIdx.y;
  const int l32 = lane & 31, lh = lane >> 5;
  floatx16_t acc[NT];
#pragma unroll
  for (int ni = 0; ni < NT; ++ni)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[ni][i] = 0.0f;
  int64_t t = t0 + l32;
  if (t >= T) t = T - 1;                                     // duplicate the last token; never stored
  const bf16_t* arow = x + t * d + lh * 8;
  const bf16_t* brow = wr + (int64_t)l32 * d + lh * 8;
  const int k_begin = ks * k_slice;
  const int k_end = (k_begin + k_slice < d) ? k_begin + k_slice : d;     // host guarantees multiples of 64
  // software pipeline over this wave's 64-wide chunks: the loads of the next chunk are issued before
  // the MFMAs of the current one, so a wave always has a chunk of loads in flight
  bf16x8_t a0[4], a1[4], b0[NT][4], b1[NT][4];
  auto load_chunk = [&](int kc, bf16x8_t (&a)[4], bf16x8_t (&b)[NT][4]) {
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      a[s4] = *reinterpret_cast<const bf16x8_t*>(arow + kc + s4 * 16);
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) b[ni][s4] = *reinterpret_cast<const bf16x8_t*>(brow + (int64_t)ni * 32 * d + kc + s4 * 16);
    }
  };
  auto mma_chunk = [&](bf16x8_t (&a)[4], bf16x8_t (&b)[NT][4]) {
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) acc[ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s4], b[ni][s4], acc[ni], 0, 0, 0);
  };
  int kc = k_begin + wave * 64;
  if (kc < k_end) load_chunk(kc, a0, b0);
  while (kc < k_end) {
    if (kc + 256 < k_end) load_chunk(kc + 256, a1, b1);
    mma_chunk(a0, b0);
    kc += 256;
    if (kc >= k_end) break;
    if (kc + 256 < k_end) load_chunk(kc + 256, a0, b0);
    mma_chunk(a1, b1);
    kc += 256;
  }
  for (int wsel = 0; wsel < 4; ++wsel) {
    if (wave == wsel) {
#pragma unroll
      for (int ni = 0; ni < NT; ++ni)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int row = (i / 4) * 8 + lh * 4 + (i % 4);
          const int col = ni * 32 + l32;
          if (wsel == 0) red[row][col] = acc[ni][i];
          else red[row][col] += acc[ni][i];
        }
    }
    __syncthreads();
  }
  const int n_rows = NT * 32;
  for (int i = tid; i < RT_TOK * n_rows; i += 256) {
    const int row = i / n_rows, col = i - row * n_rows;
    if (t0 + row < T) partial[((int64_t)ks * T + t0 + row) * n_rows + col] = red[row][col];
  }
}

// Adds the K-slice partials [slice][T][n_rows] of tokens t0 .. t0+rows-1 in slice order into pre[row][ld]
// (LDS; rows past T become zero).  n_rows is a multiple of 4: float4 loads, all slices of up to four vectors
// per thread (sixteen loads) in flight together.  Called by all 256 threads of the workgroup.
__device__ __forceinline__ void sum_partials(const float* __restrict__ partial, int n_slices, int64_t T, int64_t t0,
                                             int rows, int n_rows, float* pre, int ld, int tid) {
  const int vec_per_row = n_rows >> 2;
  const int n_vec = rows * vec_per_row;
  for (int i0 = tid; i0 < n_vec; i0 += 4 * 256) {
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int ks0 = 0; ks0 < n_slices; ks0 += 4) {
      float4 ld4[4][4];                      // [slice][vector]
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = i0 + u * 256;
          const int row = i / vec_per_row, cv = i - row * vec_per_row;
          ld4[q][u] = make_float4(0.f, 0.f, 0.f, 0.f);
          if (ks0 + q < n_slices && i < n_vec && t0 + row < T)
            ld4[q][u] = *reinterpret_cast<const float4*>(partial + ((int64_t)(ks0 + q) * T + t0 + row) * n_rows + cv * 4);
        }
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          v[u].x += ld4[q][u].x; v[u].y += ld4[q][u].y; v[u].z += ld4[q][u].z; v[u].w += ld4[q][u].w;
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * 256;
      if (i < n_vec) {
        const int row = i / vec_per_row, cv = i - row * vec_per_row;
        float* dst = pre + row * ld + cv * 4;
        dst[0] = v[u].x; dst[1] = v[u].y; dst[2] = v[u].z; dst[3] = v[u].w;
      }
    }
  }
}

// Sum the K-slice partials in slice order, then score, select and histogram a 64-token tile: the
// 256 threads load and add the partials, then route the tile's 64 tokens in teams of four lanes.
__global__ __launch_bounds__(256) void route_tile_kernel(RouterDev r, RouteIO io, const float* __restrict__ partial,
                                                         int n_slices, int64_t T, int32_t* __restrict__ tile_counts,
                                                         int G) {
  extern __shared__ float pre[];                 // [TOK_TILE][n_rows + 1], then scores [TOK_TILE][MAX_SCORED + 1]
  __shared__ int32_t hist[MAX_GROUPS];
  const int tid = threadIdx.x;
  const int n_rows = r.n_sw_rows + r.n_lin_rows;
  const int ld = n_rows + 1;
  float* sc = pre + TOK_TILE * ld;
  constexpr int LDS_SC = MAX_SCORED + 1;
  const int64_t t0 = (int64_t)blockIdx.x * TOK_TILE;
  GateRegs flat_gr;
  if (r.outer_top_k == 0) flat_gr = load_gate_regs(r, io, 0, r.n_scored, tid % TEAM);   // needed last, requested first
  sum_partials(partial, n_slices, T, t0, TOK_TILE, n_rows, pre, ld, tid);
  for (int i = tid; i < MAX_GROUPS; i += 256) hist[i] = 0;
  __syncthreads();
  const int n_tok = (T - t0 < TOK_TILE) ? (int)(T - t0) : TOK_TILE;
  score_tile(r, io, pre, ld, sc, LDS_SC, n_tok, t0, tid, 256);
  __syncthreads();
  {
    const int tok = tid / TEAM;                    // 256 threads = 64 tokens x 4 lanes
    if (tok < n_tok) route_select_team(r, io, sc + tok * LDS_SC, pre + tok * ld + r.n_sw_rows, t0 + tok, hist, tid % TEAM, flat_gr);
  }
  __syncthreads();
  for (int g = tid; g < G; g += 256) tile_counts[(int64_t)blockIdx.x * G + g] = hist[g];
}

// ---- decode front end ------------------------------------------------------------------------------
// For batches of at most one 64-token tile scoring is one launch and selection + permutation a second one.
// (Fusing all three behind a device-wide arrival counter was tried: on this multi-die part a device-scope
// release/acquire pair writes back and invalidates the whole L2, which costs far more than a launch.)
//
// decode_score_kernel: one wave per (16 router rows, eighth of K): v_mfma_f32_16x16x32_bf16 with the router rows
// as the A operand, all loads of the wave in flight at once; the eight K-slice partials of a row go to
// pre_g[slice][token][row] and are added in slice order by route_place_kernel.  Eight times as many
// workgroups as a K loop inside the workgroup would give: the router matrix (0.5 MB at d = 4096) comes
// cold from HBM, so the launch is one memory latency long instead of several.
typedef float floatx4_t __attribute__((ext_vector_type(4)));
constexpr int DEC_SLICES = 8;

template <int NTT, int KSTEPS>
__global__ __launch_bounds__(64) void decode_score_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wr,
                                                          int d, int T, int n_rows, float* __restrict__ pre_g) {
  const int lane = threadIdx.x;
  const int slice = blockIdx.y;
  const int r16 = lane & 15, kq = lane >> 4;
  const int row0 = blockIdx.x * 16;
  const int kbase = slice * (KSTEPS * 32) + kq * 8;
  const bf16_t* wrow = wr + (int64_t)(row0 + r16) * d + kbase;
  floatx4_t acc[NTT];
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[tt][i] = 0.0f;
  bf16x8_t a[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) a[ks] = *reinterpret_cast<const bf16x8_t*>(wrow + ks * 32);
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt) {
    const int col = tt * 16 + r16;
    const bool ok = col < T;
    const bf16_t* xr = x + (int64_t)(ok ? col : 0) * d + kbase;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      bf16x8_t b;
      if (ok) b = *reinterpret_cast<const bf16x8_t*>(xr + ks * 32);
      else {
#pragma unroll
        for (int i = 0; i < 8; ++i) b[i] = (__bf16)0.0f;
      }
      acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks], b, acc[tt], 0, 0, 0);
    }
  }
  // D layout: lane holds rows kq*4 .. kq*4+3 of column (token) r16
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt) {
    const int col = tt * 16 + r16;
    if (col < T) *reinterpret_cast<floatx4_t*>(pre_g + ((int64_t)slice * T + col) * n_rows + row0 + kq * 4) = acc[tt];
  }
}

// The same partials computed inside a workgroup of eight waves instead of by a launch of its own: wave w takes
// K slice w of every block of 16 router rows, with decode_score_kernel's operands and MFMA sequence (the
// router read from its copy in operand order), so the values are the same bits; they go to LDS as part[slice][token][row].  For at most 16 tokens.  The caller
// puts a barrier between this and the first read of `part`.
template <int KSTEPS>
__device__ __forceinline__ void score_slices_in_workgroup(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wr,
                                                          int d, int T, int n_rows, float* part) {
  const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int r16 = lane & 15, kq = lane >> 4;
  const int kbase = slice * (KSTEPS * 32) + kq * 8;
  const bool ok = r16 < T;
  bf16x8_t b[KSTEPS];
  const bf16_t* xr = x + (int64_t)(ok ? r16 : 0) * d + kbase;
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) {
    if (ok) b[ks] = *reinterpret_cast<const bf16x8_t*>(xr + ks * 32);
    else {
#pragma unroll
      for (int i = 0; i < 8; ++i) b[ks][i] = (__bf16)0.0f;
    }
  }
  for (int row0 = 0; row0 < n_rows; row0 += 16) {
    // wr is the copy in operand order: K step kk of row block rb is the 1 KB at ((rb * d/32 + kk) * 64 + lane) * 8
    const bf16_t* wop = wr + (((int64_t)(row0 >> 4) * (d >> 5) + slice * KSTEPS) * 64 + lane) * 8;
    bf16x8_t a[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) a[ks] = *reinterpret_cast<const bf16x8_t*>(wop + ks * 512);
    floatx4_t acc;
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks], b[ks], acc, 0, 0, 0);
    if (ok) *reinterpret_cast<floatx4_t*>(part + ((int64_t)slice * T + r16) * n_rows + row0 + kq * 4) = acc;
  }
}

// route_place_kernel: a batch that fits one 64-token tile is selected and permuted by one workgroup:
// the 256 threads add the K-slice partials of the pre-activations in slice order and route the tokens in
// teams of four lanes, then wave 0 places the tile.  Histogram and routed entries are handed over in LDS (the
// workspace copies of the entries are not written: nothing after this kernel reads them).
// The body works with the first 256 threads of the workgroup; every thread of it must call (barriers).
// `pre`: dynamic shared memory, [T][n_rows + 1] pre-activations, then scores [T][MAX_SCORED + 1].
// What a workgroup that runs gate/up units of routed group `group` learns from selecting the tile itself
// (route_place_body with `mine` set): the group's tokens in ascending order (its slots, by the placement rule),
// their number, and where the group's rows of H start (the exclusive prefix of count x padded width over the
// groups in id order, as place_tile computes it).
struct OwnSegment {
  int32_t tok[16];
  int32_t cnt;
  long long h_off;
};

__device__ __forceinline__ void route_place_body(const RouterDev& r, RouteIO io, const PlaceArgs& pl,
                                                 const float* __restrict__ partial, int n_slices, int T, float* pre,
                                                 int group = -1, OwnSegment* mine = nullptr) {
  __shared__ int32_t hist[MAX_GROUPS];
  __shared__ int32_t sel_g[TOK_TILE * MAX_DYN];
  __shared__ float sel_w[TOK_TILE * MAX_DYN];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool worker = tid < 256;
  const int n_rows = r.n_sw_rows + r.n_lin_rows;
  const int ld = n_rows + 1;
  float* sc = pre + T * ld;
  constexpr int LDS_SC = MAX_SCORED + 1;
  LaneWidths lw;
  if (wave == 0) lw = load_lane_widths(pl, lane);          // needed last, requested first
  if (mine) {                                              // (nothing of the tile's routing is written by this workgroup)
    io.topk_out = nullptr;
    io.outer_out = nullptr;
    io.scores_out = nullptr;
  }
  GateRegs flat_gr;
  if (worker) {
    if (r.outer_top_k == 0) flat_gr = load_gate_regs(r, io, 0, r.n_scored, tid % TEAM);
    sum_partials(partial, n_slices, T, 0, T, n_rows, pre, ld, tid);
    for (int i = tid; i < MAX_GROUPS; i += 256) hist[i] = 0;
  }
  __syncthreads();
  io.sel_group = sel_g;
  io.sel_weight = sel_w;
  if (T == 1) {
    // one token: wave 0 scores and selects it with one lane per expert (no team split, no barriers in between)
    if (wave == 0) {
      route_token(r, io, pre, 0, hist);
      wave_lds_sync();
      place_tile(pl, 0, hist, lane, sel_g, sel_w, lw);
    }
    return;
  }
  if (worker) score_tile(r, io, pre, ld, sc, LDS_SC, T, 0, tid, 256);
  __syncthreads();
  if (worker) {
    const int tok = tid / TEAM;                    // at most 64 tokens x 4 lanes
    if (tok < T) route_select_team(r, io, sc + tok * LDS_SC, pre + tok * ld + r.n_sw_rows, tok, hist, tid % TEAM, flat_gr);
  }
  __syncthreads();
  if (mine) {
    // T <= 16 tokens, G <= 64 groups (the caller checked): lane g holds group g's count and width, lane t token t
    if (wave == 0) {
      const int cnt = lane < pl.n_always ? T : (lane < pl.G ? hist[lane] : 0);
      const long long ah = (long long)cnt * lw.w[0];
      const long long h_incl = wave_incl_scan(ah, lane);
      if (lane == group) {
        mine->cnt = cnt;
        mine->h_off = h_incl - ah;
      }
      bool has = false;
      if (lane < T)
        for (int i = 0; i < pl.S_dyn; ++i) has = has || sel_g[lane * pl.S_dyn + i] == group;
      const unsigned long long m = __ballot(has);
      if (has) mine->tok[__popcll(m & ((1ull << lane) - 1ull))] = lane;
    }
    __syncthreads();
    return;
  }
  if (wave == 0) place_tile(pl, 0, hist, lane, sel_g, sel_w, lw);
}

__global__ __launch_bounds__(256) void route_place_kernel(RouterDev r, RouteIO io, PlaceArgs pl,
                                                          const float* __restrict__ partial, int n_slices, int T) {
  extern __shared__ float pre[];
  route_place_body(r, io, pl, partial, n_slices, T, pre);
}

// The same launch with company: workgroup 0 selects and places, the others run the gate/up units of the
// always-on (shared-expert) group, which need nothing from the router.  Selection and placement are one
// workgroup's chain of dependent steps, 8 us long at one token; the shared expert's share of the gate/up
// stream (half of the bytes at one token) is read meanwhile instead of afterwards, with no hand-off between
// workgroups and no second stream.  The gate/up work list then leaves that group out.
template <int KSTEPS>
__global__ __launch_bounds__(512) void route_place_shared_kernel(RouterDev r, RouteIO io, PlaceArgs pl,
                                                                 const float* __restrict__ partial, int n_slices, int T,
                                                                 DecArgs da) {
  extern __shared__ float pre[];
  __shared__ DecGateUpRed<1> red;
  if (blockIdx.x == 0) {
    route_place_body(r, io, pl, partial, n_slices, T, pre);
    return;
  }
  if (da.unit1 == 8) decode_gate_up_unit8<1, KSTEPS>(da, 0, (int)blockIdx.x - 1, 0, T, da.groups[0].width_pad, 0, red);
  else decode_gate_up_unit<1, KSTEPS>(da, 0, (int)blockIdx.x - 1, 0, T, da.groups[0].width_pad, 0, red);
}

// One token on a flat layer: the launch that selects and places also runs *every* gate/up unit, the routed
// ones included.  Workgroup 0 is route_place_kernel's body; workgroups 1 .. U_s run the shared group's units;
// workgroup 1 + U_s + k * U_r + j runs unit j of the k-th selected expert, which it finds by itself: its wave 0
// adds the K-slice partials of the router pre-activations in the same order as workgroup 0 does, scores them
// with the same arithmetic and runs the same top-N_k, so every workgroup arrives at the same experts with no
// hand-off between workgroups.  What it needs is 8 slices x the router rows (a few KB, the same few lines for
// all workgroups), not the router matrix.  The rows of H follow the placement rule: segments in ascending
// group id, so the expert's row of H starts after the shared group's and after the rows of the selected
// experts with smaller ids.  One launch and its gap less than scoring + (selection, shared units) + routed
// units; the separate gate/up launch is skipped.
template <int KSTEPS>
__global__ __launch_bounds__(512) void route_place_all_kernel(RouterDev r, RouteIO io, PlaceArgs pl,
                                                              const float* __restrict__ partial, int n_slices,
                                                              DecArgs da, int units_shared, int units_routed,
                                                              const bf16_t* __restrict__ wr) {
  extern __shared__ float pre[];
  __shared__ DecGateUpRed<1> red;
  __shared__ int32_t my_sel_g[MAX_DYN];
  __shared__ float my_sel_w[MAX_DYN];
  const int n_rows = r.n_sw_rows + r.n_lin_rows;
  const int b = (int)blockIdx.x - 1;
  if (b >= 0 && b < units_shared) {
    if (da.unit1 == 8) decode_gate_up_unit8<1, KSTEPS>(da, 0, b, 0, 1, da.groups[0].width_pad, 0, red);
    else decode_gate_up_unit<1, KSTEPS>(da, 0, b, 0, 1, da.groups[0].width_pad, 0, red);
    return;
  }
  if (wr) {
    // no scoring launch: every workgroup that needs the pre-activations computes the K-slice partials itself
    // (the router matrix is a few hundred KB that all of them find in L2 after the first) and keeps them in
    // LDS behind the selection's arrays
    float* part = pre + ((n_rows + 1 + MAX_SCORED + 1 + 3) & ~3);      // 16-byte aligned
    score_slices_in_workgroup<KSTEPS>(da.x, wr, da.d, 1, n_rows, part);
    __syncthreads();
    partial = part;
    n_slices = DEC_SLICES;
  }
  if (blockIdx.x == 0) {
    route_place_body(r, io, pl, partial, n_slices, 1, pre);
    return;
  }
  const int k = (b - units_shared) / units_routed, local = (b - units_shared) % units_routed;
  const int tid = threadIdx.x;
  if (tid < 64) {
    for (int row = tid; row < n_rows; row += 64) {
      float acc = 0.0f;
      for (int sl = 0; sl < n_slices; ++sl) acc += partial[(int64_t)sl * n_rows + row];     // T = 1: [slice][row]
      pre[row] = acc;
    }
    wave_lds_sync();
    RouteIO mine = io;
    mine.sel_group = my_sel_g;
    mine.sel_weight = my_sel_w;
    mine.topk_out = nullptr;
    mine.outer_out = nullptr;
    mine.scores_out = nullptr;
    route_token(r, mine, pre, 0, nullptr);
  }
  __syncthreads();
  const int g = my_sel_g[k];
  int rank = 0;
  for (int i = 0; i < r.top_k; ++i) rank += my_sel_g[i] < g ? 1 : 0;
  const int wp = da.groups[g].width_pad;
  const int64_t hoff = (r.n_always ? (int64_t)da.groups[0].width_pad : 0) + (int64_t)rank * wp;
  if (da.unit1 == 8) decode_gate_up_unit8<1, KSTEPS>(da, g, local, 0, 1, wp, hoff, red);
  else decode_gate_up_unit<1, KSTEPS>(da, g, local, 0, 1, wp, hoff, red);
}

// Two to sixteen tokens on a flat layer, the same idea: workgroup 0 selects and places the batch, the next
// workgroups run the shared group's units, and every unit of *every* routed expert has a workgroup that
// selects the whole batch by itself (the 256-thread team selection of route_place_kernel on the scorer's
// partials, 16 KB that all workgroups share in L2), learns which tokens chose its expert and where the
// expert's rows of H start, and runs its unit on them; the workgroups of experts nobody chose leave.  The
// separate gate/up launch, which could not start before selection and placement had finished in one
// workgroup, is gone.  Bit-identical to the two launches and slower than them at every batch size (the team
// selection run by hundreds of workgroups at once takes 15 us instead of the 8 us it takes one workgroup on
// an otherwise idle chip), so it is off unless the tuning switch front_tile asks for it.
template <int KSTEPS>
__global__ __launch_bounds__(512) void route_place_tile_all_kernel(RouterDev r, RouteIO io, PlaceArgs pl,
                                                                   const float* __restrict__ partial, int n_slices, int T,
                                                                   DecArgs da, int units_shared, int units_routed) {
  extern __shared__ float pre[];
  __shared__ DecGateUpRed<1> red;
  __shared__ OwnSegment own;
  const int b = (int)blockIdx.x - 1;
  if (b >= 0 && b < units_shared) {
    decode_gate_up_unit<1, KSTEPS>(da, 0, b, 0, T, da.groups[0].width_pad, 0, red);
    return;
  }
  if (blockIdx.x == 0) {
    route_place_body(r, io, pl, partial, n_slices, T, pre);
    return;
  }
  const int g = r.n_always + (b - units_shared) / units_routed, local = (b - units_shared) % units_routed;
  route_place_body(r, io, pl, partial, n_slices, T, pre, g, &own);
  const int cnt = own.cnt;
  if (cnt == 0) return;
  da.slot2tok = own.tok;                          // slot j of this group = its j-th token in ascending order
  decode_gate_up_unit<1, KSTEPS>(da, g, local, 0, cnt, da.groups[g].width_pad, own.h_off, red);
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

PlaceArgs make_place_args(const Engine& e, int64_t T, char* ws, const WsLayout& L, int32_t* counts_out);

// The MFMA scorer needs bf16 operands, K slices of 256 and whole 32-row blocks of router rows (at most five).
static bool mfma_scorer_ok(const Engine& e) {
  const int n_rows = e.r.n_sw_rows + e.r.n_lin_rows;
  return e.dtype == 1 && e.d % 256 == 0 && n_rows % 32 == 0 && n_rows / 32 <= 5;
}

// Pre-activation partials [slice][T][n_rows] of all router rows by router_gemm_kernel.
static hipError_t launch_scorer_gemm(const Engine& e, const void* x, int64_t T, float* partial, hipStream_t s,
                                     int& n_slices) {
  const int n_rows = e.r.n_sw_rows + e.r.n_lin_rows;
  // K slices: enough workgroups to fill 256 CUs, at least 256 of K per slice, at most the partial buffer's 8
  const int n_tt = (int)((T + RT_TOK - 1) / RT_TOK);
  n_slices = (512 + n_tt - 1) / n_tt;
  if (n_slices > 8) n_slices = 8;
  while (n_slices > 1 && (e.d % (n_slices * 256) != 0)) --n_slices;
  const int k_slice = e.d / n_slices;
  dim3 grid(n_tt, n_slices), block(256);
  const bf16_t* xx = static_cast<const bf16_t*>(x);
  const bf16_t* ww = static_cast<const bf16_t*>(e.wr);
  switch (n_rows / 32) {
    case 1: hipLaunchKernelGGL(router_gemm_kernel<1>, grid, block, 0, s, xx, ww, e.d, T, k_slice, partial); break;
    case 2: hipLaunchKernelGGL(router_gemm_kernel<2>, grid, block, 0, s, xx, ww, e.d, T, k_slice, partial); break;
    case 3: hipLaunchKernelGGL(router_gemm_kernel<3>, grid, block, 0, s, xx, ww, e.d, T, k_slice, partial); break;
    case 4: hipLaunchKernelGGL(router_gemm_kernel<4>, grid, block, 0, s, xx, ww, e.d, T, k_slice, partial); break;
    default: hipLaunchKernelGGL(router_gemm_kernel<5>, grid, block, 0, s, xx, ww, e.d, T, k_slice, partial); break;
  }
  return hipGetLastError();
}

// One tile of at most 64 tokens is scored in one launch and selected + placed by one workgroup in a second.
// Up to 16 tokens (one MFMA token tile) the scorer is decode_score_kernel, which beats the general one by
// 3-4 us there; from 17 tokens on it is the general scorer, whose work spreads over hundreds of workgroups
// (measured at d = 4096, 13 routed experts).  The larger batches need the tile's pre-activations and scores
// to fit the 64 KB of LDS a workgroup gets by default next to 14 KB of static arrays.
constexpr int FRONT_SCORE_MAX_T = 16;
bool decode_front_ok(const Engine& e, int64_t T) {
  const int n_rows = e.r.n_sw_rows + e.r.n_lin_rows;
  if (e.S_dyn <= 0 || T < 1 || T > TOK_TILE) return false;
  if (T <= FRONT_SCORE_MAX_T) return decode_path_ok(e, T) && n_rows % 16 == 0;
  return mfma_scorer_ok(e) && sizeof(float) * (size_t)T * (n_rows + 1 + MAX_SCORED + 1) <= 48 * 1024;
}

// Router scoring (one launch) and selection + permutation (one launch) of a decode batch.
hipError_t launch_decode_front(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L,
                               int32_t* topk_out, int32_t* outer_out, float* scores_out, int32_t* counts_out,
                               hipStream_t s) {
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
  const PlaceArgs pl = make_place_args(e, T, ws, L, counts_out);
  const int n_rows = e.r.n_sw_rows + e.r.n_lin_rows;
  float* pre_g = reinterpret_cast<float*>(ws + L.scores);
  const int Ti = (int)T;
  int n_slices = DEC_SLICES;
  hipError_t err = hipSuccess;
  // one token, every gate/up unit in the selection launch: with front_all = 2 that launch also scores
  const bool own_scores = L.gate_up_done && tuning().front_all >= 2 && e.wr_tiled != nullptr;
  if (own_scores) {
  } else if (T <= FRONT_SCORE_MAX_T) {
    dim3 grid(n_rows / 16, DEC_SLICES), block(64);
    const bf16_t* xx = static_cast<const bf16_t*>(x);
    const bf16_t* ww = static_cast<const bf16_t*>(e.wr);
    const int ksteps = e.d / 256;                 // K steps of 32 per slice: d / (8 slices * 32)
#define CMOE_SCORE(NTT, KS) hipLaunchKernelGGL((decode_score_kernel<NTT, KS>), grid, block, 0, s, xx, ww, e.d, Ti, n_rows, pre_g)
    // (measurement aid: repeat_stage = 6 issues the scoring launch twice; it overwrites its partials)
    for (int rep = tuning().repeat_stage == 6 ? 2 : 1; rep > 0; --rep)
      switch (ksteps) {
        case 16: CMOE_SCORE(1, 16); break;
        case 8: CMOE_SCORE(1, 8); break;
        case 4: CMOE_SCORE(1, 4); break;
        default: CMOE_SCORE(1, 2); break;
      }
#undef CMOE_SCORE
    err = hipGetLastError();
  } else {
    err = launch_scorer_gemm(e, x, T, pre_g, s, n_slices);
  }
  if (err != hipSuccess) return err;
  if (tuning().skip_stage == 6) return hipSuccess;        // measurement aid: the scoring launch only
  size_t smem = sizeof(float) * (size_t)T * (n_rows + 1 + MAX_SCORED + 1);
  if (L.gate_up_done && T > 1) {
    // (the caller set this from decode_front_runs_all: 2-16 tokens, flat layer of at most 64 groups, routed
    // groups of one width, 16-neuron units)
    DecArgs da = make_dec_args(e, x, T, ws, L, nullptr);
    da.slot2tok = nullptr;                        // group 0's slots are the tokens in order
    da.work = nullptr;
    const int us = e.n_always ? e.width_pad_host[0] / 16 : 0;
    const int ur = e.width_pad_host[e.n_always] / 16;
    const dim3 grid(1 + us + (e.G - e.n_always) * ur), block(512);
    for (int rep = tuning().repeat_stage == 3 ? 2 : 1; rep > 0; --rep)       // (measurement aid, as below)
      switch (e.d / 256) {
        case 16: hipLaunchKernelGGL(route_place_tile_all_kernel<16>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, Ti, da, us, ur); break;
        case 8: hipLaunchKernelGGL(route_place_tile_all_kernel<8>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, Ti, da, us, ur); break;
        case 4: hipLaunchKernelGGL(route_place_tile_all_kernel<4>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, Ti, da, us, ur); break;
        default: hipLaunchKernelGGL(route_place_tile_all_kernel<2>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, Ti, da, us, ur); break;
      }
    return hipGetLastError();
  }
  if (L.gate_up_done) {
    // (the caller set this from decode_front_runs_all: one token, flat layer, routed groups of one width)
    DecArgs da = make_dec_args(e, x, T, ws, L, nullptr);
    da.slot2tok = nullptr;                        // one token: every slot is token 0
    da.work = nullptr;
    const int us = e.n_always ? e.width_pad_host[0] / da.unit1 : 0;
    const int ur = e.width_pad_host[e.n_always] / da.unit1;
    const dim3 grid(1 + us + e.r.top_k * ur), block(512);
    const bf16_t* wr_in = own_scores ? static_cast<const bf16_t*>(e.wr_tiled) : nullptr;
    if (own_scores) smem = sizeof(float) * (size_t)(((n_rows + 1 + MAX_SCORED + 1 + 3) & ~3) + DEC_SLICES * n_rows);
    // (measurement aid: this launch is the layer's gate/up stage, so repeat_stage = 3 issues it twice; it reads
    // only the scorer's partials, the token and the weights, and every write is a plain store of a value that
    // depends on those alone, so the second launch leaves the same bits)
    for (int rep = tuning().repeat_stage == 3 ? 2 : 1; rep > 0; --rep)
      switch (e.d / 256) {
        case 16: hipLaunchKernelGGL(route_place_all_kernel<16>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, da, us, ur, wr_in); break;
        case 8: hipLaunchKernelGGL(route_place_all_kernel<8>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, da, us, ur, wr_in); break;
        case 4: hipLaunchKernelGGL(route_place_all_kernel<4>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, da, us, ur, wr_in); break;
        default: hipLaunchKernelGGL(route_place_all_kernel<2>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, da, us, ur, wr_in); break;
      }
    return hipGetLastError();
  }
  if (L.skip_always) {
    // (the caller set this from decode_front_runs_shared: one always-on group, decode kernels, T <= 16)
    DecArgs da = make_dec_args(e, x, T, ws, L, nullptr);
    da.slot2tok = nullptr;                        // group 0's slots are the tokens in order; the map is not written yet
    da.work = nullptr;
    const dim3 grid(1 + e.width_pad_host[0] / da.unit1), block(512);
    switch (e.d / 256) {
      case 16: hipLaunchKernelGGL(route_place_shared_kernel<16>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, Ti, da); break;
      case 8: hipLaunchKernelGGL(route_place_shared_kernel<8>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, Ti, da); break;
      case 4: hipLaunchKernelGGL(route_place_shared_kernel<4>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, Ti, da); break;
      default: hipLaunchKernelGGL(route_place_shared_kernel<2>, grid, block, smem, s, e.r, io, pl, pre_g, n_slices, Ti, da); break;
    }
    return hipGetLastError();
  }
  hipLaunchKernelGGL(route_place_kernel, dim3(1), dim3(256), smem, s, e.r, io, pl, pre_g, n_slices, Ti);
  return hipGetLastError();
}

bool decode_front_runs_shared(const Engine& e, int64_t T) {
  return tuning().front_shared != 0 && T <= FRONT_SCORE_MAX_T && e.n_always == 1 && decode_front_ok(e, T) && decode_path_ok(e, T);
}

// One token (switch front_all), or two to sixteen (switch front_tile; at most 64 groups, 16-neuron units), on a
// flat routed layer whose routed groups all have one width, at most one always-on group, the decode kernels'
// model widths (tuning switch front_shared = 0 switches this off together with the shared units in the front
// end).
bool decode_front_runs_all(const Engine& e, int64_t T) {
  if (T < 1 || T > FRONT_SCORE_MAX_T || tuning().front_shared == 0) return false;
  if (T == 1 ? tuning().front_all == 0 : (tuning().front_tile == 0 || e.G > 64 || tuning().decode_split == 8)) return false;
  if (e.r.outer_top_k != 0 || e.n_always > 1 || e.G <= e.n_always || e.S_dyn != e.r.top_k) return false;
  if (!decode_front_ok(e, T) || !decode_path_ok(e, T)) return false;
  for (int g = e.n_always; g < e.G; ++g)
    if (e.width_pad_host[g] != e.width_pad_host[e.n_always]) return false;
  return true;
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
  if (mfma_scorer_ok(e)) {
    int n_slices = 1;
    float* partial = reinterpret_cast<float*>(ws + L.scores);
    hipError_t err = launch_scorer_gemm(e, x, T, partial, s, n_slices);
    if (err != hipSuccess) return err;
    const size_t smem = sizeof(float) * (size_t)TOK_TILE * (n_rows + 1 + MAX_SCORED + 1);
    hipLaunchKernelGGL(route_tile_kernel, dim3(L.n_tok_tiles), dim3(256), smem, s, e.r, io, partial, n_slices, T,
                       tile_counts, e.G);
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
