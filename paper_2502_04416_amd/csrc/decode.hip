// Expert kernels for decode batches (T <= 16 tokens, bf16; the fused down + combine kernel up to 32):
// weight streaming bound by HBM bandwidth.
//
// Every expert group with at least one token is cut into units of 16 neurons (gate/up) or 16 output
// columns (down).  The weights of a unit are the A operand of v_mfma_f32_16x16x32_bf16 and are read
// straight from global memory exactly once, 64 contiguous bytes per row and instruction; the tokens
// of the group (at most 16, gathered through slot2tok) are the B operand and stay in registers for
// the whole unit.  The reduction dimension is split over the waves of a workgroup so that a unit
// keeps many independent loads in flight; the partial sums are added in a fixed order through LDS.
// This is the per-neuron form of the FFN, F(x) = sum_i h_i w_i (Eq. 1), evaluated only for the
// neurons of the experts some token selected (Eq. 4).
#include <algorithm>
#include <cstdlib>
#include "cmoe_internal.h"
#include "decode_device.h"
#include "device_utils.h"

namespace cmoe {

// The LDS operations of one wave complete in issue order: waiting for them (and keeping the compiler from
// moving LDS accesses across) is enough to order a wave's own LDS updates.
__device__ __forceinline__ void wave_lds_sync_decode() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_wave_barrier();
}

// Which unit is this workgroup?  Returns false when past the end of the list.
__device__ __forceinline__ bool find_unit(const DecArgs& p, int units_single, int& g, int& local, int& seg0, int& cnt,
                                          int& wp, int64_t& hoff) {
  const int u = blockIdx.x;
  if (p.single) {
    if (u >= units_single) return false;
    g = 0;
    local = u;
    seg0 = 0;
    cnt = (int)p.T;
    wp = p.groups[0].width_pad;
    hoff = 0;
    return true;
  }
  if (u >= p.work[p.G]) return false;
  g = find_group(p.work, p.G, u);
  local = u - p.work[g];
  seg0 = p.seg_off[g];
  cnt = p.seg_off[g + 1] - seg0;
  wp = p.groups[g].width_pad;
  hoff = p.h_off[g];
  return true;
}

// ---- gate/up: H[slot][n] = Swish(x . wgate_n) * (x . wup_n) for 16 neurons of one group ---------------
template <int NTT, int KSTEPS>
__global__ __launch_bounds__(512) void decode_gate_up_kernel(DecArgs p) {
  __shared__ DecGateUpRed<NTT> red;
  int g, local, seg0, cnt, wp;
  int64_t hoff;
  if (!find_unit(p, p.single ? p.groups[0].width_pad / p.unit1 : 0, g, local, seg0, cnt, wp, hoff)) return;
  if (p.unit1 == 8) decode_gate_up_unit8<NTT, KSTEPS>(p, g, local, seg0, cnt, wp, hoff, red);
  else decode_gate_up_unit<NTT, KSTEPS>(p, g, local, seg0, cnt, wp, hoff, red);
}

// ---- down: Y[slot][c] = sum_n H[slot][n] * Wdown[n][c] for 16 output columns of one group --------------
// 4 waves; wave w takes the 32-wide K steps w, w+4, ...
template <int NTT>
__global__ __launch_bounds__(256) void decode_down_kernel(DecArgs p) {
  __shared__ float red[4][NTT][16][17];
  int g, local, seg0, cnt, wp;
  int64_t hoff;
  if (!find_unit(p, p.single ? p.d / 16 : 0, g, local, seg0, cnt, wp, hoff)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kq = lane >> 4;
  const int c0 = local * 16;
  const bf16_t* wrow = p.w2 + p.groups[g].w2_off +
                       (p.tiled ? tiled_offset(c0 + r16, kq * 8, wp / TILE_K) : (int64_t)(c0 + r16) * wp + kq * 8);
  const int kadv = p.tiled ? TILE_ELEMS : 32;                 // elements from one K step's operand to the next
  const bf16_t* hrow[NTT];
  bool hok[NTT];
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt) {
    const int col = tt * 16 + r16;
    hok[tt] = col < cnt;
    hrow[tt] = p.h + hoff + (int64_t)(hok[tt] ? col : 0) * wp + kq * 8;
  }
  floatx4_t acc[NTT];
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[tt][i] = 0.0f;
  const int n_steps = wp / 32;
  int ks = wave;
  // eight K steps of this wave at a time: their loads are independent and all in flight together
  for (; ks + 28 < n_steps; ks += 32) {
    bf16x8_t a[8], b[NTT][8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      a[u] = ld_frag(wrow + (ks + 4 * u) * kadv);
#pragma unroll
      for (int tt = 0; tt < NTT; ++tt) b[tt][u] = hok[tt] ? ld_frag(hrow[tt] + (ks + 4 * u) * 32) : zero_frag();
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int tt = 0; tt < NTT; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], b[tt][u], acc[tt], 0, 0, 0);
  }
  for (; ks + 12 < n_steps; ks += 16) {
    bf16x8_t a[4], b[NTT][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      a[u] = ld_frag(wrow + (ks + 4 * u) * kadv);
#pragma unroll
      for (int tt = 0; tt < NTT; ++tt) b[tt][u] = hok[tt] ? ld_frag(hrow[tt] + (ks + 4 * u) * 32) : zero_frag();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int tt = 0; tt < NTT; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], b[tt][u], acc[tt], 0, 0, 0);
  }
  for (; ks < n_steps; ks += 4) {
    const bf16x8_t a = ld_frag(wrow + ks * kadv);
#pragma unroll
    for (int tt = 0; tt < NTT; ++tt) {
      const bf16x8_t b = hok[tt] ? ld_frag(hrow[tt] + ks * 32) : zero_frag();
      acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[tt], 0, 0, 0);
    }
  }
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
    for (int i = 0; i < 4; ++i) red[wave][tt][kq * 4 + i][r16] = acc[tt][i];
  __syncthreads();
  for (int e = tid; e < NTT * 256; e += 256) {
    const int tt = e >> 8, tok = (e >> 4) & 15, cc = e & 15;       // column fastest: contiguous stores
    const int col = tt * 16 + tok;
    if (col >= cnt) continue;
    const float s = (red[0][tt][cc][tok] + red[1][tt][cc][tok]) + (red[2][tt][cc][tok] + red[3][tt][cc][tok]);
    p.y[(int64_t)(seg0 + col) * p.d + c0 + cc] = f32_to_bf16(s);
  }
}

// ---- down + combine: y[t][c] = sum over the token's slots of weight * sum_n H[slot][n] * Wdown[n][c] ---------
// One workgroup owns 16 output columns of every token, so the weighted sum over a token's experts (Eq. 4,
// Eq. 10) needs no second pass and no per-slot outputs in memory.  Its work items are (non-empty group,
// chunk of DC_CH K steps); wave w takes items w, w + 16, ... and adds its weighted partial products into
// accumulators of its own in LDS, which are summed in wave order at the end: the result does not depend on
// timing.  All loads of an item are in flight together.
constexpr int DC_CH = 8;
constexpr int DC_WAVES = 16;
template <int NTT>
__global__ __launch_bounds__(DC_WAVES * 64) void decode_down_combine_kernel(DecArgs p, const float* __restrict__ w_by_slot,
                                                                            bf16_t* __restrict__ y_out) {
  __shared__ float yacc[DC_WAVES][NTT * 16][17];
  __shared__ int32_t item0[MAX_GROUPS + 1];       // prefix of work items over groups
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kq = lane >> 4;
  const int c0 = blockIdx.x * 16;
  float* mine = &yacc[wave][0][0];
  for (int e = lane; e < NTT * 16 * 17; e += 64) mine[e] = 0.0f;
  if (wave == 0) {
    int run0 = 0;
#pragma unroll
    for (int k = 0; k < MAX_GROUPS / 64; ++k) {
      const int g = lane + 64 * k;
      int n = 0;
      if (g < p.G && p.seg_off[g + 1] > p.seg_off[g]) n = cdiv(p.groups[g].width_pad / 32, DC_CH);
      const int inc = wave_incl_scan(n, lane);
      if (g < p.G) item0[g] = run0 + inc - n;
      run0 += __shfl(inc, 63, 64);
    }
    if (lane == 0) item0[p.G] = run0;
  }
  __syncthreads();
  const int n_items = item0[p.G];
  for (int u = wave; u < n_items; u += DC_WAVES) {
    const int g = find_group(item0, p.G, u);
    const int ks0 = (u - item0[g]) * DC_CH;
    const int seg0 = p.seg_off[g], cnt = p.seg_off[g + 1] - seg0;
    const int wp = p.groups[g].width_pad;
    const int ns = min(DC_CH, wp / 32 - ks0);
    const int kadv = p.tiled ? TILE_ELEMS : 32;
    const bf16_t* wrow = p.w2 + p.groups[g].w2_off +
                         (p.tiled ? tiled_offset(c0 + r16, ks0 * 32 + kq * 8, wp / TILE_K)
                                  : (int64_t)(c0 + r16) * wp + kq * 8 + ks0 * 32);
    const bf16_t* hbase = p.h + p.h_off[g] + kq * 8 + ks0 * 32;
    bf16x8_t a[DC_CH], b[NTT][DC_CH];
    int tok[NTT];
    float wt[NTT];
#pragma unroll
    for (int s = 0; s < DC_CH; ++s) a[s] = s < ns ? ld_frag(wrow + s * kadv) : zero_frag();
#pragma unroll
    for (int tt = 0; tt < NTT; ++tt) {
      const int col = tt * 16 + r16;
      const bool ok = col < cnt;
      const bf16_t* hrow = hbase + (int64_t)(ok ? col : 0) * wp;
#pragma unroll
      for (int s = 0; s < DC_CH; ++s) b[tt][s] = (ok && s < ns) ? ld_frag(hrow + s * 32) : zero_frag();
      tok[tt] = ok ? p.slot2tok[seg0 + col] : -1;
      wt[tt] = ok ? w_by_slot[seg0 + col] : 0.0f;
    }
#pragma unroll
    for (int tt = 0; tt < NTT; ++tt) {
      floatx4_t acc;
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = 0.0f;
#pragma unroll
      for (int s = 0; s < DC_CH; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[s], b[tt][s], acc, 0, 0, 0);
      // accumulator element i: output column (lane/16)*4 + i, token of segment position lane%16
      if (tok[tt] >= 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) yacc[wave][tok[tt]][kq * 4 + i] += wt[tt] * acc[i];
      }
    }
  }
  __syncthreads();
  for (int e = tid; e < (int)p.T * 16; e += DC_WAVES * 64) {
    const int t = e >> 4, cc = e & 15;
    float s = 0.0f;
#pragma unroll
    for (int w = 0; w < DC_WAVES; ++w) s += yacc[w][t][cc];
    y_out[(int64_t)t * p.d + c0 + cc] = f32_to_bf16(s);
  }
}


// ---- neuron-level activation sparsity inside the routed experts (Sec. 5; Eq. 1 restricted to surviving neurons) ----
// A hidden activation h_n of a routed group survives iff |h_n| * scale_n >= tau, decided on the bf16 value the
// gate/up kernels stored (scale_n = 1, or the L2 norm of the neuron's row of W_down).
__device__ __forceinline__ bool neuron_survives(bf16_t v, int mode, float scale, float tau) {
  const float key = fabsf(bf16_to_f32(v)) * (mode == 2 ? scale : 1.0f);
  return key >= tau;                                          // (a NaN is dropped)
}

// Every batch but the one- and two-token ones: the dropped activations are zeroed in H after the gate/up
// contraction, so that the layer computes the same function at every batch size; one workgroup per slot row.
__global__ __launch_bounds__(256) void mask_hidden_kernel(bf16_t* __restrict__ h, const GroupDev* __restrict__ groups,
                                                          const int32_t* __restrict__ seg_off,
                                                          const int64_t* __restrict__ h_off,
                                                          const float* __restrict__ nscale, int G, int n_always, int mode,
                                                          float tau) {
  const int row = blockIdx.x;
  if (row >= seg_off[G]) return;
  const int g = find_group(seg_off, G, row);
  if (g < n_always) return;                                   // shared experts are never sparsified
  const int wp = groups[g].width_pad;
  const int64_t base = h_off[g] + (int64_t)(row - seg_off[g]) * wp;
  const int n0 = groups[g].w1_row0 / 2;
  for (int n = threadIdx.x; n < wp; n += 256)
    if (!neuron_survives(h[base + n], mode, nscale[n0 + n], tau)) h[base + n] = 0;
}

// One or two tokens: down projection + weighted sum over slots that reads only the surviving neurons' weights.
// A workgroup owns 16 output columns of both tokens.  The always-on groups go through the matrix cores as in
// decode_down_combine_kernel.  For a routed group every thread looks at one neuron: if it survives, the thread
// reads the 32 bytes of that neuron's row of the neuron-major copy of W_down that belong to the workgroup's
// columns and adds h_n * w_n (Eq. 1); the rows of dropped neurons are never touched.  The per-thread sums are
// added across the wave by exchanges in a fixed pattern, across waves in wave order: deterministic.
// Column blocks are dealt so that the four workgroups sharing a 128-byte line of a row run on one XCD.
constexpr int DS_WAVES = 16;
__global__ __launch_bounds__(DS_WAVES * 64) void decode_down_sparse_kernel(DecArgs p, const float* __restrict__ w_by_slot,
                                                                           bf16_t* __restrict__ y_out,
                                                                           const bf16_t* __restrict__ w2n,
                                                                           const float* __restrict__ nscale, int n_always,
                                                                           int mode, float tau, int cb_per_xcd) {
  __shared__ float yacc[DS_WAVES][2][16];
  __shared__ int32_t item0[MAX_GROUPS + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kq = lane >> 4;
  const int cb = (blockIdx.x & 7) * cb_per_xcd + (blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= cb_per_xcd || cb >= p.d / 16) return;
  const int c0 = cb * 16;
  if (lane < 32) yacc[wave][lane >> 4][lane & 15] = 0.0f;
  if (wave == 0) {
    int run0 = 0;
#pragma unroll
    for (int k = 0; k < MAX_GROUPS / 64; ++k) {
      const int g = lane + 64 * k;
      int n = 0;
      if (g < n_always && p.seg_off[g + 1] > p.seg_off[g]) n = cdiv(p.groups[g].width_pad / 32, DC_CH);
      const int inc = wave_incl_scan(n, lane);
      if (g < p.G) item0[g] = run0 + inc - n;
      run0 += __shfl(inc, 63, 64);
    }
    if (lane == 0) item0[p.G] = run0;
  }
  __syncthreads();
  // ---- always-on groups: 16 columns x 8 K steps per work item, matrix cores ----
  const int n_items = item0[p.G];
  for (int u = wave; u < n_items; u += DS_WAVES) {
    const int g = find_group(item0, p.G, u);
    const int ks0 = (u - item0[g]) * DC_CH;
    const int seg0 = p.seg_off[g], cnt = p.seg_off[g + 1] - seg0;
    const int wp = p.groups[g].width_pad;
    const int ns = min(DC_CH, wp / 32 - ks0);
    const int kadv = p.tiled ? TILE_ELEMS : 32;
    const bf16_t* wrow = p.w2 + p.groups[g].w2_off +
                         (p.tiled ? tiled_offset(c0 + r16, ks0 * 32 + kq * 8, wp / TILE_K)
                                  : (int64_t)(c0 + r16) * wp + kq * 8 + ks0 * 32);
    const bool ok = r16 < cnt;
    const bf16_t* hrow = p.h + p.h_off[g] + kq * 8 + ks0 * 32 + (int64_t)(ok ? r16 : 0) * wp;
    bf16x8_t a[DC_CH], b[DC_CH];
#pragma unroll
    for (int s = 0; s < DC_CH; ++s) {
      a[s] = s < ns ? ld_frag(wrow + s * kadv) : zero_frag();
      b[s] = (ok && s < ns) ? ld_frag(hrow + s * 32) : zero_frag();
    }
    const int tok = ok ? p.slot2tok[seg0 + r16] : -1;
    const float wt = ok ? w_by_slot[seg0 + r16] : 0.0f;
    floatx4_t acc;
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int s = 0; s < DC_CH; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[s], b[s], acc, 0, 0, 0);
    if (tok >= 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) yacc[wave][tok][kq * 4 + i] += wt * acc[i];
    }
  }
  // ---- routed groups: one neuron per thread, surviving rows only ----
  float a0[16], a1[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) { a0[i] = 0.0f; a1[i] = 0.0f; }
  const int routed_row0 = p.groups[n_always].w1_row0 / 2;
  for (int g = n_always; g < p.G; ++g) {
    const int seg0 = p.seg_off[g], cnt = p.seg_off[g + 1] - seg0;
    if (cnt == 0) continue;
    const int wp = p.groups[g].width_pad;
    const int64_t hoff = p.h_off[g];
    const int n0 = p.groups[g].w1_row0 / 2;
    for (int col = 0; col < cnt; ++col) {
      const int tok = p.slot2tok[seg0 + col];
      const float wt = w_by_slot[seg0 + col];
      for (int n = tid; n < wp; n += DS_WAVES * 64) {
        const bf16_t hv = p.h[hoff + (int64_t)col * wp + n];
        if (!neuron_survives(hv, mode, nscale[n0 + n], tau)) continue;
        const uint4* src = reinterpret_cast<const uint4*>(w2n + (int64_t)(n0 - routed_row0 + n) * p.d + c0);
        const uint4 q0 = src[0], q1 = src[1];
        const uint32_t w[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
        const float coef = wt * bf16_to_f32(hv);
        if (tok == 0) {
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            a0[2 * i] = fmaf(coef, __uint_as_float(w[i] << 16), a0[2 * i]);
            a0[2 * i + 1] = fmaf(coef, __uint_as_float(w[i] & 0xffff0000u), a0[2 * i + 1]);
          }
        } else {
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            a1[2 * i] = fmaf(coef, __uint_as_float(w[i] << 16), a1[2 * i]);
            a1[2 * i + 1] = fmaf(coef, __uint_as_float(w[i] & 0xffff0000u), a1[2 * i + 1]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    a0[i] = wave_sum(a0[i]);
    a1[i] = wave_sum(a1[i]);
  }
  wave_lds_sync_decode();                                   // the MFMA part's LDS updates of this wave are done
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      yacc[wave][0][i] += a0[i];
      yacc[wave][1][i] += a1[i];
    }
  }
  __syncthreads();
  for (int e = tid; e < (int)p.T * 16; e += DS_WAVES * 64) {
    const int t = e >> 4, cc = e & 15;
    float s = 0.0f;
#pragma unroll
    for (int w = 0; w < DS_WAVES; ++w) s += yacc[w][t][cc];
    y_out[(int64_t)t * p.d + c0 + cc] = f32_to_bf16(s);
  }
}

// Up to 16 tokens (one MFMA token tile) the weight-streaming kernels are the fastest form of both
// contractions; from 17 tokens on a second token tile would double their register footprint, and the tiled
// contraction on skinny tiles is as fast for the routed layer and 10-20 us faster for the dense one
// (measured at d = 4096).
constexpr int DECODE_MAX_T = 16;
bool decode_path_ok(const Engine& e, int64_t T) {
  if (e.dtype != 1 || T < 1 || T > DECODE_MAX_T) return false;
  if (e.d % 256 != 0) return false;
  const int ksteps = e.d / 256;
  return ksteps == 16 || ksteps == 8 || ksteps == 4 || ksteps == 2;
}

// The fused down + combine kernel serves every routed bf16 batch of at most 32 tokens with more than one slot
// per token, whichever kernel produced the hidden activations (the decode_fuse tuning switch selects the separate
// kernels, for comparison).
constexpr int DOWN_COMBINE_MAX_T = 32;
bool decode_fuses_combine(const Engine& e, int64_t T) {
  if (tuning().decode_fuse == 0 || use_simt_experts(e.dtype) || e.dtype != 1 || T < 1 || T > DOWN_COMBINE_MAX_T || e.d % 16 != 0) return false;
  return !(e.G == 1 && e.n_always == 1) && e.S_all() > 1;
}

// 8-neuron units when they still number at most one per CU (the always-on groups count unless the routing
// front end runs them).  Measured at one token: four routed experts of 448 neurons (224 units of 8) 10.1 ->
// 8.9 us for the gate/up launch, three of 688 (258 units of 8) 12.0 -> 14.8 us; at 16 tokens 28.7 -> 32.4 us.
// CMOE_DECODE_SPLIT = 8 / 16 forces a size.
int decode_unit_neurons(const Engine& e, int64_t T) {
  const int forced = tuning().decode_split;
  if (forced == 8 || forced == 16) return forced;
  if (decode_front_runs_all(e, T)) return 16;     // (measured: 27.9 against 31.4 us and 30.4 against 31.6 us at one token)
  const int64_t dyn_groups = std::min<int64_t>(T * e.S_dyn, e.G - e.n_always);
  int64_t units8 = e.G > e.n_always ? dyn_groups * (e.width_pad_host[e.n_always] / 8) : 0;
  if (!decode_front_runs_shared(e, T))
    for (int g = 0; g < e.n_always; ++g) units8 += e.width_pad_host[g] / 8;
  return units8 <= 256 ? 8 : 16;
}

int64_t decode_unit_bound(const Engine& e, int64_t T, int which) {
  const int64_t dyn_groups = std::min<int64_t>(T * e.S_dyn, e.G - e.n_always);
  const int64_t per_group = which == 1 ? e.max_width_pad / decode_unit_neurons(e, T) : e.d / 16;
  return std::max<int64_t>((e.n_always + dyn_groups) * per_group, 1);
}

template <int NTT>
static hipError_t launch_gate_up(const DecArgs& a, int ksteps, int64_t n_blocks, hipStream_t s) {
  dim3 grid((unsigned)n_blocks), block(512);
  switch (ksteps) {
    case 16: hipLaunchKernelGGL((decode_gate_up_kernel<NTT, 16>), grid, block, 0, s, a); break;
    case 8: hipLaunchKernelGGL((decode_gate_up_kernel<NTT, 8>), grid, block, 0, s, a); break;
    case 4: hipLaunchKernelGGL((decode_gate_up_kernel<NTT, 4>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((decode_gate_up_kernel<NTT, 2>), grid, block, 0, s, a); break;
  }
  return hipGetLastError();
}

DecArgs make_dec_args(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y) {
  DecArgs a;
  a.x = static_cast<const bf16_t*>(x);
  a.w1 = static_cast<const bf16_t*>(e.w1);
  a.w2 = static_cast<const bf16_t*>(e.w2);
  a.h = reinterpret_cast<bf16_t*>(ws + L.h);
  a.y = e.direct_output() ? static_cast<bf16_t*>(y) : reinterpret_cast<bf16_t*>(ws + L.y_slots);
  a.groups = e.groups;
  a.seg_off = reinterpret_cast<const int32_t*>(ws + L.seg_off);
  a.work = nullptr;
  a.h_off = reinterpret_cast<const int64_t*>(ws + L.h_off);
  a.G = e.G;
  a.d = e.d;
  a.ldw = e.ldw1;
  a.tiled = e.w_tiled;
  a.T = T;
  a.single = (e.G == 1 && e.n_always == 1) ? 1 : 0;
  a.slot2tok = a.single ? nullptr : reinterpret_cast<const int32_t*>(ws + L.slot2tok);
  a.unit1 = decode_unit_neurons(e, T);
  return a;
}

// Down contraction + weighted sum over slots in one launch (callers check decode_fuses_combine first).
hipError_t launch_decode_down_combine(const Engine& e, int64_t T, char* ws, const WsLayout& L, void* y, hipStream_t s) {
  const DecArgs a = make_dec_args(e, nullptr, T, ws, L, y);
  const float* wbs = reinterpret_cast<const float*>(ws + L.w_by_slot);
  bf16_t* yo = static_cast<bf16_t*>(y);
  if (T > 16) hipLaunchKernelGGL((decode_down_combine_kernel<2>), dim3(e.d / 16), dim3(DC_WAVES * 64), 0, s, a, wbs, yo);
  else hipLaunchKernelGGL((decode_down_combine_kernel<1>), dim3(e.d / 16), dim3(DC_WAVES * 64), 0, s, a, wbs, yo);
  return hipGetLastError();
}

bool decode_sparse_down_ok(const Engine& e, int64_t T) {
  return e.sparse_mode != 0 && e.w2n != nullptr && T >= 1 && T <= 2 && decode_fuses_combine(e, T);
}

hipError_t launch_decode_down_sparse(const Engine& e, int64_t T, char* ws, const WsLayout& L, void* y, hipStream_t s) {
  const DecArgs a = make_dec_args(e, nullptr, T, ws, L, y);
  const float* wbs = reinterpret_cast<const float*>(ws + L.w_by_slot);
  const int per_xcd = cdiv(e.d / 16, 8);
  hipLaunchKernelGGL(decode_down_sparse_kernel, dim3(8 * per_xcd), dim3(DS_WAVES * 64), 0, s, a, wbs, static_cast<bf16_t*>(y),
                     static_cast<const bf16_t*>(e.w2n), e.nscale, e.n_always, e.sparse_mode, e.sparse_tau, per_xcd);
  return hipGetLastError();
}

hipError_t launch_mask_hidden(const Engine& e, int64_t T, char* ws, const WsLayout& L, hipStream_t s) {
  if (e.sparse_mode == 0 || e.nscale == nullptr || e.G <= e.n_always) return hipSuccess;
  hipLaunchKernelGGL(mask_hidden_kernel, dim3((unsigned)(T * e.S_all())), dim3(256), 0, s, reinterpret_cast<bf16_t*>(ws + L.h),
                     e.groups, reinterpret_cast<const int32_t*>(ws + L.seg_off), reinterpret_cast<const int64_t*>(ws + L.h_off),
                     e.nscale, e.G, e.n_always, e.sparse_mode, e.sparse_tau);
  return hipGetLastError();
}

hipError_t launch_experts_decode(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y,
                                 hipStream_t s, int stage) {
  DecArgs a = make_dec_args(e, x, T, ws, L, y);
  if (stage != 2) {
    a.work = reinterpret_cast<const int32_t*>(ws + L.work1);
    const int64_t nb = a.single ? e.max_width_pad / a.unit1 : decode_unit_bound(e, T, 1);
    hipError_t err = launch_gate_up<1>(a, e.d / 256, nb, s);
    if (err != hipSuccess || stage == 1) return err;
  }
  if (decode_fuses_combine(e, T)) return launch_decode_down_combine(e, T, ws, L, y, s);
  a.work = reinterpret_cast<const int32_t*>(ws + L.work2);
  const int64_t nb = a.single ? e.d / 16 : decode_unit_bound(e, T, 2);
  hipLaunchKernelGGL((decode_down_kernel<1>), dim3((unsigned)nb), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace cmoe
