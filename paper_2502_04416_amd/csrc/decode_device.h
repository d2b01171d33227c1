// Pieces of the decode kernels that more than one translation unit launches: the argument block and the
// gate/up contraction of one 16-neuron unit (the routing front end runs the shared expert's units in the
// launch that selects and places the tokens).
#pragma once
#include "cmoe_internal.h"
#include "device_utils.h"

namespace cmoe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

struct DecArgs {
  const bf16_t* x;          // [T][d]
  const bf16_t* w1;
  const bf16_t* w2;
  bf16_t* h;                // ragged hidden activations
  bf16_t* y;                // per-slot outputs [n_slots][d] (or y itself when every token has one slot)
  const GroupDev* groups;
  const int32_t* seg_off;
  const int32_t* work;      // [G+1] prefix of units
  const int64_t* h_off;
  const int32_t* slot2tok;
  int G, d;
  int ldw;                  // elements per row of w1
  int tiled;                // 1: w1 and w2 are tiled 16 x 32: the weights of one operand are 1 KB of consecutive memory
  int64_t T;
  int single;
  int unit1;                // neurons per gate/up unit: 16 or 8
};

__device__ __forceinline__ bf16x8_t ld_frag(const bf16_t* p) { return *reinterpret_cast<const bf16x8_t*>(p); }
__device__ __forceinline__ bf16x8_t zero_frag() {
  bf16x8_t z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = (__bf16)0.0f;
  return z;
}

// Shared memory a workgroup needs for decode_gate_up_unit.
template <int NTT>
struct DecGateUpRed { float v[8][2][NTT][16][17]; };

// H[slot][n] = Swish(x . wgate_n) * (x . wup_n) for the 16 neurons [local*16, local*16+16) of group g, whose
// cnt <= 16*NTT tokens are the slots seg0 .. seg0+cnt-1 and whose rows of H start at element hoff.
// Called by all 512 threads of a workgroup: 8 waves, wave w multiplies the K slice [w*d/8, (w+1)*d/8).
// NTT = token tiles of 16.  KSTEPS = d/8/32.
template <int NTT, int KSTEPS>
__device__ __forceinline__ void decode_gate_up_unit(const DecArgs& p, int g, int local, int seg0, int cnt, int wp,
                                                    int64_t hoff, DecGateUpRed<NTT>& redbuf) {
  float (*red)[2][NTT][16][17] = redbuf.v;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kq = lane >> 4;
  const int neuron0 = local * 16;
  const int kbase = wave * (KSTEPS * 32) + kq * 8;
  // weight rows of this lane: packed row = (n / IL) * 2 * IL + n % IL (+ IL for the up row)
  const int n = neuron0 + r16;
  const int64_t grow = (int64_t)p.groups[g].w1_row0 + (n / IL) * 2 * IL + (n % IL);
  // (grow is a multiple of 16 plus lane%16, kbase a multiple of 32 plus (lane/16)*8: one tile per K step)
  const bf16_t* wg = p.w1 + (p.tiled ? tiled_offset(grow, kbase, p.ldw / TILE_K) : grow * p.ldw + kbase);
  const bf16_t* wu = wg + (p.tiled ? (int64_t)(IL / TILE_ROWS) * (p.ldw / TILE_K) * TILE_ELEMS : (int64_t)IL * p.ldw);
  const int kadv = p.tiled ? TILE_ELEMS : 32;                 // elements from one K step's operand to the next
  // The gate rows of the unit are requested before anything else (the stream from HBM is what the kernel
  // waits for; left to itself the compiler keeps half a dozen weight loads in flight per wave), the up rows
  // as the loop goes.  Requesting those up front as well costs a third workgroup per CU and gains nothing.
  bf16x8_t ag[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) ag[ks] = ld_frag(wg + ks * kadv);
  __builtin_amdgcn_sched_barrier(0);
  // tokens (B operand), kept for the whole unit
  bf16x8_t bx[NTT][KSTEPS];
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt) {
    const int col = tt * 16 + r16;
    const bool ok = col < cnt;
    int64_t tok = 0;
    if (ok) tok = p.slot2tok ? p.slot2tok[seg0 + col] : (seg0 + col);
    const bf16_t* xr = p.x + tok * p.d + kbase;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) bx[tt][ks] = ok ? ld_frag(xr + ks * 32) : zero_frag();
  }
  floatx4_t accg[NTT], accu[NTT];
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
    for (int i = 0; i < 4; ++i) { accg[tt][i] = 0.0f; accu[tt][i] = 0.0f; }
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) {
    const bf16x8_t au = ld_frag(wu + ks * kadv);
#pragma unroll
    for (int tt = 0; tt < NTT; ++tt) {
      accg[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ag[ks], bx[tt][ks], accg[tt], 0, 0, 0);
      accu[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(au, bx[tt][ks], accu[tt], 0, 0, 0);
    }
  }
  // accumulator element i: neuron row (lane/16)*4 + i, token column lane%16
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      red[wave][0][tt][kq * 4 + i][r16] = accg[tt][i];
      red[wave][1][tt][kq * 4 + i][r16] = accu[tt][i];
    }
  __syncthreads();
  for (int e = tid; e < NTT * 256; e += 512) {
    const int tt = e >> 8, tok = (e >> 4) & 15, nn = e & 15;     // neuron fastest: contiguous stores
    const int col = tt * 16 + tok;
    if (col >= cnt) continue;
    float sg = 0.0f, su = 0.0f;
#pragma unroll
    for (int w = 0; w < 8; ++w) { sg += red[w][0][tt][nn][tok]; su += red[w][1][tt][nn][tok]; }
    p.h[hoff + (int64_t)col * wp + neuron0 + nn] = f32_to_bf16(silu_f32(sg) * su);
  }
}

// The same for 8 neurons: one MFMA operand holds the 8 gate rows (operand rows 0-7) and the 8 up rows (8-15) of
// the unit, so a unit is half as long and a launch has twice as many; taken when 16-neuron units would leave
// CUs without a workgroup (one token on a layer of few selected experts).  A load instruction covers two
// 512-byte pieces instead of 1 KB.  K slices, their order and the order of the final sum are those of the
// 16-neuron unit: H comes out bit for bit the same.
template <int NTT, int KSTEPS>
__device__ __forceinline__ void decode_gate_up_unit8(const DecArgs& p, int g, int local, int seg0, int cnt, int wp,
                                                     int64_t hoff, DecGateUpRed<NTT>& redbuf) {
  float (*red)[2][NTT][16][17] = redbuf.v;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kq = lane >> 4;
  const int neuron0 = local * 8;
  const int kbase = wave * (KSTEPS * 32) + kq * 8;
  const int n = neuron0 + (r16 & 7);
  const int64_t grow = (int64_t)p.groups[g].w1_row0 + (n / IL) * 2 * IL + (n % IL) + (r16 >= 8 ? IL : 0);
  const bf16_t* wrow = p.w1 + (p.tiled ? tiled_offset(grow, kbase, p.ldw / TILE_K) : grow * p.ldw + kbase);
  const int kadv = p.tiled ? TILE_ELEMS : 32;
  bf16x8_t a[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) a[ks] = ld_frag(wrow + ks * kadv);
  __builtin_amdgcn_sched_barrier(0);
  floatx4_t acc[NTT];
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[tt][i] = 0.0f;
    const int col = tt * 16 + r16;
    const bool ok = col < cnt;
    int64_t tok = 0;
    if (ok) tok = p.slot2tok ? p.slot2tok[seg0 + col] : (seg0 + col);
    const bf16_t* xr = p.x + tok * p.d + kbase;
    bf16x8_t bx[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) bx[ks] = ok ? ld_frag(xr + ks * 32) : zero_frag();
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks], bx[ks], acc[tt], 0, 0, 0);
  }
  // accumulator element i: operand row (lane/16)*4 + i (0-7 gate, 8-15 up of neuron row % 8), token column lane%16
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
    for (int i = 0; i < 4; ++i) red[wave][0][tt][kq * 4 + i][r16] = acc[tt][i];
  __syncthreads();
  for (int e = tid; e < NTT * 128; e += 512) {
    const int tt = e >> 7, tok = (e >> 3) & 15, nn = e & 7;
    const int col = tt * 16 + tok;
    if (col >= cnt) continue;
    float sg = 0.0f, su = 0.0f;
#pragma unroll
    for (int w = 0; w < 8; ++w) { sg += red[w][0][tt][nn][tok]; su += red[w][0][tt][8 + nn][tok]; }
    p.h[hoff + (int64_t)col * wp + neuron0 + nn] = f32_to_bf16(silu_f32(sg) * su);
  }
}

// Host side (decode.hip): the argument block of a forward.
DecArgs make_dec_args(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y);
// Neurons per gate/up unit of the decode kernels for this batch (16, or 8 when that fills the chip better).
int decode_unit_neurons(const Engine& e, int64_t T);

}  // namespace cmoe
