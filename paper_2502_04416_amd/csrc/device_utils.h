// Small device helpers: bf16 conversion, wave reductions, the wave-level top-k.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cmoe {

typedef uint16_t bf16_t;   // storage type of a bf16 element (bit pattern)

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even; NaN stays NaN.  The cast compiles to the hardware conversion of gfx950
// (v_cvt_pk_bf16_f32): no integer rounding sequence and no branch for the NaN case.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  const __bf16 h = static_cast<__bf16>(f);
  return __builtin_bit_cast(bf16_t, h);
}

// Work lists: work[0..G] is a non-decreasing prefix array (work[0] = 0, G <= 128 groups) and item u belongs
// to the last group g with work[g] <= u (empty groups are skipped).  Every lane looks at two entries and
// a ballot counts the entries that do not exceed u: one round of loads instead of the seven dependent
// ones of a binary search, which matters because every workgroup starts with this lookup.  Requires
// u < work[G]; all lanes of the wave must call it.
__device__ __forceinline__ int find_group(const int32_t* __restrict__ work, int G, int u) {
  const int lane = threadIdx.x & 63;
  const int i0 = 1 + lane, i1 = 65 + lane;
  const bool b0 = i0 <= G && work[i0] <= u;
  const bool b1 = i1 <= G && work[i1] <= u;
  return __popcll(__ballot(b0)) + __popcll(__ballot(b1));
}

// Inclusive prefix sums over the 64 lanes of a wave (six exchange steps).
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int n = __shfl_up(v, o, 64);
    if (lane >= o) v += n;
  }
  return v;
}
__device__ __forceinline__ long long wave_incl_scan(long long v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const long long n = __shfl_up(v, o, 64);
    if (lane >= o) v += n;
  }
  return v;
}

__device__ __forceinline__ float wave_incl_scan(float v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const float n = __shfl_up(v, o, 64);
    if (lane >= o) v += n;
  }
  return v;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// SiLU / Swish with beta = 1 (Eq. 3): z * sigmoid(z), evaluated in fp32.
__device__ __forceinline__ float silu_f32(float z) { return z / (1.0f + expf(-z)); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Monotone map float -> uint32 (larger float <=> larger integer; -0 < +0).
__device__ __forceinline__ uint32_t ordered_key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Wave arg-max: every lane passes (key, active); returns the lane index holding the largest key
// among active lanes, ties to the lowest lane; -1 when no lane is active.  All 64 lanes must call.
__device__ __forceinline__ int wave_argmax(float key, bool active) {
  const int lane = threadIdx.x & 63;
  uint32_t hi = active ? ordered_key(key) : 0u;
  uint32_t lo = active ? (uint32_t)(64 - lane) : 0u;     // larger = lower lane; 0 = inactive
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    uint32_t ohi = __shfl_xor(hi, o, 64);
    uint32_t olo = __shfl_xor(lo, o, 64);
    bool take = (ohi > hi) || (ohi == hi && olo > lo);
    hi = take ? ohi : hi;
    lo = take ? olo : lo;
  }
  return lo == 0u ? -1 : 64 - (int)lo;
}

}  // namespace cmoe
