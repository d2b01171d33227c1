// Host-side weight slicing and packing (Sec. 4.1: experts are slices of the dense matrices by neuron
// index; Eq. 8: the router is the pair of columns of the representative neurons).
#pragma once
#include <cstdint>
#include <cstring>
#include <functional>
#include <thread>
#include <vector>
#include "cmoe_internal.h"

namespace cmoe {

// fp32 -> bf16 bit pattern, round-to-nearest-even (NaN kept quiet)
static inline uint16_t host_f32_to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
static inline float host_bf16_to_f32(uint16_t v) {
  uint32_t u = ((uint32_t)v) << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

// Run fn(i) for i in [0, n) on up to `max_threads` host threads (static chunks).
void parallel_for(int64_t n, const std::function<void(int64_t)>& fn, int max_threads = 0);

// Packed weights of a list of expert groups, kept on the host until upload.
struct PackedSet {
  int dtype = 1;
  int d = 0;
  int ld = 0;                       // elements per row of w1 (row-major: w1_row_stride(d); tiled: 32 * tiles along K)
  bool tiled = false;               // 16 x 32 tiles (bf16) instead of row-major rows (fp32)
  std::vector<GroupDev> groups;     // offsets relative to this set's own W1 / W2
  std::vector<int> width;           // real neuron count per group
  std::vector<uint8_t> w1;          // [rows][ld] interleaved gate/up rows (tiled: tiles of all 16-row blocks)
  std::vector<uint8_t> w2;          // per group [d][width_pad] (tiled: d padded to a multiple of 16 rows)
  int64_t w1_rows = 0;
  int64_t w2_elems = 0;
};

// Dense matrices transposed to neuron-major and rounded to the layer dtype once:
// gate_t, up_t: [d_ff][d]; down: [d_ff][d] (already neuron-major).
struct RoundedDense {
  int dtype = 1, d = 0, d_ff = 0;
  std::vector<uint8_t> gate_t, up_t, down;
  void from_fp32(int dtype_, int d_, int d_ff_, const float* w_gate, const float* w_up, const float* w_down);
  const uint8_t* gate_row(int64_t i) const { return gate_t.data() + i * d * elem_size(dtype); }
  const uint8_t* up_row(int64_t i) const { return up_t.data() + i * d * elem_size(dtype); }
  const uint8_t* down_row(int64_t i) const { return down.data() + i * d * elem_size(dtype); }
};

// Append one group (the listed dense neuron ids, padded with zero neurons to a multiple of WPAD).
void pack_group(PackedSet& ps, const RoundedDense& rd, const int32_t* neurons, int width);
// Layout of a set for the layer's dtype and width (call before the first pack_group).
void init_packed_set(PackedSet& ps, int dtype, int d);

// Router rows for `n` representative neurons in SwiGLU blocks of 2*IL rows; appended to `out`
// ([rows][d] in the layer dtype); scored expert index = first_index + j decides the block and row.
void pack_router_rows(std::vector<uint8_t>& out, int dtype, int d, int n_scored_total);
void set_router_rows(std::vector<uint8_t>& out, const RoundedDense& rd, int scored_index, int32_t rep_neuron);

}  // namespace cmoe
