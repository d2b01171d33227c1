// C ABI of libcmoe (see include/cmoe.h): handles, argument checks, weight packing and upload, and the
// forward calls, which only enqueue kernels on the caller's stream.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <exception>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/cmoe.h"
#include "cmoe_internal.h"
#include "host_build.h"
#include "host_pack.h"

namespace cmoe {

// ---------------------------------------------------------------------------------- errors
static thread_local std::string g_err = "";
int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
static int fail_hip(hipError_t e, const char* what) {
  return fail(CMOE_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// ---------------------------------------------------------------------------------- small helpers
size_t elem_size(int dtype) { return dtype == CMOE_BF16 ? 2 : 4; }

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct TuningField { const char* name; int Tuning::*field; };
static const TuningField kTuningFields[] = {
    {"CMOE_GEMM1_CFG", &Tuning::gemm1_cfg},     {"CMOE_GEMM2_CFG", &Tuning::gemm2_cfg},
    {"CMOE_XCD_REMAP", &Tuning::xcd_remap},     {"CMOE_SPLITK", &Tuning::splitk},
    {"CMOE_ZERO_PAD", &Tuning::zero_pad},       {"CMOE_DECODE_FUSE", &Tuning::decode_fuse},
    {"CMOE_FRONT_SHARED", &Tuning::front_shared}, {"CMOE_FORCE_SIMT", &Tuning::force_simt},
    {"CMOE_LDPAD", &Tuning::ldpad},             {"CMOE_HOST_THREADS", &Tuning::host_threads},
    {"CMOE_SKIP_ROWS", &Tuning::skip_rows},     {"CMOE_DECODE_SPLIT", &Tuning::decode_split},
    {"CMOE_WS_DOWN", &Tuning::ws_down},         {"CMOE_SKIP_STAGE", &Tuning::skip_stage},
    {"CMOE_REPEAT_STAGE", &Tuning::repeat_stage}, {"CMOE_FRONT_ALL", &Tuning::front_all},
    {"CMOE_FRONT_TILE", &Tuning::front_tile},
};

Tuning& tuning() {
  static Tuning t = [] {
    Tuning v;
    for (const TuningField& f : kTuningFields)
      if (const char* e = std::getenv(f.name)) v.*(f.field) = std::atoi(e);
    return v;
  }();
  return t;
}

int w1_row_stride(int d) {
  const int pad = tuning().ldpad;
  return d + ((pad > 0 && pad % 8 == 0) ? pad : 0);
}

void parallel_for(int64_t n, const std::function<void(int64_t)>& fn, int max_threads) {
  int nt = max_threads > 0 ? max_threads : (int)std::thread::hardware_concurrency();
  if (tuning().host_threads > 0) nt = tuning().host_threads;
  if (nt > 16) nt = 16;
  if (nt < 1) nt = 1;
  if ((int64_t)nt > n) nt = (int)std::max<int64_t>(n, 1);
  if (nt == 1) {
    for (int64_t i = 0; i < n; ++i) fn(i);
    return;
  }
  // An exception inside a worker (an allocation that fails) is carried over to the calling thread; one
  // thrown while the threads are being created (std::system_error) leaves after the ones that exist joined.
  std::vector<std::thread> th;
  std::vector<std::exception_ptr> err(nt);
  std::exception_ptr spawn_err;
  try {
    th.reserve(nt);
    for (int w = 0; w < nt; ++w)
      th.emplace_back([=, &fn, &err]() {
        try {
          const int64_t lo = n * w / nt, hi = n * (w + 1) / nt;
          for (int64_t i = lo; i < hi; ++i) fn(i);
        } catch (...) {
          err[w] = std::current_exception();
        }
      });
  } catch (...) {
    spawn_err = std::current_exception();
  }
  const size_t started = th.size();
  for (auto& t : th) t.join();
  if (spawn_err) {
    // the chunks of the threads that never started still have to run
    for (int w = (int)started; w < nt; ++w) {
      const int64_t lo = n * w / nt, hi = n * (w + 1) / nt;
      for (int64_t i = lo; i < hi; ++i) fn(i);
    }
  }
  for (auto& e : err)
    if (e) std::rethrow_exception(e);
}

bool use_simt_experts(int dtype) { return dtype != CMOE_BF16 || tuning().force_simt != 0; }

int gemm_tile(const Engine& e, int64_t T, int which) {
  return use_simt_experts(e.dtype) ? simt_gemm_tile(which) : bf16_gemm_tile(which, e, T);
}

int64_t gemm_work_bound(const Engine& e, int64_t T, int which) {
  const int bm = gemm_tile(e, T, which == 1 ? 1 : 2);
  const int bn = gemm_tile(e, T, which == 1 ? 3 : 4);
  auto nt_of = [&](int g) { return which == 1 ? cdiv(2 * e.width_pad_host[g], bn) : cdiv(e.d, bn); };
  const int64_t mt_all = (T + bm - 1) / bm;
  int64_t total = 0;
  for (int g = 0; g < e.n_always; ++g) total += mt_all * nt_of(g);
  int64_t per_group = 0;
  int nt_max = 0;
  for (int g = e.n_always; g < e.G; ++g) {
    per_group += mt_all * nt_of(g);
    nt_max = std::max(nt_max, nt_of(g));
  }
  const int64_t by_entries = (int64_t)nt_max * (T * e.S_dyn / bm + (e.G - e.n_always));
  total += std::min(per_group, by_entries);
  return std::max<int64_t>(total, 1);
}

WsLayout ws_layout(const Engine& e, int64_t T, size_t splitk_cap) {
  WsLayout L{};
  const size_t es = elem_size(e.dtype);
  const int64_t Tn = std::max<int64_t>(T, 1);
  const int S_all = e.S_all();
  L.n_slots = Tn * S_all;
  L.n_tok_tiles = (int)((Tn + TOK_TILE - 1) / TOK_TILE);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
  L.sel_group = take(sizeof(int32_t) * Tn * std::max(e.S_dyn, 1));
  L.sel_weight = take(sizeof(float) * Tn * std::max(e.S_dyn, 1));
  L.tile_counts = take(sizeof(int32_t) * (size_t)L.n_tok_tiles * e.G);
  L.seg_off = take(sizeof(int32_t) * (e.G + 1));
  L.counts = take(sizeof(int32_t) * (e.G + 1));
  L.work1 = take(sizeof(int32_t) * (e.G + 1 + 9));       // + first work item of each XCD's share
  L.work2 = take(sizeof(int32_t) * (e.G + 1 + 9));
  L.h_off = take(sizeof(int64_t) * (e.G + 1));
  L.slot2tok = take(sizeof(int32_t) * L.n_slots);
  L.tok2slot = take(sizeof(int32_t) * L.n_slots);
  L.slot_w = take(sizeof(float) * L.n_slots);
  L.w_by_slot = take(sizeof(float) * L.n_slots);
  L.scores = take(sizeof(float) * 8 * Tn * std::max(e.r.n_sw_rows + e.r.n_lin_rows, 1));   // router K-slice partials
  L.h = take(es * (size_t)Tn * (size_t)e.h_per_token);
  L.y_slots = take(e.direct_output() ? 0 : es * (size_t)L.n_slots * e.d);
  // Partial sums of a K-split contraction: reserved in full whenever the largest batch runs the tiled
  // contraction kernels (then smaller ones may too, and may split further), so that the size grows with T.
  L.splitk_bytes = (!use_simt_experts(e.dtype) && !decode_path_ok(e, Tn)) ? std::min(bf16_splitk_bytes(e, Tn), splitk_cap) : 0;
  L.splitk = take(L.splitk_bytes);
  L.total = off;
  return L;
}

hipError_t launch_experts(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y,
                          hipStream_t s, int stage) {
  if (T == 0) return hipSuccess;
  if (use_simt_experts(e.dtype)) return launch_experts_simt(e, x, T, ws, L, y, s, stage);
  if (stage == 2 && e.sparse_mode != 0 && decode_sparse_down_ok(e, T)) return launch_decode_down_sparse(e, T, ws, L, y, s);
  if (stage == 2 && decode_fuses_combine(e, T)) return launch_decode_down_combine(e, T, ws, L, y, s);
  if (decode_path_ok(e, T)) return launch_experts_decode(e, x, T, ws, L, y, s, stage);
  return launch_experts_bf16(e, x, T, ws, L, y, s, stage);
}

// ---------------------------------------------------------------------------------- packing
static void store_elem(uint8_t* dst, int dtype, float v) {
  if (dtype == CMOE_BF16) {
    const uint16_t b = host_f32_to_bf16(v);
    std::memcpy(dst, &b, 2);
  } else {
    std::memcpy(dst, &v, 4);
  }
}

void RoundedDense::from_fp32(int dtype_, int d_, int d_ff_, const float* w_gate, const float* w_up,
                             const float* w_down) {
  dtype = dtype_;
  d = d_;
  d_ff = d_ff_;
  const size_t es = elem_size(dtype);
  gate_t.assign((size_t)d * d_ff * es, 0);
  up_t.assign((size_t)d * d_ff * es, 0);
  down.assign((size_t)d * d_ff * es, 0);
  // blocked transpose [d][d_ff] -> [d_ff][d] with rounding; 64 neurons per task
  const int64_t n_blocks = (d_ff + 63) / 64;
  parallel_for(n_blocks, [&](int64_t b) {
    const int i0 = (int)b * 64, i1 = std::min(d_ff, i0 + 64);
    for (int k0 = 0; k0 < d; k0 += 64) {
      const int k1 = std::min(d, k0 + 64);
      for (int k = k0; k < k1; ++k) {
        const float* gs = w_gate + (size_t)k * d_ff;
        const float* us = w_up + (size_t)k * d_ff;
        for (int i = i0; i < i1; ++i) {
          store_elem(gate_t.data() + ((size_t)i * d + k) * es, dtype, gs[i]);
          store_elem(up_t.data() + ((size_t)i * d + k) * es, dtype, us[i]);
        }
      }
    }
    for (int i = i0; i < i1; ++i) {
      const float* src = w_down + (size_t)i * d;
      uint8_t* dst = down.data() + (size_t)i * d * es;
      for (int c = 0; c < d; ++c) store_elem(dst + (size_t)c * es, dtype, src[c]);
    }
  });
}

void init_packed_set(PackedSet& ps, int dtype, int d) {
  ps.dtype = dtype;
  ps.d = d;
  ps.tiled = dtype == CMOE_BF16;
  ps.ld = ps.tiled ? TILE_K * tiles_along_k(d) : w1_row_stride(d);
}

// Tiled variant of pack_group: same rows, same zero padding, 16 x 32 tiles.
static void pack_group_tiled(PackedSet& ps, const RoundedDense& rd, const int32_t* neurons, int width) {
  const size_t es = elem_size(ps.dtype);
  const int d = ps.d;
  const int wp = round_up(width, WPAD);
  const int kt1 = ps.ld / TILE_K;                     // tiles along K of W1
  const int kt2 = wp / TILE_K;                        // tiles along K (= neurons) of this group's W2
  const int d16 = round_up(d, TILE_ROWS);
  GroupDev gd;
  gd.width_pad = wp;
  gd.w1_row0 = (int32_t)ps.w1_rows;
  gd.w2_off = ps.w2_elems;
  ps.groups.push_back(gd);
  ps.width.push_back(width);
  const int64_t row0 = ps.w1_rows;                    // a multiple of 2 * IL, hence of the tile height
  ps.w1.resize((size_t)(row0 + 2 * wp) * ps.ld * es, 0);
  const size_t w2_base = ps.w2.size();
  ps.w2.resize(w2_base + (size_t)d16 * wp * es, 0);
  ps.w1_rows += 2 * wp;
  ps.w2_elems += (int64_t)d16 * wp;
  auto put_row = [&](int64_t row, const uint8_t* src) {
    for (int k0 = 0; k0 < d; k0 += TILE_K) {
      const int n = std::min(TILE_K, d - k0);
      std::memcpy(ps.w1.data() + (size_t)tiled_offset(row, k0, kt1) * es, src + (size_t)k0 * es, (size_t)n * es);
    }
  };
  parallel_for(wp / IL, [&](int64_t blk) {
    for (int c = 0; c < IL; ++c) {
      const int n = (int)blk * IL + c;
      if (n >= width) continue;
      put_row(row0 + blk * 2 * IL + c, rd.gate_row(neurons[n]));
      put_row(row0 + blk * 2 * IL + IL + c, rd.up_row(neurons[n]));
    }
  });
  parallel_for((d + 63) / 64, [&](int64_t cb) {
    const int c0 = (int)cb * 64, c1 = std::min(d, c0 + 64);
    for (int n = 0; n < width; ++n) {
      const uint8_t* src = rd.down_row(neurons[n]);
      for (int c = c0; c < c1; ++c)
        std::memcpy(ps.w2.data() + w2_base + (size_t)tiled_offset(c, n, kt2) * es, src + (size_t)c * es, es);
    }
  });
}

void pack_group(PackedSet& ps, const RoundedDense& rd, const int32_t* neurons, int width) {
  if (ps.tiled) {
    pack_group_tiled(ps, rd, neurons, width);
    return;
  }
  const size_t es = elem_size(ps.dtype);
  const int d = ps.d;
  const int wp = round_up(width, WPAD);
  GroupDev gd;
  gd.width_pad = wp;
  gd.w1_row0 = (int32_t)ps.w1_rows;
  gd.w2_off = ps.w2_elems;
  ps.groups.push_back(gd);
  ps.width.push_back(width);
  const size_t row_bytes = (size_t)d * es;            // payload of a row
  const size_t ld_bytes = (size_t)ps.ld * es;         // distance between rows of w1
  const size_t w1_base = ps.w1.size();
  ps.w1.resize(w1_base + (size_t)2 * wp * ld_bytes, 0);
  const size_t w2_base = ps.w2.size();
  ps.w2.resize(w2_base + (size_t)d * wp * es, 0);
  ps.w1_rows += 2 * wp;
  ps.w2_elems += (int64_t)d * wp;
  // gate/up rows: packed row = blk*2*IL + {0: gate, IL: up} + c  <->  neuron blk*IL + c
  parallel_for(wp / IL, [&](int64_t blk) {
    for (int c = 0; c < IL; ++c) {
      const int n = (int)blk * IL + c;
      if (n >= width) continue;
      uint8_t* g_dst = ps.w1.data() + w1_base + ((size_t)blk * 2 * IL + c) * ld_bytes;
      uint8_t* u_dst = ps.w1.data() + w1_base + ((size_t)blk * 2 * IL + IL + c) * ld_bytes;
      std::memcpy(g_dst, rd.gate_row(neurons[n]), row_bytes);
      std::memcpy(u_dst, rd.up_row(neurons[n]), row_bytes);
    }
  });
  // down: W2[c][n] = W_down[neuron n][c]; tiles of 64 output columns per task
  parallel_for((d + 63) / 64, [&](int64_t cb) {
    const int c0 = (int)cb * 64, c1 = std::min(d, c0 + 64);
    for (int n = 0; n < width; ++n) {
      const uint8_t* src = rd.down_row(neurons[n]);
      for (int c = c0; c < c1; ++c)
        std::memcpy(ps.w2.data() + w2_base + ((size_t)c * wp + n) * es, src + (size_t)c * es, es);
    }
  });
}

void pack_router_rows(std::vector<uint8_t>& out, int dtype, int d, int n_scored_total) {
  const int rows = 2 * IL * cdiv(std::max(n_scored_total, 0), IL);
  out.assign((size_t)rows * d * elem_size(dtype), 0);
}

void set_router_rows(std::vector<uint8_t>& out, const RoundedDense& rd, int scored_index, int32_t rep) {
  const size_t row_bytes = (size_t)rd.d * elem_size(rd.dtype);
  const int blk = scored_index / IL, c = scored_index % IL;
  std::memcpy(out.data() + ((size_t)blk * 2 * IL + c) * row_bytes, rd.gate_row(rep), row_bytes);
  std::memcpy(out.data() + ((size_t)blk * 2 * IL + IL + c) * row_bytes, rd.up_row(rep), row_bytes);
}

}  // namespace cmoe

using namespace cmoe;

// ---------------------------------------------------------------------------------- handles
struct cmoe_layer {
  cmoe_config cfg{};
  int m = 0, n_r = 0;
  std::vector<int32_t> neuron_order, rep_neuron;
  std::vector<float> mu;
  double cost = 0.0;
  PackedSet moe, dense;
  std::vector<uint8_t> router;                 // [n_sw_rows][d]
  std::vector<uint8_t> rep_rows;               // [N_r][2][d] gate row, up row of each R_j (for a hierarchy)
  std::vector<float> u, b;
  bool has_u = false, has_b = false;
  bool uploaded = false;
  bool in_hier = false;
  bool baseline = true;                        // the dense single-group copy is packed and uploaded too
  // neuron-level sparsity inside the routed experts (cmoe_set_neuron_sparsity)
  int sparse_mode = 0;
  float sparse_tau = 0.0f;
  bool sparse_reserved = false;                // w2n / nscale are built and belong to the packed weights
  std::vector<uint8_t> w2n;                    // routed groups' down rows, neuron-major [sum width_pad][d]
  std::vector<float> nscale;                   // [sum of all width_pad] L2 norm of each neuron's down row
  int64_t calib_routed = -1, calib_used = -1;  // cmoe_hier_build: calibration tokens routed to / used for this expert
  Engine e_moe, e_dense;
  float* d_u = nullptr;
  float* d_b = nullptr;
};

struct cmoe_hier {
  std::vector<cmoe_layer*> experts;
  cmoe_config cfg{};
  int n_outer = 0, outer_top_k = 0;
  std::vector<uint8_t> router;                 // SwiGLU rows of all sub-routers, then IL linear rows
  std::vector<uint8_t> lin_rows;               // [IL][d] outer router, rows = outer experts
  std::vector<float> lin_off;
  bool uploaded = false;
  bool owns_experts = false;                   // built by cmoe_hier_build: destroyed with the hierarchy
  bool baseline = true;
  Engine e_moe, e_dense;
};

// Every entry point that can reach an allocation or a thread runs its body between these two: nothing
// may propagate through the C boundary.
#define CMOE_TRY try {
#define CMOE_CATCH                                                                             \
  }                                                                                            \
  catch (const std::bad_alloc&) { return fail(CMOE_ENOMEM, "out of host memory"); }            \
  catch (const std::exception& ex) { return fail(CMOE_EINVAL, "internal error: %s", ex.what()); } \
  catch (...) { return fail(CMOE_EINVAL, "internal error"); }

static int check_config(const cmoe_config* c) {
  if (!c) return fail(CMOE_EINVAL, "config is null");
  if (c->dtype != CMOE_F32 && c->dtype != CMOE_BF16) return fail(CMOE_EINVAL, "dtype must be CMOE_F32 or CMOE_BF16");
  if (c->d_model < 1 || c->d_ff < 1 || c->n_experts < 1) return fail(CMOE_EINVAL, "d_model, d_ff, n_experts must be positive");
  if (c->d_ff % c->n_experts != 0)
    return fail(CMOE_EINVAL, "d_ff (%d) is not a multiple of n_experts (%d): m = d_h / N must be integral", c->d_ff, c->n_experts);
  if (c->n_shared < 0 || c->n_shared >= c->n_experts) return fail(CMOE_EINVAL, "need 0 <= n_shared < n_experts");
  const int n_r = c->n_experts - c->n_shared;
  if (c->top_k < 1 || c->top_k > n_r) return fail(CMOE_EINVAL, "need 1 <= top_k <= n_experts - n_shared (%d)", n_r);
  if (c->top_k > MAX_TOPK) return fail(CMOE_EINVAL, "top_k above %d is not supported", MAX_TOPK);
  if (n_r > MAX_SCORED) return fail(CMOE_EINVAL, "more than %d routed experts are not supported", MAX_SCORED);
  if (c->dtype == CMOE_BF16 && c->d_model % 8 != 0) return fail(CMOE_EINVAL, "bf16 layers need d_model %% 8 == 0");
  if (c->score_mode != 0 && c->score_mode != 1) return fail(CMOE_EINVAL, "score_mode must be 0 or 1");
  return CMOE_OK;
}

static void fill_flat_engines(cmoe_layer* L) {
  const cmoe_config& c = L->cfg;
  Engine& e = L->e_moe;
  e = Engine{};
  e.dtype = c.dtype;
  e.d = c.d_model;
  e.ldw1 = L->moe.ld;
  e.w_tiled = L->moe.tiled ? 1 : 0;
  e.G = (int)L->moe.groups.size();
  e.n_always = c.n_shared > 0 ? 1 : 0;
  e.S_dyn = c.top_k;
  e.h_per_token = 0;
  for (int g = 0; g < e.G; ++g) {
    e.width_pad_host[g] = L->moe.groups[g].width_pad;
    e.max_width_pad = std::max(e.max_width_pad, L->moe.groups[g].width_pad);
  }
  if (e.n_always) e.h_per_token += L->moe.groups[0].width_pad;
  e.h_per_token += (int64_t)c.top_k * L->moe.groups[e.G - 1].width_pad;
  RouterDev& r = e.r;
  r.n_scored = L->n_r;
  r.n_sw_rows = 2 * IL * cdiv(L->n_r, IL);
  r.n_lin = 0;
  r.n_lin_rows = 0;
  r.top_k = c.top_k;
  r.outer_top_k = 0;
  r.n_r_sub = L->n_r;
  r.n_always = e.n_always;
  r.score_abs = c.score_mode;
  r.use_gate = (L->has_u || L->has_b) ? 1 : 0;
  r.groups_per_outer = 0;
  r.sub_has_shared = 0;
  Engine& dn = L->e_dense;
  dn = Engine{};
  dn.dtype = c.dtype;
  dn.d = c.d_model;
  dn.ldw1 = L->dense.ld;
  dn.w_tiled = L->dense.tiled ? 1 : 0;
  dn.G = 1;
  dn.n_always = 1;
  dn.S_dyn = 0;
  dn.width_pad_host[0] = L->dense.groups[0].width_pad;
  dn.max_width_pad = dn.width_pad_host[0];
  dn.h_per_token = dn.width_pad_host[0];
  dn.r.n_always = 1;
}

static int build_common(const cmoe_config* cfg, const float* w_gate, const float* w_up, const float* w_down,
                        const float* calib_x, int64_t q, const int32_t* order_in, const int32_t* rep_in,
                        cmoe_layer** out, bool profile_on_gpu = false) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!w_gate || !w_up || !w_down || !out) return fail(CMOE_EINVAL, "null weight or output pointer");
  const int d = cfg->d_model, d_ff = cfg->d_ff, N = cfg->n_experts, m = d_ff / N;
  const int n_r = N - cfg->n_shared;
  std::unique_ptr<cmoe_layer> L(new (std::nothrow) cmoe_layer());
  if (!L) return fail(CMOE_ENOMEM, "out of host memory");
  try {
    L->cfg = *cfg;
    L->m = m;
    L->n_r = n_r;
    L->mu.assign(d_ff, 0.0f);
    RoundedDense rd;
    rd.from_fp32(cfg->dtype, d, d_ff, w_gate, w_up, w_down);
    if (order_in) {
      if (!rep_in) return fail(CMOE_EINVAL, "rep_neuron is null");
      std::vector<char> seen(d_ff, 0);
      for (int i = 0; i < d_ff; ++i) {
        const int v = order_in[i];
        if (v < 0 || v >= d_ff || seen[v]) return fail(CMOE_EINVAL, "neuron_order is not a permutation of 0..d_ff-1 (entry %d)", i);
        seen[v] = 1;
      }
      for (int j = 0; j < n_r; ++j)
        if (rep_in[j] < 0 || rep_in[j] >= d_ff) return fail(CMOE_EINVAL, "rep_neuron[%d] out of range", j);
      L->neuron_order.assign(order_in, order_in + d_ff);
      L->rep_neuron.assign(rep_in, rep_in + n_r);
    } else {
      if (!calib_x || q < 1) return fail(CMOE_EINVAL, "calibration set is null or empty");
      if (q > (int64_t)0x7fffffff / std::max(cfg->k_act, 1)) return fail(CMOE_EINVAL, "calibration set too large");
      for (int64_t i = 0; i < q * d; ++i)
        if (!std::isfinite(calib_x[i])) return fail(CMOE_EINVAL, "calibration token %lld has a non-finite entry", (long long)(i / d));
      if (cfg->k_act < 1 || cfg->k_act > d_ff) return fail(CMOE_EINVAL, "need 1 <= k_act <= d_ff");
      if (cfg->kmeans_iters < 1) return fail(CMOE_EINVAL, "kmeans_iters must be >= 1");
      if (cfg->dist_mode != 0 && cfg->dist_mode != 1) return fail(CMOE_EINVAL, "dist_mode must be 0 or 1");
      std::string msg;
      L->neuron_order.resize(d_ff);
      L->rep_neuron.resize(n_r);
      if (profile_on_gpu) {
        std::vector<int32_t> active((size_t)q * cfg->k_act);
        const int herr = gpu_profile(*cfg, rd, calib_x, q, active.data(), &msg);
        if (herr != 0)
          return fail(herr == (int)hipErrorInvalidValue ? CMOE_EINVAL : CMOE_EHIP, "GPU profiling failed: %s", msg.c_str());
        if (!host_construct_from_active(*cfg, q, active.data(), L->neuron_order.data(), L->rep_neuron.data(),
                                        L->mu.data(), &L->cost, &msg))
          return fail(CMOE_EINVAL, "construction failed: %s", msg.c_str());
      } else if (!host_construct(*cfg, rd, calib_x, q, L->neuron_order.data(), L->rep_neuron.data(), L->mu.data(),
                                 &L->cost, &msg)) {
        return fail(CMOE_EINVAL, "construction failed: %s", msg.c_str());
      }
    }
    // expert groups: one shared group of N_s*m neurons (if any), then the routed experts
    init_packed_set(L->moe, cfg->dtype, d);
    if (cfg->n_shared > 0) pack_group(L->moe, rd, L->neuron_order.data(), cfg->n_shared * m);
    for (int j = 0; j < n_r; ++j) pack_group(L->moe, rd, L->neuron_order.data() + (size_t)(cfg->n_shared + j) * m, m);
    // dense baseline: every neuron in its original order, one group, padded once
    init_packed_set(L->dense, cfg->dtype, d);
    std::vector<int32_t> ident(d_ff);
    for (int i = 0; i < d_ff; ++i) ident[i] = i;
    pack_group(L->dense, rd, ident.data(), d_ff);
    // router rows (Eq. 8)
    pack_router_rows(L->router, cfg->dtype, d, n_r);
    const size_t row_bytes = (size_t)d * elem_size(cfg->dtype);
    L->rep_rows.assign((size_t)n_r * 2 * row_bytes, 0);
    for (int j = 0; j < n_r; ++j) {
      set_router_rows(L->router, rd, j, L->rep_neuron[j]);
      std::memcpy(L->rep_rows.data() + (size_t)(2 * j) * row_bytes, rd.gate_row(L->rep_neuron[j]), row_bytes);
      std::memcpy(L->rep_rows.data() + (size_t)(2 * j + 1) * row_bytes, rd.up_row(L->rep_neuron[j]), row_bytes);
    }
    L->u.assign(n_r, 0.0f);
    L->b.assign(n_r, 0.0f);
    fill_flat_engines(L.get());
  } catch (const std::bad_alloc&) {
    return fail(CMOE_ENOMEM, "out of host memory while packing");
  } catch (const std::exception& ex) {
    return fail(CMOE_EINVAL, "internal error: %s", ex.what());
  } catch (...) {
    return fail(CMOE_EINVAL, "internal error");
  }
  *out = L.release();
  return CMOE_OK;
}

extern "C" {

int cmoe_build(const cmoe_config* cfg, const float* w_gate, const float* w_up, const float* w_down,
               const float* calib_x, int64_t q, cmoe_layer** out) {
  if (!calib_x) return fail(CMOE_EINVAL, "calib_x is null");
  return build_common(cfg, w_gate, w_up, w_down, calib_x, q, nullptr, nullptr, out);
}

int cmoe_build_gpu(const cmoe_config* cfg, const float* w_gate, const float* w_up, const float* w_down,
                   const float* calib_x, int64_t q, cmoe_layer** out) {
  if (!calib_x) return fail(CMOE_EINVAL, "calib_x is null");
  return build_common(cfg, w_gate, w_up, w_down, calib_x, q, nullptr, nullptr, out, true);
}

int cmoe_profile_activations(const cmoe_config* cfg, const float* w_gate, const float* w_up, const float* calib_x,
                             int64_t q, int on_gpu, int32_t* active_out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!w_gate || !w_up || !calib_x || !active_out) return fail(CMOE_EINVAL, "null argument");
  if (q < 1) return fail(CMOE_EINVAL, "calibration set is empty");
  if (cfg->k_act < 1 || cfg->k_act > cfg->d_ff) return fail(CMOE_EINVAL, "need 1 <= k_act <= d_ff");
  for (int64_t i = 0; i < q * cfg->d_model; ++i)
    if (!std::isfinite(calib_x[i])) return fail(CMOE_EINVAL, "calibration token %lld has a non-finite entry", (long long)(i / cfg->d_model));
  try {
    RoundedDense rd;
    rd.from_fp32(cfg->dtype, cfg->d_model, cfg->d_ff, w_gate, w_up, w_up);   // the down matrix plays no part here
    if (on_gpu) {
      std::string msg;
      const int herr = gpu_profile(*cfg, rd, calib_x, q, active_out, &msg);
      if (herr != 0)
        return fail(herr == (int)hipErrorInvalidValue ? CMOE_EINVAL : CMOE_EHIP, "GPU profiling failed: %s", msg.c_str());
    } else {
      host_profile(*cfg, rd, calib_x, q, active_out);
    }
  } catch (const std::bad_alloc&) {
    return fail(CMOE_ENOMEM, "out of host memory");
  } catch (const std::exception& ex) {
    return fail(CMOE_EINVAL, "internal error: %s", ex.what());
  } catch (...) {
    return fail(CMOE_EINVAL, "internal error");
  }
  return CMOE_OK;
}

int cmoe_balanced_assignment(const double* dist, int32_t n, int32_t n_r, int32_t m, int32_t* label_out,
                             double* cost_out) {
  if (!dist || !label_out) return fail(CMOE_EINVAL, "null argument");
  if (n < 1 || n_r < 1 || m < 1 || (int64_t)n_r * m != n) return fail(CMOE_EINVAL, "need n == n_r * m with positive sizes");
  std::string msg;
  try {
    if (!solve_balanced_assignment(dist, n, n_r, m, label_out, cost_out, &msg))
      return fail(CMOE_EINVAL, "%s", msg.c_str());
  } catch (const std::bad_alloc&) {
    return fail(CMOE_ENOMEM, "out of host memory");
  } catch (const std::exception& ex) {
    return fail(CMOE_EINVAL, "internal error: %s", ex.what());
  } catch (...) {
    return fail(CMOE_EINVAL, "internal error");
  }
  return CMOE_OK;
}

int cmoe_build_from_partition(const cmoe_config* cfg, const float* w_gate, const float* w_up, const float* w_down,
                              const int32_t* neuron_order, const int32_t* rep_neuron, cmoe_layer** out) {
  if (!neuron_order) return fail(CMOE_EINVAL, "neuron_order is null");
  return build_common(cfg, w_gate, w_up, w_down, nullptr, 0, neuron_order, rep_neuron, out);
}

int cmoe_export_partition(const cmoe_layer* L, int32_t* neuron_order, int32_t* rep_neuron, float* mu, double* cost) {
  if (!L) return fail(CMOE_EINVAL, "layer is null");
  if (neuron_order) std::memcpy(neuron_order, L->neuron_order.data(), sizeof(int32_t) * L->neuron_order.size());
  if (rep_neuron) std::memcpy(rep_neuron, L->rep_neuron.data(), sizeof(int32_t) * L->rep_neuron.size());
  if (mu) std::memcpy(mu, L->mu.data(), sizeof(float) * L->mu.size());
  if (cost) *cost = L->cost;
  return CMOE_OK;
}

int cmoe_set_gate_params(cmoe_layer* L, const float* u, const float* b) {
  if (!L) return fail(CMOE_EINVAL, "layer is null");
  if (L->in_hier) return fail(CMOE_ESTATE, "gate parameters of a layer inside a hierarchy must be set before cmoe_hier_create");
  L->has_u = u != nullptr;
  L->has_b = b != nullptr;
  for (int j = 0; j < L->n_r; ++j) {
    L->u[j] = u ? u[j] : 0.0f;
    L->b[j] = b ? b[j] : 0.0f;
  }
  L->e_moe.r.use_gate = (L->has_u || L->has_b) ? 1 : 0;
  if (L->uploaded) {
    // a forward still in flight on some stream may be reading the old values: wait for the device first
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(L->d_u, L->u.data(), sizeof(float) * L->n_r, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(L->d_b, L->b.data(), sizeof(float) * L->n_r, hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail_hip(e, "copying gate parameters");
  }
  return CMOE_OK;
}

int cmoe_get_gate_params(const cmoe_layer* L, float* u, float* b) {
  if (!L) return fail(CMOE_EINVAL, "layer is null");
  for (int j = 0; j < L->n_r; ++j) {
    if (u) u[j] = L->u[j];
    if (b) b[j] = L->b[j];
  }
  return CMOE_OK;
}

int cmoe_update_bias(cmoe_layer* L, const int32_t* counts, float gamma) {
  if (!L || !counts) return fail(CMOE_EINVAL, "null argument");
  if (!(gamma >= 0.0f)) return fail(CMOE_EINVAL, "gamma must be non-negative");
  int64_t total = 0;
  for (int j = 0; j < L->n_r; ++j) {
    if (counts[j] < 0) return fail(CMOE_EINVAL, "counts[%d] is negative", j);
    total += counts[j];
  }
  if (total == 0) return CMOE_OK;
  CMOE_TRY
  std::vector<float> b(L->b.begin(), L->b.begin() + L->n_r);
  for (int j = 0; j < L->n_r; ++j) {
    const int64_t c = (int64_t)counts[j] * L->n_r;       // p_j > 1/N_r  <=>  counts_j * N_r > total
    if (c > total) b[j] -= gamma;
    else if (c < total) b[j] += gamma;
  }
  std::vector<float> u(L->u.begin(), L->u.begin() + L->n_r);
  return cmoe_set_gate_params(L, L->has_u ? u.data() : nullptr, b.data());
  CMOE_CATCH
}

// device buffer of a flat layer: [moe W1][moe W2][dense W1][dense W2][router][moe groups][dense groups][u][b]
// [neuron-major routed W2][neuron norms][router in operand order]
static bool router_tiled_ok(const cmoe_layer* L) {
  const int d = L->cfg.d_model;
  return L->cfg.dtype == CMOE_BF16 && d % 256 == 0 && !L->router.empty() && (L->router.size() / ((size_t)d * 2)) % 16 == 0;
}
struct FlatOffsets { size_t w1, w2, dw1, dw2, wr, g, dg, u, b, w2n, nscale, wrt, total; };
static FlatOffsets flat_offsets(const cmoe_layer* L) {
  FlatOffsets o{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t r = off; off = align256(off + bytes); return r; };
  o.w1 = take(L->moe.w1.size());
  o.w2 = take(L->moe.w2.size());
  o.dw1 = take(L->baseline ? L->dense.w1.size() : 0);
  o.dw2 = take(L->baseline ? L->dense.w2.size() : 0);
  o.wr = take(L->router.size());
  o.g = take(sizeof(GroupDev) * L->moe.groups.size());
  o.dg = take(L->baseline ? sizeof(GroupDev) * L->dense.groups.size() : 0);
  o.u = take(sizeof(float) * L->n_r);
  o.b = take(sizeof(float) * L->n_r);
  o.w2n = take(L->sparse_reserved ? L->w2n.size() : 0);
  o.nscale = take(L->sparse_reserved ? sizeof(float) * L->nscale.size() : 0);
  o.wrt = take(router_tiled_ok(L) ? L->router.size() : 0);
  o.total = off;
  return o;
}

// Second copy of a bf16 router in the MFMA operand order of the one-token front end: the 1 KB that one wave
// loads as an A operand (16 rows x 32 columns; lane = (column / 8) * 16 + row holds 8 consecutive columns) is
// consecutive memory, [row block][K step][lane][8].  In the row-major matrix the 16 rows of an operand lie a
// power of two apart and meet in one L2 channel, which does not matter for the one scoring launch that reads
// the matrix once but does when hundreds of workgroups read it at the same time.
static std::vector<uint8_t> tile_router_rows(const std::vector<uint8_t>& rows, int d) {
  const size_t n_rows = rows.size() / ((size_t)d * 2);
  std::vector<uint8_t> out(rows.size());
  const uint16_t* src = reinterpret_cast<const uint16_t*>(rows.data());
  uint16_t* dst = reinterpret_cast<uint16_t*>(out.data());
  const int ksteps = d / 32;
  for (size_t rb = 0; rb < n_rows / 16; ++rb)
    for (int kk = 0; kk < ksteps; ++kk)
      for (int lane = 0; lane < 64; ++lane) {
        const size_t row = rb * 16 + (lane & 15);
        const int col = kk * 32 + (lane >> 4) * 8;
        std::memcpy(dst + ((rb * ksteps + kk) * 64 + lane) * 8, src + row * d + col, 16);
      }
  return out;
}

size_t cmoe_packed_bytes(const cmoe_layer* L) { return L ? flat_offsets(L).total : 0; }

int cmoe_set_neuron_sparsity(cmoe_layer* L, int mode, float tau) {
  if (!L) return fail(CMOE_EINVAL, "layer is null");
  if (mode < 0 || mode > 2) return fail(CMOE_EINVAL, "mode must be 0 (off), 1 (magnitude) or 2 (weight-informed)");
  if (mode != 0 && !(tau >= 0.0f)) return fail(CMOE_EINVAL, "tau must be a non-negative number");
  if (mode == 0) {
    L->sparse_mode = 0;
    return CMOE_OK;
  }
  if (L->in_hier) return fail(CMOE_ESTATE, "neuron-level sparsity is not available for layers inside a hierarchy");
  if (L->cfg.dtype != CMOE_BF16) return fail(CMOE_EINVAL, "neuron-level sparsity needs a bf16 layer");
  if (!L->sparse_reserved) {
    if (L->uploaded) return fail(CMOE_ESTATE, "the first cmoe_set_neuron_sparsity must come before cmoe_upload (it adds a "
                                 "neuron-major copy of the routed down matrices to the packed weights)");
    CMOE_TRY
    const PackedSet& ps = L->moe;
    const int d = L->cfg.d_model;
    const int first = L->cfg.n_shared > 0 ? 1 : 0;
    int64_t total_wp = 0, routed_wp = 0;
    for (size_t g = 0; g < ps.groups.size(); ++g) {
      total_wp += ps.groups[g].width_pad;
      if ((int)g >= first) routed_wp += ps.groups[g].width_pad;
    }
    L->nscale.assign((size_t)total_wp, 0.0f);
    L->w2n.assign((size_t)routed_wp * d * 2, 0);
    const uint16_t* w2 = reinterpret_cast<const uint16_t*>(ps.w2.data());
    uint16_t* out = reinterpret_cast<uint16_t*>(L->w2n.data());
    const int64_t routed_row0 = ps.groups[first].w1_row0 / 2;
    for (size_t g = 0; g < ps.groups.size(); ++g) {
      const GroupDev& gd = ps.groups[g];
      const int wp = gd.width_pad, kt2 = wp / TILE_K;
      const int64_t n0 = gd.w1_row0 / 2;
      parallel_for(wp, [&](int64_t n) {
        double ss = 0.0;
        for (int c = 0; c < d; ++c) {
          const uint16_t v = w2[gd.w2_off + tiled_offset(c, (int)n, kt2)];
          const double f = (double)host_bf16_to_f32(v);
          ss += f * f;
          if ((int)g >= first) out[(size_t)(n0 - routed_row0 + n) * d + c] = v;
        }
        L->nscale[(size_t)(n0 + n)] = (float)std::sqrt(ss);
      });
    }
    L->sparse_reserved = true;
    CMOE_CATCH
  }
  L->sparse_mode = mode;
  L->sparse_tau = tau;
  return CMOE_OK;
}

size_t cmoe_workspace_bytes(const cmoe_layer* L, int64_t max_tokens) {
  if (!L || max_tokens < 0) return 0;
  const size_t moe = ws_layout(L->e_moe, max_tokens).total;
  return L->baseline ? std::max(moe, ws_layout(L->e_dense, max_tokens).total) : moe;
}

int cmoe_set_baseline(cmoe_layer* L, int enabled) {
  if (!L) return fail(CMOE_EINVAL, "layer is null");
  if (L->uploaded || L->in_hier) return fail(CMOE_ESTATE, "cmoe_set_baseline must come before cmoe_upload / cmoe_hier_create");
  if (enabled && !L->baseline) return fail(CMOE_ESTATE, "the dense copy of this layer has been released");
  if (!enabled && L->baseline) {
    L->baseline = false;
    std::vector<uint8_t>().swap(L->dense.w1);       // release the host copy: it is never uploaded
    std::vector<uint8_t>().swap(L->dense.w2);
  }
  return CMOE_OK;
}

static hipError_t h2d(void* dst, const void* src, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  return hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, s);
}

int cmoe_upload(cmoe_layer* L, void* dev_weights, void* hip_stream) {
  if (!L || !dev_weights) return fail(CMOE_EINVAL, "layer or device buffer is null");
  if (L->in_hier) return fail(CMOE_ESTATE, "layer belongs to a hierarchy; upload the hierarchy instead");
  if (((uintptr_t)dev_weights & 255) != 0) return fail(CMOE_EINVAL, "device weight buffer must be 256-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const FlatOffsets o = flat_offsets(L);
  char* base = static_cast<char*>(dev_weights);
  hipError_t e = h2d(base + o.w1, L->moe.w1.data(), L->moe.w1.size(), s);
  if (e == hipSuccess) e = h2d(base + o.w2, L->moe.w2.data(), L->moe.w2.size(), s);
  if (e == hipSuccess && L->baseline) e = h2d(base + o.dw1, L->dense.w1.data(), L->dense.w1.size(), s);
  if (e == hipSuccess && L->baseline) e = h2d(base + o.dw2, L->dense.w2.data(), L->dense.w2.size(), s);
  if (e == hipSuccess) e = h2d(base + o.wr, L->router.data(), L->router.size(), s);
  if (e == hipSuccess) e = h2d(base + o.g, L->moe.groups.data(), sizeof(GroupDev) * L->moe.groups.size(), s);
  if (e == hipSuccess && L->baseline) e = h2d(base + o.dg, L->dense.groups.data(), sizeof(GroupDev) * L->dense.groups.size(), s);
  if (e == hipSuccess) e = h2d(base + o.u, L->u.data(), sizeof(float) * L->n_r, s);
  if (e == hipSuccess) e = h2d(base + o.b, L->b.data(), sizeof(float) * L->n_r, s);
  if (e == hipSuccess && L->sparse_reserved) e = h2d(base + o.w2n, L->w2n.data(), L->w2n.size(), s);
  if (e == hipSuccess && L->sparse_reserved) e = h2d(base + o.nscale, L->nscale.data(), sizeof(float) * L->nscale.size(), s);
  std::vector<uint8_t> wrt;                      // (alive until the stream has been synchronised)
  if (e == hipSuccess && router_tiled_ok(L)) {
    wrt = tile_router_rows(L->router, L->cfg.d_model);
    e = h2d(base + o.wrt, wrt.data(), wrt.size(), s);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail_hip(e, "uploading packed weights");
  Engine& m = L->e_moe;
  m.wr_tiled = router_tiled_ok(L) ? base + o.wrt : nullptr;
  m.w2n = L->sparse_reserved ? base + o.w2n : nullptr;
  m.nscale = L->sparse_reserved ? reinterpret_cast<const float*>(base + o.nscale) : nullptr;
  m.w1 = base + o.w1;
  m.w2 = base + o.w2;
  m.wr = base + o.wr;
  m.groups = reinterpret_cast<const GroupDev*>(base + o.g);
  L->d_u = reinterpret_cast<float*>(base + o.u);
  L->d_b = reinterpret_cast<float*>(base + o.b);
  m.gate_u = L->d_u;
  m.gate_b = L->d_b;
  Engine& dn = L->e_dense;
  dn.w1 = base + o.dw1;
  dn.w2 = base + o.dw2;
  dn.groups = reinterpret_cast<const GroupDev*>(base + o.dg);
  L->uploaded = true;
  return CMOE_OK;
}

static int run_engine(const Engine& e, const void* x, int64_t T, void* y, int32_t* topk, int32_t* outer,
                      float* scores, int32_t* counts, void* ws, size_t ws_bytes, hipStream_t s,
                      hipEvent_t* ev = nullptr, size_t splitk_cap = ~(size_t)0) {
  if (T < 0) return fail(CMOE_EINVAL, "negative token count");
  if (T == 0) return CMOE_OK;
  if (!x || !y || !ws) return fail(CMOE_EINVAL, "x, y or workspace is null");
  if (T * (int64_t)e.S_all() > (int64_t)0x7fffffff / 2) return fail(CMOE_EINVAL, "batch too large for 32-bit slot indices");
  WsLayout L = ws_layout(e, T, splitk_cap);
  if (ws_bytes < L.total) return fail(CMOE_EINVAL, "workspace too small: %zu bytes given, %zu needed", ws_bytes, L.total);
  if (((uintptr_t)ws & 255) != 0) return fail(CMOE_EINVAL, "workspace must be 256-byte aligned");
  char* w = static_cast<char*>(ws);
  const bool single = (e.G == 1 && e.n_always == 1);
  hipError_t err = hipSuccess;
  auto mark = [&](int i) { if (ev) (void)hipEventRecord(ev[i], s); };
  // decode batches: scoring is one kernel, selection + permutation a second one
  const bool front = !single && !use_simt_experts(e.dtype) && decode_front_ok(e, T);
  L.skip_always = (front && decode_front_runs_shared(e, T)) ? 1 : 0;
  L.gate_up_done = (front && decode_front_runs_all(e, T)) ? 1 : 0;
  mark(0);
  if (!single) {
    err = front ? launch_decode_front(e, x, T, w, L, topk, outer, scores, counts, s)
                : launch_router(e, x, T, w, L, topk, outer, scores, s);
    if (err != hipSuccess) return fail_hip(err, "router kernel");
  }
  mark(1);
  if (front && tuning().skip_stage == 6) return CMOE_OK;   // (measurement aid: nothing after the scoring launch)
  if (!single && !front) {
    err = launch_permute(e, T, w, L, counts, s);
    if (err != hipSuccess) return fail_hip(err, "permute kernel");
  }
  mark(2);
  // (skip: measurement aid, see Tuning::skip_stage; only launches that produce no control data can be left out)
  const int skip = tuning().skip_stage, twice = tuning().repeat_stage;
  for (int n = ((skip == 3 || L.gate_up_done) ? 0 : twice == 3 ? 2 : 1); n > 0 && err == hipSuccess; --n) err = launch_experts(e, x, T, w, L, y, s, 1);
  if (err == hipSuccess && e.sparse_mode != 0 && !decode_sparse_down_ok(e, T)) err = launch_mask_hidden(e, T, w, L, s);
  if (err != hipSuccess) return fail_hip(err, "gate/up expert kernel");
  mark(3);
  for (int n = (skip == 4 ? 0 : twice == 4 ? 2 : 1); n > 0 && err == hipSuccess; --n) err = launch_experts(e, x, T, w, L, y, s, 2);
  if (err != hipSuccess) return fail_hip(err, "down expert kernel");
  mark(4);
  for (int n = (skip == 5 ? 0 : twice == 5 ? 2 : 1); n > 0 && err == hipSuccess; --n) err = launch_combine(e, T, w, L, y, s);
  if (err != hipSuccess) return fail_hip(err, "combine kernel");
  mark(5);
  return CMOE_OK;
}

// Timed variant shared by the two *_forward_timed entry points: five stages bracketed by six events.
static int run_engine_timed(const Engine& e, const void* x, int64_t T, void* y, void* ws, size_t ws_bytes,
                            hipStream_t s, float* stage_ms) {
  if (!stage_ms) return fail(CMOE_EINVAL, "stage_ms is null");
  hipEvent_t ev[6];
  for (int i = 0; i < 6; ++i) {
    hipError_t err = hipEventCreate(&ev[i]);
    if (err != hipSuccess) return fail_hip(err, "hipEventCreate");
  }
  int rc = run_engine(e, x, T, y, nullptr, nullptr, nullptr, nullptr, ws, ws_bytes, s, ev);
  if (rc == CMOE_OK && T > 0) {
    hipError_t err = hipEventSynchronize(ev[5]);
    if (err != hipSuccess) rc = fail_hip(err, "hipEventSynchronize");
    for (int i = 0; i < 5 && rc == CMOE_OK; ++i) {
      err = hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]);
      if (err != hipSuccess) rc = fail_hip(err, "hipEventElapsedTime");
    }
  } else {
    for (int i = 0; i < 5; ++i) stage_ms[i] = 0.0f;
  }
  for (int i = 0; i < 6; ++i) (void)hipEventDestroy(ev[i]);
  return rc;
}

int cmoe_forward(cmoe_layer* L, const void* x_dev, int64_t T, void* y_dev, int32_t* topk_idx_dev,
                 float* scores_dev, int32_t* counts_dev, void* workspace_dev, size_t workspace_bytes,
                 void* hip_stream) {
  if (!L) return fail(CMOE_EINVAL, "layer is null");
  if (!L->uploaded) return fail(CMOE_ESTATE, "cmoe_upload has not been called");
  Engine e = L->e_moe;
  if (!L->has_u) e.gate_u = nullptr;
  if (!L->has_b) e.gate_b = nullptr;
  e.sparse_mode = L->sparse_reserved ? L->sparse_mode : 0;
  e.sparse_tau = L->sparse_tau;
  return run_engine(e, x_dev, T, y_dev, topk_idx_dev, nullptr, scores_dev, counts_dev, workspace_dev,
                    workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

// ---- the forward for callers that cannot allocate: its workspace is a static device array ----------------
// Each GPU the library runs on holds its own copy of the array from the moment the code object is loaded
// until the process ends.  In host code the array's name is only a stand-in: the device address of the
// copy on the current device comes from hipGetSymbolAddress, once per device, and only that pointer is ever
// handed to a kernel.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)32 << 20;
constexpr size_t STATIC_SPLITK_CAP = (size_t)8 << 20;
constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

static int static_scratch_ptr(void** out) {
  static std::mutex mu;
  static void* ptr_of_device[STATIC_MAX_DEVICES] = {nullptr};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return fail(CMOE_EINVAL, "device index %d is outside the table of %d devices", dev, STATIC_MAX_DEVICES);
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress(scratch)");
    if (!p || ((uintptr_t)p & 255) != 0) return fail(CMOE_EHIP, "static scratch array has no usable device address");
    ptr_of_device[dev] = p;
  }
  *out = ptr_of_device[dev];
  return CMOE_OK;
}

size_t cmoe_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int64_t cmoe_forward_static_max_tokens(const cmoe_layer* L) {
  if (!L) return 0;
  int64_t lo = 0, hi = 1 << 20;            // the layout grows with T: bisect the largest batch that fits
  while (lo < hi) {
    const int64_t mid = (lo + hi + 1) / 2;
    if (ws_layout(L->e_moe, mid, STATIC_SPLITK_CAP).total <= STATIC_SCRATCH_BYTES) lo = mid;
    else hi = mid - 1;
  }
  return lo;
}

int cmoe_forward_static(cmoe_layer* L, const void* x_dev, int64_t T, void* y_dev, int32_t* topk_idx_dev,
                        float* scores_dev, int32_t* counts_dev, void* hip_stream) {
  if (!L) return fail(CMOE_EINVAL, "layer is null");
  if (!L->uploaded) return fail(CMOE_ESTATE, "cmoe_upload has not been called");
  if (T < 0) return fail(CMOE_EINVAL, "negative token count");
  if (T == 0) return CMOE_OK;
  const size_t need = ws_layout(L->e_moe, T, STATIC_SPLITK_CAP).total;
  if (need > STATIC_SCRATCH_BYTES)
    return fail(CMOE_EINVAL, "batch of %lld tokens needs %zu bytes of workspace, the static scratch array holds %zu "
                "(at most %lld tokens for this layer): use cmoe_forward with a workspace of your own",
                (long long)T, need, STATIC_SCRATCH_BYTES, (long long)cmoe_forward_static_max_tokens(L));
  void* ws = nullptr;
  const int rc = static_scratch_ptr(&ws);
  if (rc) return rc;
  Engine e = L->e_moe;
  if (!L->has_u) e.gate_u = nullptr;
  if (!L->has_b) e.gate_b = nullptr;
  e.sparse_mode = L->sparse_reserved ? L->sparse_mode : 0;
  e.sparse_tau = L->sparse_tau;
  return run_engine(e, x_dev, T, y_dev, topk_idx_dev, nullptr, scores_dev, counts_dev, ws, STATIC_SCRATCH_BYTES,
                    static_cast<hipStream_t>(hip_stream), nullptr, STATIC_SPLITK_CAP);
}

int cmoe_dense_forward(cmoe_layer* L, const void* x_dev, int64_t T, void* y_dev, void* workspace_dev,
                       size_t workspace_bytes, void* hip_stream) {
  if (!L) return fail(CMOE_EINVAL, "layer is null");
  if (!L->uploaded) return fail(CMOE_ESTATE, "cmoe_upload has not been called");
  if (!L->baseline) return fail(CMOE_ESTATE, "the layer was uploaded without its dense baseline (cmoe_set_baseline)");
  return run_engine(L->e_dense, x_dev, T, y_dev, nullptr, nullptr, nullptr, nullptr, workspace_dev, workspace_bytes,
                    static_cast<hipStream_t>(hip_stream));
}

int cmoe_forward_timed(cmoe_layer* L, int dense, const void* x_dev, int64_t T, void* y_dev, void* workspace_dev,
                       size_t workspace_bytes, void* hip_stream, float* stage_ms) {
  if (!L) return fail(CMOE_EINVAL, "layer is null");
  if (!L->uploaded) return fail(CMOE_ESTATE, "cmoe_upload has not been called");
  if (dense && !L->baseline) return fail(CMOE_ESTATE, "the layer was uploaded without its dense baseline (cmoe_set_baseline)");
  Engine e = dense ? L->e_dense : L->e_moe;
  if (!L->has_u) e.gate_u = nullptr;
  if (!L->has_b) e.gate_b = nullptr;
  if (!dense) {
    e.sparse_mode = L->sparse_reserved ? L->sparse_mode : 0;
    e.sparse_tau = L->sparse_tau;
  }
  return run_engine_timed(e, x_dev, T, y_dev, workspace_dev, workspace_bytes, static_cast<hipStream_t>(hip_stream), stage_ms);
}

void cmoe_destroy(cmoe_layer* L) { delete L; }

// ---------------------------------------------------------------------------------- hierarchy
int cmoe_hier_create(cmoe_layer* const* experts, int32_t n_outer, int32_t outer_top_k, const float* w_router,
                     const float* logit_offset, cmoe_hier** out) {
  if (!experts || !w_router || !out) return fail(CMOE_EINVAL, "null argument");
  if (n_outer < 1 || n_outer > IL) return fail(CMOE_EINVAL, "need 1 <= n_outer <= %d", IL);
  if (outer_top_k < 1 || outer_top_k > n_outer || outer_top_k > MAX_OUTER_TOPK) return fail(CMOE_EINVAL, "bad outer_top_k");
  for (int e = 0; e < n_outer; ++e) {
    if (!experts[e]) return fail(CMOE_EINVAL, "expert %d is null", e);
    if (experts[e]->uploaded || experts[e]->in_hier) return fail(CMOE_ESTATE, "expert %d is already uploaded or owned", e);
    if (std::memcmp(&experts[e]->cfg, &experts[0]->cfg, sizeof(cmoe_config)) != 0)
      return fail(CMOE_EINVAL, "expert %d has a different configuration", e);
    if (experts[e]->sparse_mode != 0) return fail(CMOE_EINVAL, "expert %d has neuron-level sparsity switched on", e);
    if (experts[e]->baseline != experts[0]->baseline)
      return fail(CMOE_EINVAL, "expert %d differs from expert 0 in cmoe_set_baseline", e);
  }
  const cmoe_config& c = experts[0]->cfg;
  const int n_r = c.n_experts - c.n_shared;
  const int has_shared = c.n_shared > 0 ? 1 : 0;
  if (n_outer * n_r > MAX_SCORED) return fail(CMOE_EINVAL, "n_outer * N_r = %d exceeds %d scored experts", n_outer * n_r, MAX_SCORED);
  if (outer_top_k * (has_shared + c.top_k) > MAX_DYN) return fail(CMOE_EINVAL, "too many slots per token");
  if (n_outer * (has_shared + n_r) > MAX_GROUPS) return fail(CMOE_EINVAL, "too many expert groups");
  std::unique_ptr<cmoe_hier> H(new (std::nothrow) cmoe_hier());
  if (!H) return fail(CMOE_ENOMEM, "out of host memory");
  try {
    H->experts.assign(experts, experts + n_outer);
    H->cfg = c;
    H->n_outer = n_outer;
    H->outer_top_k = outer_top_k;
    H->baseline = experts[0]->baseline;
    const int d = c.d_model;
    const size_t es = elem_size(c.dtype), row_bytes = (size_t)d * es;
    pack_router_rows(H->router, c.dtype, d, n_outer * n_r);
    for (int e = 0; e < n_outer; ++e)
      for (int j = 0; j < n_r; ++j) {
        const int idx = e * n_r + j, blk = idx / IL, cc = idx % IL;
        std::memcpy(H->router.data() + ((size_t)blk * 2 * IL + cc) * row_bytes,
                    experts[e]->rep_rows.data() + (size_t)(2 * j) * row_bytes, row_bytes);
        std::memcpy(H->router.data() + ((size_t)blk * 2 * IL + IL + cc) * row_bytes,
                    experts[e]->rep_rows.data() + (size_t)(2 * j + 1) * row_bytes, row_bytes);
      }
    H->lin_rows.assign((size_t)IL * row_bytes, 0);
    for (int e = 0; e < n_outer; ++e)
      for (int k = 0; k < d; ++k) store_elem(H->lin_rows.data() + ((size_t)e * d + k) * es, c.dtype, w_router[(size_t)k * n_outer + e]);
    H->lin_off.assign(n_outer, 0.0f);
    if (logit_offset) H->lin_off.assign(logit_offset, logit_offset + n_outer);
    // engines
    Engine& m = H->e_moe;
    m = Engine{};
    m.dtype = c.dtype;
    m.d = d;
    m.ldw1 = experts[0]->moe.ld;
    m.w_tiled = experts[0]->moe.tiled ? 1 : 0;
    const int gpo = has_shared + n_r;
    m.G = n_outer * gpo;
    m.n_always = 0;
    m.S_dyn = outer_top_k * (has_shared + c.top_k);
    for (int e = 0; e < n_outer; ++e)
      for (int g = 0; g < gpo; ++g) {
        const int wp = experts[e]->moe.groups[g].width_pad;
        m.width_pad_host[e * gpo + g] = wp;
        m.max_width_pad = std::max(m.max_width_pad, wp);
      }
    m.h_per_token = (int64_t)outer_top_k * ((has_shared ? experts[0]->moe.groups[0].width_pad : 0) +
                                            (int64_t)c.top_k * experts[0]->moe.groups[gpo - 1].width_pad);
    RouterDev& r = m.r;
    r.n_scored = n_outer * n_r;
    r.n_sw_rows = 2 * IL * cdiv(n_outer * n_r, IL);
    r.n_lin = n_outer;
    r.n_lin_rows = IL;
    r.top_k = c.top_k;
    r.outer_top_k = outer_top_k;
    r.n_r_sub = n_r;
    r.n_always = 0;
    r.score_abs = c.score_mode;
    r.use_gate = 0;
    for (int e = 0; e < n_outer; ++e) r.use_gate |= (experts[e]->has_u || experts[e]->has_b) ? 1 : 0;
    r.groups_per_outer = gpo;
    r.sub_has_shared = has_shared;
    Engine& dn = H->e_dense;
    dn = Engine{};
    dn.dtype = c.dtype;
    dn.d = d;
    dn.ldw1 = experts[0]->dense.ld;
    dn.w_tiled = experts[0]->dense.tiled ? 1 : 0;
    dn.G = n_outer;
    dn.n_always = 0;
    dn.S_dyn = outer_top_k;
    for (int e = 0; e < n_outer; ++e) dn.width_pad_host[e] = experts[e]->dense.groups[0].width_pad;
    dn.max_width_pad = dn.width_pad_host[0];
    dn.h_per_token = (int64_t)outer_top_k * dn.width_pad_host[0];
    dn.r = RouterDev{};
    dn.r.n_lin = n_outer;
    dn.r.n_lin_rows = IL;
    dn.r.outer_top_k = outer_top_k;
    dn.r.groups_per_outer = 1;
    dn.r.sub_has_shared = 1;
    for (int e = 0; e < n_outer; ++e) experts[e]->in_hier = true;
  } catch (const std::bad_alloc&) {
    return fail(CMOE_ENOMEM, "out of host memory");
  } catch (const std::exception& ex) {
    return fail(CMOE_EINVAL, "internal error: %s", ex.what());
  } catch (...) {
    return fail(CMOE_EINVAL, "internal error");
  }
  *out = H.release();
  return CMOE_OK;
}

// Sec. 4.4 end to end: route the calibration tokens through the outer router on the host, restructure every
// outer expert on the tokens that reach it, and tie the results together.
int cmoe_hier_build(const cmoe_config* cfg, int32_t n_outer, int32_t outer_top_k, const float* const* w_gate,
                    const float* const* w_up, const float* const* w_down, const float* w_router,
                    const float* logit_offset, const float* calib_x, int64_t q, int32_t min_tokens, int on_gpu,
                    int with_baseline, cmoe_hier** out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!w_gate || !w_up || !w_down || !w_router || !calib_x || !out) return fail(CMOE_EINVAL, "null argument");
  if (n_outer < 1 || n_outer > IL) return fail(CMOE_EINVAL, "need 1 <= n_outer <= %d", IL);
  if (outer_top_k < 1 || outer_top_k > n_outer || outer_top_k > MAX_OUTER_TOPK) return fail(CMOE_EINVAL, "bad outer_top_k");
  if (q < 1) return fail(CMOE_EINVAL, "calibration set is empty");
  for (int e = 0; e < n_outer; ++e)
    if (!w_gate[e] || !w_up[e] || !w_down[e]) return fail(CMOE_EINVAL, "weights of outer expert %d are null", e);
  const int d = cfg->d_model;
  const int64_t need = std::max<int64_t>(min_tokens > 0 ? min_tokens : 64, cfg->k_act);
  std::vector<cmoe_layer*> layers;
  auto drop = [&]() { for (cmoe_layer* L : layers) delete L; };
  CMOE_TRY
  // outer routing of the calibration tokens: logits in double precision on the dtype-rounded operands,
  // top-k with ties to the lowest expert id (the same rule as the forward)
  auto rnd = [&](float v) { return cfg->dtype == CMOE_BF16 ? host_bf16_to_f32(host_f32_to_bf16(v)) : v; };
  std::vector<double> wr((size_t)d * n_outer);
  for (size_t i = 0; i < wr.size(); ++i) wr[i] = (double)rnd(w_router[i]);
  std::vector<std::vector<int64_t>> rows(n_outer);
  for (int64_t t = 0; t < q; ++t) {
    double logit[IL];
    for (int e = 0; e < n_outer; ++e) logit[e] = logit_offset ? (double)logit_offset[e] : 0.0;
    for (int k = 0; k < d; ++k) {
      const float xv = calib_x[(size_t)t * d + k];
      if (!std::isfinite(xv)) return fail(CMOE_EINVAL, "calibration token %lld has a non-finite entry", (long long)t);
      const double x = (double)rnd(xv);
      for (int e = 0; e < n_outer; ++e) logit[e] += x * wr[(size_t)k * n_outer + e];
    }
    uint32_t taken = 0u;
    for (int i = 0; i < outer_top_k; ++i) {
      int best = -1;
      for (int e = 0; e < n_outer; ++e)
        if (((taken >> e) & 1u) == 0u && (best < 0 || logit[e] > logit[best])) best = e;
      taken |= 1u << best;
      rows[best].push_back(t);
    }
  }
  for (int e = 0; e < n_outer; ++e) {
    const std::vector<int64_t>& r = rows[e];
    const bool whole = (int64_t)r.size() < need;
    const int64_t n_e = whole ? q : (int64_t)r.size();
    std::vector<float> xs;
    if (!whole) {
      xs.resize((size_t)n_e * d);
      for (int64_t i = 0; i < n_e; ++i) std::memcpy(&xs[(size_t)i * d], calib_x + (size_t)r[i] * d, sizeof(float) * d);
    }
    cmoe_layer* L = nullptr;
    rc = build_common(cfg, w_gate[e], w_up[e], w_down[e], whole ? calib_x : xs.data(), n_e, nullptr, nullptr, &L, on_gpu != 0);
    if (rc) {
      drop();
      return rc;
    }
    L->calib_routed = (int64_t)r.size();
    L->calib_used = n_e;
    layers.push_back(L);
    if (!with_baseline) (void)cmoe_set_baseline(L, 0);
  }
  cmoe_hier* H = nullptr;
  rc = cmoe_hier_create(layers.data(), n_outer, outer_top_k, w_router, logit_offset, &H);
  if (rc) {
    drop();
    return rc;
  }
  H->owns_experts = true;
  *out = H;
  return CMOE_OK;
  }
  catch (const std::bad_alloc&) { drop(); return fail(CMOE_ENOMEM, "out of host memory"); }
  catch (const std::exception& ex) { drop(); return fail(CMOE_EINVAL, "internal error: %s", ex.what()); }
  catch (...) { drop(); return fail(CMOE_EINVAL, "internal error"); }
}

const cmoe_layer* cmoe_hier_expert(const cmoe_hier* H, int32_t e, int64_t* calib_routed, int64_t* calib_used) {
  if (!H || e < 0 || e >= H->n_outer) {
    (void)fail(CMOE_EINVAL, "no such outer expert");
    return nullptr;
  }
  if (calib_routed) *calib_routed = H->experts[e]->calib_routed;
  if (calib_used) *calib_used = H->experts[e]->calib_used;
  return H->experts[e];
}

// device buffer of a hierarchy:
// [moe W1 of all experts][moe W2 ...][dense W1 ...][dense W2 ...][router sw rows][lin rows][moe groups][dense groups][u][b][offsets]
struct HierOffsets { size_t w1, w2, dw1, dw2, wr, g, dg, u, b, off, total; };
static HierOffsets hier_offsets(const cmoe_hier* H) {
  HierOffsets o{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t r = off; off = align256(off + bytes); return r; };
  size_t w1 = 0, w2 = 0, dw1 = 0, dw2 = 0;
  for (auto* L : H->experts) {
    w1 += L->moe.w1.size();
    w2 += L->moe.w2.size();
    if (H->baseline) { dw1 += L->dense.w1.size(); dw2 += L->dense.w2.size(); }
  }
  o.w1 = take(w1);
  o.w2 = take(w2);
  o.dw1 = take(dw1);
  o.dw2 = take(dw2);
  o.wr = take(H->router.size() + H->lin_rows.size());
  o.g = take(sizeof(GroupDev) * H->e_moe.G);
  o.dg = take(sizeof(GroupDev) * H->e_dense.G);
  o.u = take(sizeof(float) * std::max(H->e_moe.r.n_scored, 1));
  o.b = take(sizeof(float) * std::max(H->e_moe.r.n_scored, 1));
  o.off = take(sizeof(float) * H->n_outer);
  o.total = off;
  return o;
}

size_t cmoe_hier_packed_bytes(const cmoe_hier* H) { return H ? hier_offsets(H).total : 0; }

size_t cmoe_hier_workspace_bytes(const cmoe_hier* H, int64_t max_tokens) {
  if (!H || max_tokens < 0) return 0;
  const size_t moe = ws_layout(H->e_moe, max_tokens).total;
  return H->baseline ? std::max(moe, ws_layout(H->e_dense, max_tokens).total) : moe;
}

int cmoe_hier_upload(cmoe_hier* H, void* dev_weights, void* hip_stream) {
  if (!H || !dev_weights) return fail(CMOE_EINVAL, "hierarchy or device buffer is null");
  if (((uintptr_t)dev_weights & 255) != 0) return fail(CMOE_EINVAL, "device weight buffer must be 256-byte aligned");
  CMOE_TRY
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const HierOffsets o = hier_offsets(H);
  char* base = static_cast<char*>(dev_weights);
  const size_t es = elem_size(H->cfg.dtype);
  std::vector<GroupDev> g_moe, g_dense;
  std::vector<float> u, b;
  size_t w1 = 0, w2 = 0, dw1 = 0, dw2 = 0;
  hipError_t e = hipSuccess;
  for (auto* L : H->experts) {
    const int64_t row_shift = (int64_t)(w1 / ((size_t)L->moe.ld * es));
    const int64_t el_shift = (int64_t)(w2 / es);
    for (const GroupDev& gd : L->moe.groups) g_moe.push_back(GroupDev{gd.width_pad, (int32_t)(gd.w1_row0 + row_shift), gd.w2_off + el_shift});
    const int64_t drow_shift = (int64_t)(dw1 / ((size_t)L->dense.ld * es));
    const int64_t del_shift = (int64_t)(dw2 / es);
    for (const GroupDev& gd : L->dense.groups) g_dense.push_back(GroupDev{gd.width_pad, (int32_t)(gd.w1_row0 + drow_shift), gd.w2_off + del_shift});
    if (e == hipSuccess) e = h2d(base + o.w1 + w1, L->moe.w1.data(), L->moe.w1.size(), s);
    if (e == hipSuccess) e = h2d(base + o.w2 + w2, L->moe.w2.data(), L->moe.w2.size(), s);
    if (e == hipSuccess && H->baseline) e = h2d(base + o.dw1 + dw1, L->dense.w1.data(), L->dense.w1.size(), s);
    if (e == hipSuccess && H->baseline) e = h2d(base + o.dw2 + dw2, L->dense.w2.data(), L->dense.w2.size(), s);
    w1 += L->moe.w1.size();
    w2 += L->moe.w2.size();
    if (H->baseline) {
      dw1 += L->dense.w1.size();
      dw2 += L->dense.w2.size();
    }
    u.insert(u.end(), L->u.begin(), L->u.end());
    b.insert(b.end(), L->b.begin(), L->b.end());
  }
  if (e == hipSuccess) e = h2d(base + o.wr, H->router.data(), H->router.size(), s);
  if (e == hipSuccess) e = h2d(base + o.wr + H->router.size(), H->lin_rows.data(), H->lin_rows.size(), s);
  if (e == hipSuccess) e = h2d(base + o.g, g_moe.data(), sizeof(GroupDev) * g_moe.size(), s);
  if (e == hipSuccess) e = h2d(base + o.dg, g_dense.data(), sizeof(GroupDev) * g_dense.size(), s);
  if (e == hipSuccess) e = h2d(base + o.u, u.data(), sizeof(float) * u.size(), s);
  if (e == hipSuccess) e = h2d(base + o.b, b.data(), sizeof(float) * b.size(), s);
  if (e == hipSuccess) e = h2d(base + o.off, H->lin_off.data(), sizeof(float) * H->lin_off.size(), s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail_hip(e, "uploading packed weights");
  Engine& m = H->e_moe;
  m.w1 = base + o.w1;
  m.w2 = base + o.w2;
  m.wr = base + o.wr;
  m.groups = reinterpret_cast<const GroupDev*>(base + o.g);
  m.gate_u = m.r.use_gate ? reinterpret_cast<const float*>(base + o.u) : nullptr;
  m.gate_b = m.r.use_gate ? reinterpret_cast<const float*>(base + o.b) : nullptr;
  m.lin_off = reinterpret_cast<const float*>(base + o.off);
  Engine& dn = H->e_dense;
  dn.w1 = base + o.dw1;
  dn.w2 = base + o.dw2;
  dn.wr = base + o.wr + H->router.size();      // the linear rows only
  dn.groups = reinterpret_cast<const GroupDev*>(base + o.dg);
  dn.lin_off = m.lin_off;
  H->uploaded = true;
  return CMOE_OK;
  CMOE_CATCH
}

int cmoe_hier_forward(cmoe_hier* H, const void* x_dev, int64_t T, void* y_dev, int32_t* outer_idx_dev,
                      int32_t* sub_idx_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!H) return fail(CMOE_EINVAL, "hierarchy is null");
  if (!H->uploaded) return fail(CMOE_ESTATE, "cmoe_hier_upload has not been called");
  return run_engine(H->e_moe, x_dev, T, y_dev, sub_idx_dev, outer_idx_dev, nullptr, nullptr, workspace_dev,
                    workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int cmoe_hier_dense_forward(cmoe_hier* H, const void* x_dev, int64_t T, void* y_dev, void* workspace_dev,
                            size_t workspace_bytes, void* hip_stream) {
  if (!H) return fail(CMOE_EINVAL, "hierarchy is null");
  if (!H->uploaded) return fail(CMOE_ESTATE, "cmoe_hier_upload has not been called");
  if (!H->baseline) return fail(CMOE_ESTATE, "the hierarchy was built without its un-restructured baseline");
  return run_engine(H->e_dense, x_dev, T, y_dev, nullptr, nullptr, nullptr, nullptr, workspace_dev, workspace_bytes,
                    static_cast<hipStream_t>(hip_stream));
}

int cmoe_hier_forward_timed(cmoe_hier* H, int dense, const void* x_dev, int64_t T, void* y_dev, void* workspace_dev,
                            size_t workspace_bytes, void* hip_stream, float* stage_ms) {
  if (!H) return fail(CMOE_EINVAL, "hierarchy is null");
  if (!H->uploaded) return fail(CMOE_ESTATE, "cmoe_hier_upload has not been called");
  if (dense && !H->baseline) return fail(CMOE_ESTATE, "the hierarchy was built without its un-restructured baseline");
  return run_engine_timed(dense ? H->e_dense : H->e_moe, x_dev, T, y_dev, workspace_dev, workspace_bytes,
                          static_cast<hipStream_t>(hip_stream), stage_ms);
}

void cmoe_hier_destroy(cmoe_hier* H) {
  if (!H) return;
  for (auto* L : H->experts) {
    L->in_hier = false;
    if (H->owns_experts) delete L;
  }
  delete H;
}

int cmoe_set_tuning(const char* name, int value) {
  if (!name) return fail(CMOE_EINVAL, "name is null");
  for (const TuningField& f : kTuningFields)
    if (std::strcmp(name, f.name) == 0) {
      tuning().*(f.field) = value;
      return CMOE_OK;
    }
  return fail(CMOE_EINVAL, "unknown tuning switch '%s'", name);
}

const char* cmoe_last_error(void) { return g_err.c_str(); }
const char* cmoe_version(void) { return "cmoe 0.1 (gfx950)"; }

}  // extern "C"
