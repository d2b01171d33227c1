// Grouped SwiGLU expert kernels for bf16 layers (Eq. 3 restricted to an expert's neurons):
//   MODE 1  H_g = Swish(X_g Wgate_g) * (X_g Wup_g)     rows of X gathered through slot2tok, K = d
//   MODE 2  Y_g = H_g Wdown_g                          K = width_pad(g), N = d
// Both are C = A * B^T with K contiguous in A and in B, computed with v_mfma_f32_32x32x16_bf16 from
// LDS-staged, XOR-swizzled tiles.  A work item is (group, row tile, column tile); the list of work
// items is a device-side prefix array written by the permute kernel, so ragged, empty and skewed
// groups need no host round trip.  Workgroups whose index is past the list exit at once.
#include <cstdlib>
#include "cmoe_internal.h"
#include "device_utils.h"

namespace cmoe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

struct GemmArgs {
  const bf16_t* A;
  const bf16_t* B;
  bf16_t* C;
  const GroupDev* groups;
  const int32_t* seg_off;    // [G+1]
  const int32_t* work;       // [G+1]
  const int64_t* h_off;      // [G+1]
  const int32_t* slot2tok;   // MODE 1 gather; null = identity
  int G;
  int d;
  int64_t T;
  int single;                // 1: one always-on group holding all T tokens; no device schedule is read
  int n_blocks;              // grid size (multiple of 8)
  int xcd_remap;             // 1: consecutive work items run on the same XCD
};

constexpr int BK = 64;

// element offset of 16-byte chunk c (0..7) of row `row` in a [rows][64] bf16 tile; the XOR spreads the
// 16 rows that one ds_read_b128 wave-quarter touches over all 64 banks
__device__ __forceinline__ int lds_off(int row, int c) { return row * BK + ((c ^ ((row >> 1) & 7)) << 3); }

template <int BM, int BN, int WGM, int WGN, int MODE>
__global__ __launch_bounds__(WGM* WGN * 64) void grouped_gemm_bf16(GemmArgs p) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int TM = BM / WGM, TN = BN / WGN, MI = TM / 32, NI = TN / 32;
  constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;
  static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "tile");
  static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "loader");
  static_assert(MODE != 1 || TN % 64 == 0, "gate/up pairs must stay inside a wave tile");
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t* As = smem;                       // [2][BM*BK]
  bf16_t* Bs = smem + 2 * BM * BK;         // [2][BN*BK]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int l32 = lane & 31, lh = lane >> 5;

  // ---- which work item? ----
  // Workgroup b runs on XCD b % 8.  With the remap, XCD x works through the contiguous range
  // [x * ceil(W/8), (x+1) * ceil(W/8)) of the W work items, so tiles that share operands meet in one L2.
  int g = 0, cnt, seg0 = 0, wp;
  int64_t hoff = 0;
  int n_work;
  if (p.single) {
    cnt = (int)p.T;
    wp = p.groups[0].width_pad;
    const int nc = (MODE == 1) ? 2 * wp : p.d;
    n_work = ((cnt + BM - 1) / BM) * ((nc + BN - 1) / BN);
  } else {
    n_work = p.work[p.G];
  }
  int wid = blockIdx.x;
  if (p.xcd_remap) {
    const int chunk = (n_work + 7) >> 3;
    if ((wid >> 3) >= chunk) return;
    wid = (wid & 7) * chunk + (wid >> 3);
  }
  if (wid >= n_work) return;
  int local = wid;
  if (!p.single) {
    // G is small: binary search over the prefix array
    int lo = 0, hi = p.G;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.work[mid] <= wid) lo = mid; else hi = mid;
    }
    // skip empty groups that share the same prefix value
    g = lo;
    local = wid - p.work[g];
    seg0 = p.seg_off[g];
    cnt = p.seg_off[g + 1] - seg0;
    wp = p.groups[g].width_pad;
    hoff = p.h_off[g];
  }
  const int K = (MODE == 1) ? p.d : wp;
  const int n_cols = (MODE == 1) ? 2 * wp : p.d;         // columns of C^T = rows of B
  const int n_nt = (n_cols + BN - 1) / BN;
  const int mt = local / n_nt, nt = local % n_nt;

  // ---- per-thread global sources ----
  const bf16_t* a_src[A_CH];
  const bf16_t* b_src[B_CH];
  int a_dst[A_CH], b_dst[B_CH];
  const int cchunk = tid & 7;
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int row = (tid >> 3) + i * (NT >> 3);
    int r = mt * BM + row;
    if (r >= cnt) r = cnt - 1;
    if (MODE == 1) {
      const int64_t tok = p.slot2tok ? p.slot2tok[seg0 + r] : (seg0 + r);
      a_src[i] = p.A + tok * p.d + cchunk * 8;
    } else {
      a_src[i] = p.A + hoff + (int64_t)r * wp + cchunk * 8;
    }
    a_dst[i] = lds_off(row, cchunk);
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int row = (tid >> 3) + i * (NT >> 3);
    int n = nt * BN + row;
    if (n >= n_cols) n = n_cols - 1;
    if (MODE == 1) b_src[i] = p.B + ((int64_t)p.groups[g].w1_row0 + n) * p.d + cchunk * 8;
    else b_src[i] = p.B + p.groups[g].w2_off + (int64_t)n * wp + cchunk * 8;
    b_dst[i] = lds_off(row, cchunk);
  }

  floatx16_t acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.0f;

  uint4 ra[A_CH], rb[B_CH];
  const int KT = (K + BK - 1) / BK;
  auto g_load = [&](int kt) {
    const int k = kt * BK + cchunk * 8;
    const bool ok = k < K;                       // K is a multiple of 8: a chunk is all in or all out
#pragma unroll
    for (int i = 0; i < A_CH; ++i) ra[i] = ok ? *reinterpret_cast<const uint4*>(a_src[i] + kt * BK) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < B_CH; ++i) rb[i] = ok ? *reinterpret_cast<const uint4*>(b_src[i] + kt * BK) : make_uint4(0, 0, 0, 0);
  };
  auto s_store = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) *reinterpret_cast<uint4*>(As + buf * BM * BK + a_dst[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *reinterpret_cast<uint4*>(Bs + buf * BN * BK + b_dst[i]) = rb[i];
  };

  g_load(0);
  s_store(0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) g_load(kt + 1);
    const bf16_t* as = As + buf * BM * BK;
    const bf16_t* bs = Bs + buf * BN * BK;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8_t af[MI], bfr[NI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        af[mi] = *reinterpret_cast<const bf16x8_t*>(as + lds_off(wm * TM + mi * 32 + l32, ks * 2 + lh));
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        bfr[ni] = *reinterpret_cast<const bf16x8_t*>(bs + lds_off(wn * TN + ni * 32 + l32, ks * 2 + lh));
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
    }
    if (kt + 1 < KT) s_store(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue ----
  // accumulator element i of a 32x32 tile: row (i/4)*8 + (lane/32)*4 + i%4, column lane%32
  if (MODE == 1) {
    bf16_t* H = p.C + hoff;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int pi = 0; pi < NI / 2; ++pi) {
        const int neuron = (nt * BN + wn * TN) / 2 + pi * 32 + l32;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int r = mt * BM + wm * TM + mi * 32 + (i / 4) * 8 + lh * 4 + (i % 4);
          if (r < cnt && neuron < wp) {
            const float gt = acc[mi][2 * pi][i], up = acc[mi][2 * pi + 1][i];
            H[(int64_t)r * wp + neuron] = f32_to_bf16(silu_f32(gt) * up);
          }
        }
      }
  } else {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const int col = nt * BN + wn * TN + ni * 32 + l32;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int r = mt * BM + wm * TM + mi * 32 + (i / 4) * 8 + lh * 4 + (i % 4);
          if (r < cnt && col < p.d) p.C[(int64_t)(seg0 + r) * p.d + col] = f32_to_bf16(acc[mi][ni][i]);
        }
      }
  }
}

// ---- tile configurations ---------------------------------------------------------------------
struct TileCfg { int bm, bn, wgm, wgn; };
static const TileCfg kCfgs[] = {
    {256, 128, 2, 2},   // 0
    {128, 128, 2, 2},   // 1
    {256, 256, 2, 4},   // 2
    {256, 128, 4, 2},   // 3
    {128, 256, 2, 2},   // 4
};
constexpr int kNumCfgs = sizeof(kCfgs) / sizeof(kCfgs[0]);

static int env_int(const char* name, int dflt) {
  const char* v = std::getenv(name);
  return v ? std::atoi(v) : dflt;
}
// The environment is read at every call (a getenv is nothing next to a kernel launch) so that a tuning
// script can switch tile shapes inside one process.
static int cfg_index(int which) {
  int c = env_int(which == 1 ? "CMOE_GEMM1_CFG" : "CMOE_GEMM2_CFG", 0);
  if (c < 0 || c >= kNumCfgs) c = 0;
  return c;
}

// which = 1: BM of gate/up, 2: BM of down, 3: BN of gate/up (packed rows), 4: BN of down
int bf16_gemm_tile(int which) {
  switch (which) {
    case 1: return kCfgs[cfg_index(1)].bm;
    case 2: return kCfgs[cfg_index(2)].bm;
    case 3: return kCfgs[cfg_index(1)].bn;
    default: return kCfgs[cfg_index(2)].bn;
  }
}

template <int BM, int BN, int WGM, int WGN, int MODE>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s) {
  constexpr size_t smem = 2 * (size_t)(BM + BN) * BK * sizeof(bf16_t);
  static bool attr_done = false;
  auto kern = grouped_gemm_bf16<BM, BN, WGM, WGN, MODE>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3(a.n_blocks), dim3(WGM * WGN * 64), smem, s, a);
  return hipGetLastError();
}

template <int MODE>
static hipError_t launch_cfg(int ci, const GemmArgs& a, hipStream_t s) {
  switch (ci) {
    case 0: return launch_one<256, 128, 2, 2, MODE>(a, s);
    case 1: return launch_one<128, 128, 2, 2, MODE>(a, s);
    case 2: return launch_one<256, 256, 2, 4, MODE>(a, s);
    case 3: return launch_one<256, 128, 4, 2, MODE>(a, s);
    default: return launch_one<128, 256, 2, 2, MODE>(a, s);
  }
}

hipError_t launch_experts_bf16(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y,
                               hipStream_t s, int stage) {
  const int remap = env_int("CMOE_XCD_REMAP", 1);
  GemmArgs a;
  a.groups = e.groups;
  a.seg_off = reinterpret_cast<const int32_t*>(ws + L.seg_off);
  a.h_off = reinterpret_cast<const int64_t*>(ws + L.h_off);
  a.G = e.G;
  a.d = e.d;
  a.T = T;
  a.single = (e.G == 1 && e.n_always == 1) ? 1 : 0;
  a.xcd_remap = remap;
  // gate/up
  a.A = static_cast<const bf16_t*>(x);
  a.B = static_cast<const bf16_t*>(e.w1);
  a.C = reinterpret_cast<bf16_t*>(ws + L.h);
  a.work = reinterpret_cast<const int32_t*>(ws + L.work1);
  a.slot2tok = a.single ? nullptr : reinterpret_cast<const int32_t*>(ws + L.slot2tok);
  a.n_blocks = (int)round_up64(gemm_work_bound(e, T, 1), 8);
  if (stage != 2) {
    hipError_t err = launch_cfg<1>(cfg_index(1), a, s);
    if (err != hipSuccess || stage == 1) return err;
  }
  // down
  a.A = reinterpret_cast<const bf16_t*>(ws + L.h);
  a.B = static_cast<const bf16_t*>(e.w2);
  a.C = (e.S_all() == 1) ? static_cast<bf16_t*>(y) : reinterpret_cast<bf16_t*>(ws + L.y_slots);
  a.work = reinterpret_cast<const int32_t*>(ws + L.work2);
  a.slot2tok = nullptr;
  a.n_blocks = (int)round_up64(gemm_work_bound(e, T, 2), 8);
  return launch_cfg<2>(cfg_index(2), a, s);
}

}  // namespace cmoe
