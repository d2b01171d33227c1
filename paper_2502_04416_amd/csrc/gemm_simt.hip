// Grouped SwiGLU expert kernels with plain fp32 FMA arithmetic (no matrix cores).  They serve the
// fp32 layers (tolerance 1e-5, where bf16 MFMA inputs would be too coarse) and follow the same work
// list, gather and ragged layouts as the bf16 MFMA kernels:
//   MODE 1  H_g = Swish(X_g Wgate_g) * (X_g Wup_g)   (Eq. 3, first line, on the group's neurons)
//   MODE 2  Y_g = H_g Wdown_g                        (Eq. 3, second line)
#include "cmoe_internal.h"
#include "device_utils.h"

namespace cmoe {

template <typename T>
struct SimtArgs {
  const T* A;
  const T* B;
  T* C;
  const GroupDev* groups;
  const int32_t* seg_off;
  const int32_t* work;
  const int64_t* h_off;
  const int32_t* slot2tok;
  int G;
  int d;
  int ldb;
  int b_tiled;               // 1: B is tiled 16 x 32 (bf16 layers run here only when forced to)
  int64_t T_tokens;
  int single;
};

constexpr int SB = 64;     // tile rows and tile columns
constexpr int SK = 16;     // K step

template <typename T, int MODE>
__global__ __launch_bounds__(256) void grouped_gemm_simt(SimtArgs<T> p) {
  __shared__ float As[SK][SB + 4];
  __shared__ float Bs[SK][SB + 4];
  const int tid = threadIdx.x;
  const int ty = tid >> 4, tx = tid & 15;
  int wid = blockIdx.x;
  int g = 0, local = wid, cnt, seg0 = 0, wp;
  int64_t hoff = 0;
  if (p.single) {
    cnt = (int)p.T_tokens;
    wp = p.groups[0].width_pad;
  } else {
    if (wid >= p.work[p.G]) return;
    g = find_group(p.work, p.G, wid);
    local = wid - p.work[g];
    seg0 = p.seg_off[g];
    cnt = p.seg_off[g + 1] - seg0;
    wp = p.groups[g].width_pad;
    hoff = p.h_off[g];
  }
  const int K = (MODE == 1) ? p.d : wp;
  const int n_cols = (MODE == 1) ? 2 * wp : p.d;
  const int n_nt = (n_cols + SB - 1) / SB;
  const int n_mt = (cnt + SB - 1) / SB;
  if (p.single && local >= n_mt * n_nt) return;
  const int mt = local / n_nt, nt = local % n_nt;

  // loader: thread loads 4 consecutive k of one row for A and for B
  const int lrow = tid >> 2, lk = (tid & 3) * 4;
  int ar = mt * SB + lrow;
  if (ar >= cnt) ar = cnt - 1;
  const T* a_src;
  if (MODE == 1) {
    const int64_t tok = p.slot2tok ? p.slot2tok[seg0 + ar] : (seg0 + ar);
    a_src = p.A + tok * p.d;
  } else {
    a_src = p.A + hoff + (int64_t)ar * wp;
  }
  int bn = nt * SB + lrow;
  if (bn >= n_cols) bn = n_cols - 1;
  const T* b_src = (MODE == 1) ? p.B + ((int64_t)p.groups[g].w1_row0 + bn) * p.ldb
                               : p.B + p.groups[g].w2_off + (int64_t)bn * wp;
  // tiled weights: element (row, k) through the layout function instead of b_src + k
  const int64_t b_rowg = (MODE == 1) ? (int64_t)p.groups[g].w1_row0 + bn : bn;
  const T* b_base = (MODE == 1) ? p.B : p.B + p.groups[g].w2_off;
  const int b_kt32 = (MODE == 1) ? p.ldb / TILE_K : wp / TILE_K;
  // columns owned by this thread inside the 64-wide tile
  int cols[4];
  if (MODE == 1) { cols[0] = 2 * tx; cols[1] = 2 * tx + 1; cols[2] = IL + 2 * tx; cols[3] = IL + 2 * tx + 1; }
  else { cols[0] = 4 * tx; cols[1] = 4 * tx + 1; cols[2] = 4 * tx + 2; cols[3] = 4 * tx + 3; }

  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;

  for (int k0 = 0; k0 < K; k0 += SK) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + lk + j;
      As[lk + j][lrow] = (k < K) ? Elem<T>::ld(a_src + k) : 0.0f;
      Bs[lk + j][lrow] = (k < K) ? Elem<T>::ld(p.b_tiled ? b_base + tiled_offset(b_rowg, k, b_kt32) : b_src + k) : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < SK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][cols[j]];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = mt * SB + ty * 4 + i;
    if (r >= cnt) continue;
    if (MODE == 1) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int neuron = nt * (SB / 2) + 2 * tx + j;
        if (neuron < wp) Elem<T>::st(p.C + hoff + (int64_t)r * wp + neuron, silu_f32(acc[i][j]) * acc[i][j + 2]);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = nt * SB + cols[j];
        if (col < p.d) Elem<T>::st(p.C + (int64_t)(seg0 + r) * p.d + col, acc[i][j]);
      }
    }
  }
}

template <typename T>
static hipError_t run_simt(const Engine& e, const void* x, int64_t Tn, char* ws, const WsLayout& L, void* y,
                           hipStream_t s, int stage) {
  SimtArgs<T> a;
  a.groups = e.groups;
  a.seg_off = reinterpret_cast<const int32_t*>(ws + L.seg_off);
  a.h_off = reinterpret_cast<const int64_t*>(ws + L.h_off);
  a.G = e.G;
  a.d = e.d;
  a.ldb = e.ldw1;
  a.b_tiled = e.w_tiled;
  a.T_tokens = Tn;
  a.single = (e.G == 1 && e.n_always == 1) ? 1 : 0;
  a.A = static_cast<const T*>(x);
  a.B = static_cast<const T*>(e.w1);
  a.C = reinterpret_cast<T*>(ws + L.h);
  a.work = reinterpret_cast<const int32_t*>(ws + L.work1);
  a.slot2tok = a.single ? nullptr : reinterpret_cast<const int32_t*>(ws + L.slot2tok);
  if (stage != 2) {
    hipLaunchKernelGGL((grouped_gemm_simt<T, 1>), dim3((unsigned)gemm_work_bound(e, Tn, 1)), dim3(256), 0, s, a);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || stage == 1) return err;
  }
  a.A = reinterpret_cast<const T*>(ws + L.h);
  a.B = static_cast<const T*>(e.w2);
  a.C = e.direct_output() ? static_cast<T*>(y) : reinterpret_cast<T*>(ws + L.y_slots);
  a.work = reinterpret_cast<const int32_t*>(ws + L.work2);
  a.slot2tok = nullptr;
  hipLaunchKernelGGL((grouped_gemm_simt<T, 2>), dim3((unsigned)gemm_work_bound(e, Tn, 2)), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_experts_simt(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y,
                               hipStream_t s, int stage) {
  if (e.dtype == 1) return run_simt<bf16_t>(e, x, T, ws, L, y, s, stage);
  return run_simt<float>(e, x, T, ws, L, y, s, stage);
}

int simt_gemm_tile(int which) { return which >= 5 ? 0 : SB; }   // (5, 6: no tiles of dynamic height here)

}  // namespace cmoe
