// Activation profiling of the calibration set on the GPU (App. A.2 steps 1-2): hidden states
// H = Swish(X W_gate) * (X W_up) of every calibration token (Eq. 3, first line), then the K_a neurons of
// largest |h| per token (the ATopK matrix, kept as index lists).  Everything after that (rates, shared
// neurons, balanced clustering, representatives) stays on the host.
//
// profile_hidden_kernel  64 tokens x 64 neurons per workgroup, four waves of 32 x 32, bf16 MFMA with fp32
//                        accumulation straight out of global memory (the operands are read once per
//                        workgroup and mostly hit L2: 0.37 TFLOP at the LLaMA-2-7B shape take a few ms,
//                        against seconds on the host), |h| written as fp32
// profile_topk_kernel    one wave per token: the row of |h| is copied to LDS, then K_a rounds of
//                        (lane-local maximum, wave arg-max, mark as taken); ties go to the lowest index
#include <hip/hip_runtime.h>
#include <string>
#include <vector>
#include "cmoe_internal.h"
#include "device_utils.h"
#include "host_build.h"

namespace cmoe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void profile_hidden_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wg,
                                                             const bf16_t* __restrict__ wu, int d, int64_t q, int d_ff,
                                                             float* __restrict__ habs) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int64_t t0 = (int64_t)blockIdx.x * 64 + (wave & 1) * 32;
  const int n0 = blockIdx.y * 64 + (wave >> 1) * 32;
  int64_t t = t0 + l32;
  if (t >= q) t = q - 1;                      // duplicates of the last token; never stored
  int n = n0 + l32;
  if (n >= d_ff) n = d_ff - 1;
  const bf16_t* arow = x + t * d + lh * 8;
  const bf16_t* grow = wg + (int64_t)n * d + lh * 8;
  const bf16_t* urow = wu + (int64_t)n * d + lh * 8;
  floatx16_t accg, accu;
#pragma unroll
  for (int i = 0; i < 16; ++i) { accg[i] = 0.0f; accu[i] = 0.0f; }
  // 64-deep chunks of K, the loads of the next chunk issued before the MFMAs of the current one
  bf16x8_t a[2][4], bg[2][4], bu[2][4];
  auto load_chunk = [&](int kc, int buf) {
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      a[buf][s4] = *reinterpret_cast<const bf16x8_t*>(arow + kc + s4 * 16);
      bg[buf][s4] = *reinterpret_cast<const bf16x8_t*>(grow + kc + s4 * 16);
      bu[buf][s4] = *reinterpret_cast<const bf16x8_t*>(urow + kc + s4 * 16);
    }
  };
  load_chunk(0, 0);
  for (int kc = 0; kc < d; kc += 128) {        // two chunks per trip so that the buffer index is static
    if (kc + 64 < d) load_chunk(kc + 64, 1);
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      accg = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][s4], bg[0][s4], accg, 0, 0, 0);
      accu = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][s4], bu[0][s4], accu, 0, 0, 0);
    }
    if (kc + 64 < d) {
      if (kc + 128 < d) load_chunk(kc + 128, 0);
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        accg = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][s4], bg[1][s4], accg, 0, 0, 0);
        accu = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][s4], bu[1][s4], accu, 0, 0, 0);
      }
    }
  }
  // accumulator element i: token row (i/4)*8 + lh*4 + i%4, neuron column l32
  const int nn = n0 + l32;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int64_t tt = t0 + (i / 4) * 8 + lh * 4 + (i % 4);
    if (tt < q && nn < d_ff) habs[tt * d_ff + nn] = fabsf(silu_f32(accg[i]) * accu[i]);
  }
}

__global__ __launch_bounds__(64) void profile_topk_kernel(const float* __restrict__ habs, int d_ff, int k_act,
                                                          int32_t* __restrict__ active) {
  extern __shared__ float row[];               // [d_ff]
  const int lane = threadIdx.x;
  const int64_t t = blockIdx.x;
  for (int i = lane; i < d_ff; i += 64) row[i] = habs[t * d_ff + i];
  __syncthreads();
  for (int k = 0; k < k_act; ++k) {
    float best = -1.0f;
    int bi = 0x7fffffff;
    for (int i = lane; i < d_ff; i += 64) {    // ascending index: a later equal value never replaces
      const float v = row[i];
      if (v > best) { best = v; bi = i; }
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const float ob = __shfl_xor(best, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
    }
    if (lane == 0) active[t * k_act + k] = bi;
    if ((bi & 63) == lane && bi < d_ff) row[bi] = -2.0f;   // taken (magnitudes are >= 0)
    __syncthreads();
  }
}

int gpu_profile(const cmoe_config& cfg, const RoundedDense& rd, const float* calib_x, int64_t q, int32_t* active,
                std::string* msg) {
  const int d = cfg.d_model, d_ff = cfg.d_ff, k_act = cfg.k_act;
  auto bad = [&](const char* m) { if (msg) *msg = m; return (int)hipErrorInvalidValue; };
  if (cfg.dtype != CMOE_BF16) return bad("GPU profiling needs a bf16 layer");
  if (d % 64 != 0) return bad("GPU profiling needs d_model to be a multiple of 64");
  if ((size_t)d_ff * sizeof(float) > 160 * 1024) return bad("GPU profiling needs d_ff <= 40960");
  std::vector<uint16_t> xb((size_t)q * d);
  for (size_t i = 0; i < xb.size(); ++i) xb[i] = host_f32_to_bf16(calib_x[i]);
  const size_t w_bytes = (size_t)d_ff * d * 2, x_bytes = xb.size() * 2;
  const size_t h_bytes = (size_t)q * d_ff * sizeof(float), a_bytes = (size_t)q * k_act * sizeof(int32_t);
  char *dx = nullptr, *dg = nullptr, *du = nullptr, *dh = nullptr, *da = nullptr;
  hipError_t e = hipSuccess;
  auto ok = [&](hipError_t r) { if (e == hipSuccess && r != hipSuccess) e = r; return e == hipSuccess; };
  if (ok(hipMalloc(&dx, x_bytes)) && ok(hipMalloc(&dg, w_bytes)) && ok(hipMalloc(&du, w_bytes)) &&
      ok(hipMalloc(&dh, h_bytes)) && ok(hipMalloc(&da, a_bytes)) &&
      ok(hipMemcpy(dx, xb.data(), x_bytes, hipMemcpyHostToDevice)) &&
      ok(hipMemcpy(dg, rd.gate_t.data(), w_bytes, hipMemcpyHostToDevice)) &&
      ok(hipMemcpy(du, rd.up_t.data(), w_bytes, hipMemcpyHostToDevice))) {
    const dim3 grid((unsigned)((q + 63) / 64), (unsigned)((d_ff + 63) / 64));
    hipLaunchKernelGGL(profile_hidden_kernel, grid, dim3(256), 0, nullptr, reinterpret_cast<const bf16_t*>(dx),
                       reinterpret_cast<const bf16_t*>(dg), reinterpret_cast<const bf16_t*>(du), d, q, d_ff,
                       reinterpret_cast<float*>(dh));
    ok(hipGetLastError());
    const size_t smem = (size_t)d_ff * sizeof(float);
    if (e == hipSuccess)
      ok(hipFuncSetAttribute(reinterpret_cast<const void*>(profile_topk_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)smem));
    if (e == hipSuccess) {
      hipLaunchKernelGGL(profile_topk_kernel, dim3((unsigned)q), dim3(64), smem, nullptr,
                         reinterpret_cast<const float*>(dh), d_ff, k_act, reinterpret_cast<int32_t*>(da));
      ok(hipGetLastError());
    }
    ok(hipMemcpy(active, da, a_bytes, hipMemcpyDeviceToHost));   // synchronises with the null stream
  }
  (void)hipFree(dx);
  (void)hipFree(dg);
  (void)hipFree(du);
  (void)hipFree(dh);
  (void)hipFree(da);
  if (e != hipSuccess && msg) *msg = hipGetErrorString(e);
  return (int)e;
}

}  // namespace cmoe
