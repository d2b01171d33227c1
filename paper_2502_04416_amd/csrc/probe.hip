// Measurement aid: what the matrix cores of this device sustain when nothing but the MFMA pipe is in use.
// The expert contractions (Eq. 3 on neuron slices, Sec. 4.1) are priced against the published MFMA peak;
// this probe shows how much of that peak the device delivers at all once the operands are not zeros
// (the shader clock drops under the power the multipliers draw).
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstring>
#include <vector>
#include "../../include/cmoe.h"
#include "cmoe_internal.h"

namespace cmoe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

constexpr int PROBE_VECS = 4096;     // 16-byte operand vectors in the source buffer

// Eight waves per workgroup, one workgroup per CU; every wave keeps eight independent 32x32 accumulators
// and issues 8 MFMAs per round from six operand registers loaded once.
__global__ __launch_bounds__(512) void mfma_probe_kernel(const uint4* __restrict__ src, int iters, float* sink,
                                                         long long* clk, int store) {
  const int tid = threadIdx.x;
  bf16x8_t fa[4], fb[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) { const uint4 v = src[(tid * 6 + i) & (PROBE_VECS - 1)]; fa[i] = *reinterpret_cast<const bf16x8_t*>(&v); }
#pragma unroll
  for (int i = 0; i < 2; ++i) { const uint4 v = src[(tid * 6 + 4 + i) & (PROBE_VECS - 1)]; fb[i] = *reinterpret_cast<const bf16x8_t*>(&v); }
  floatx16_t acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.0f;
  long long t0 = 0, w0 = 0;
  if (blockIdx.x == 0 && tid == 0) { t0 = __builtin_readcyclecounter(); w0 = wall_clock64(); }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[j >> 1], fb[j & 1], acc[j], 0, 0, 0);
  }
  if (blockIdx.x == 0 && tid == 0) { clk[0] = __builtin_readcyclecounter() - t0; clk[1] = wall_clock64() - w0; }
  if (store) {                        // never taken by the probe; keeps the accumulators alive
    float t = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 16; ++i) t += acc[j][i];
    sink[tid] = t;
  }
}

// Streaming read: every workgroup of eight waves reads its own 256 KB of consecutive memory, each load
// instruction 1 KB of consecutive bytes, all 32 loads of a lane in flight: the access pattern the weight
// layout gives the decode kernels, with nothing else to do.
constexpr int HBM_PROBE_BLOCK_BYTES = 512 * 32 * 16;
__global__ __launch_bounds__(512) void hbm_probe_kernel(const uint4* __restrict__ src, float* sink) {
  const uint4* p = src + (size_t)blockIdx.x * (HBM_PROBE_BLOCK_BYTES / 16) + (threadIdx.x >> 6) * (32 * 64) + (threadIdx.x & 63);
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    const uint4 v = p[i * 64];
    acc ^= v.x ^ v.w;
  }
  if (acc == 0x12345678u) sink[0] = 1.0f;        // never true for the zero-filled buffer; keeps the loads alive
}

}  // namespace cmoe

extern "C" int cmoe_probe_hbm(size_t bytes, int reps, double* gbytes_per_s) {
  using namespace cmoe;
  if (!gbytes_per_s || reps < 1 || reps > 1000 || bytes < HBM_PROBE_BLOCK_BYTES || bytes > ((size_t)64 << 30))
    return fail(CMOE_EINVAL, "cmoe_probe_hbm: need 256 KB <= bytes <= 64 GiB, 1 <= reps <= 1000, a result pointer");
  const size_t n_blocks = bytes / HBM_PROBE_BLOCK_BYTES;
  if (n_blocks > 0x7fffffffu) return fail(CMOE_EINVAL, "cmoe_probe_hbm: too many workgroups");
  const size_t used = n_blocks * HBM_PROBE_BLOCK_BYTES;
  char* buf = nullptr;
  if (hipMalloc(&buf, used + 256) != hipSuccess) return fail(CMOE_ENOMEM, "cmoe_probe_hbm: device allocation failed");
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = CMOE_OK;
  float best = 0.0f;
  auto ok = [&](hipError_t e) { if (e != hipSuccess && rc == CMOE_OK) rc = fail(CMOE_EHIP, "cmoe_probe_hbm: %s", hipGetErrorString(e)); return e == hipSuccess; };
  if (ok(hipMemset(buf, 0, used + 256)) && ok(hipEventCreate(&e0)) && ok(hipEventCreate(&e1))) {
    const uint4* src = reinterpret_cast<const uint4*>(buf);
    float* sink = reinterpret_cast<float*>(buf + used);
    for (int rep = 0; rep <= reps && rc == CMOE_OK; ++rep) {     // the first launch is a warm-up
      float ms = 0.0f;
      ok(hipEventRecord(e0, nullptr));
      hipLaunchKernelGGL(hbm_probe_kernel, dim3((unsigned)n_blocks), dim3(512), 0, nullptr, src, sink);
      ok(hipGetLastError());
      ok(hipEventRecord(e1, nullptr));
      ok(hipEventSynchronize(e1));
      ok(hipEventElapsedTime(&ms, e0, e1));
      if (rep > 0 && (best == 0.0f || ms < best)) best = ms;
    }
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(buf);
  if (rc != CMOE_OK) return rc;
  *gbytes_per_s = (double)used / (best * 1e-3) / 1e9;
  return CMOE_OK;
}

extern "C" int cmoe_probe_mfma(int random_operands, int iters, double* tflops, double* shader_mhz) {
  using namespace cmoe;
  if (iters < 1 || iters > (1 << 22) || !tflops) return fail(CMOE_EINVAL, "cmoe_probe_mfma: need 1 <= iters <= 2^22 and tflops != NULL");
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return fail(CMOE_EHIP, "no device");
  const int n_cu = prop.multiProcessorCount;
  std::vector<uint16_t> host((size_t)PROBE_VECS * 8, 0);
  if (random_operands) {              // N(0, 0.05^2) by Box-Muller on a fixed xorshift stream
    uint64_t s = 0x9E3779B97F4A7C15ull;
    auto uni = [&]() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return ((s >> 11) + 1) * (1.0 / 9007199254740993.0); };
    for (auto& v : host) {
      const float f = (float)(0.05 * std::sqrt(-2.0 * std::log(uni())) * std::cos(6.283185307179586 * uni()));
      uint32_t u;
      std::memcpy(&u, &f, 4);
      u += 0x7fffu + ((u >> 16) & 1u);
      v = (uint16_t)(u >> 16);
    }
  }
  char* buf = nullptr;
  const size_t src_bytes = (size_t)PROBE_VECS * 16, sink_bytes = 512 * sizeof(float);
  if (hipMalloc(&buf, src_bytes + sink_bytes + 64) != hipSuccess) return fail(CMOE_ENOMEM, "cmoe_probe_mfma: device allocation failed");
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = CMOE_OK;
  float ms = 0.0f;
  long long c[2] = {0, 0};
  auto ok = [&](hipError_t e) { if (e != hipSuccess && rc == CMOE_OK) rc = fail(CMOE_EHIP, "cmoe_probe_mfma: %s", hipGetErrorString(e)); return e == hipSuccess; };
  if (ok(hipMemcpy(buf, host.data(), src_bytes, hipMemcpyHostToDevice)) && ok(hipEventCreate(&e0)) && ok(hipEventCreate(&e1))) {
    uint4* src = reinterpret_cast<uint4*>(buf);
    float* sink = reinterpret_cast<float*>(buf + src_bytes);
    long long* clk = reinterpret_cast<long long*>(buf + src_bytes + sink_bytes);
    for (int rep = 0; rep < 2 && rc == CMOE_OK; ++rep) {   // the first launch warms the clocks up
      ok(hipEventRecord(e0, nullptr));
      hipLaunchKernelGGL(mfma_probe_kernel, dim3(n_cu), dim3(512), 0, nullptr, src, iters, sink, clk, 0);
      ok(hipGetLastError());
      ok(hipEventRecord(e1, nullptr));
      ok(hipEventSynchronize(e1));
      ok(hipEventElapsedTime(&ms, e0, e1));
    }
    ok(hipMemcpy(c, clk, sizeof(c), hipMemcpyDeviceToHost));
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(buf);
  if (rc != CMOE_OK) return rc;
  const double flop = (double)n_cu * 8.0 * iters * 8.0 * 2.0 * 32 * 32 * 16;
  *tflops = flop / (ms * 1e-3) / 1e12;
  if (shader_mhz) *shader_mhz = c[1] > 0 ? c[0] * 100.0 / c[1] : 0.0;   // cycle counter ticks per 100 MHz wall tick
  return CMOE_OK;
}
