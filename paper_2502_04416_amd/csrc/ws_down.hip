// Weight-stationary down contraction for narrow experts (Eq. 3, second line, on an expert's neuron slice):
//   Y_g = H_g Wdown_g        rows = the slots of group g, K = width_pad(g) in {352, 448, 704}, N = d.
//
// With K this short a (rows x 256 columns) tile of the general kernel is a dozen K steps between a prologue of
// three memory round trips and an epilogue: the launch is bound by what a CU can ingest (85 flop per byte
// fetched), not by its matrix cores.  Here a workgroup owns a strip of 256 output columns of one group for a
// chunk of that group's rows.  Each of its four waves keeps its 64 columns x K of Wdown in registers as MFMA
// operands for the whole item (K / 2 registers per lane), the rows of H stream through LDS in pieces of 64 (or
// 32) rows that are contiguous in memory, and every A fragment read from LDS feeds two MFMAs.  Per piece a
// workgroup fetches rows x K x 2 bytes and writes rows x 512 bytes for rows x 256 x K x 2 flop: 150-250 flop per
// byte, on the compute side of the balance.
//
// Measured (config 2, 8192 tokens, 189 GFLOP): 351 us against 267 us for the 128 x 256 tiles of the general
// kernel; config 1, 2048 tokens: 90 against 72 us.  With the stores, the piece transfers or the MFMAs switched
// off in turn the launch loses 60, 117 and 110 us: the three do not overlap.  One workgroup of four waves per
// CU (the weights take 176-352 registers per lane) has a single 56 KB piece in flight while it multiplies the
// other, against 150 KB for two co-resident workgroups of the tiled kernel, and every strip re-reads the rows
// of H.  The kernel is therefore not chosen by default (tuning switch ws_down = 2 selects it); it is kept
// because it is exact, tested, and the arrangement to start from if the rows of H can be shared between strips.
//
// Work items are (group, row chunk, strip) in the same device-side
// prefix list the general kernel uses; groups whose width has no instantiation here are left to that kernel
// (it skips the others), so both can be launched over one list.
#include <type_traits>
#include "cmoe_internal.h"
#include "device_utils.h"

namespace cmoe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

__device__ __attribute__((aligned(16))) uint32_t g_ws_zero_chunk[4] = {0, 0, 0, 0};

struct WsArgs {
  const bf16_t* H;
  const bf16_t* W2;
  bf16_t* Y;
  const GroupDev* groups;
  const int32_t* seg_off;    // [G+1]
  const int32_t* work;       // [G+1] prefix of work items, then [9] first item of each XCD's share
  const int64_t* h_off;      // [G+1]
  int G, d;
  int rc;                    // rows of a group per work item
  int xcd_remap;
};

__device__ __forceinline__ void ws_dma16(const void* gsrc, char* lds_dst) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gsrc),
                                   (__attribute__((address_space(3))) void*)(lds_dst), 16, 0, 0);
}
template <int N>
__device__ __forceinline__ void ws_wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Row stride of a piece in LDS: the row's K * 2 bytes rounded up to an odd number of 128-byte groups, so that
// consecutive rows start in alternate halves of the 256-byte bank span; inside a group the eight 16-byte chunks
// are XOR-swizzled with (row >> 1) & 7.  The 16 rows a quarter of a ds_read_b128 touches then fall into 16
// different 16-byte bank groups.
__host__ __device__ constexpr int ws_stride_bytes(int ks) {
  const int groups = (ks * 32 + 127) / 128;
  return ((groups & 1) ? groups : groups + 1) * 128;
}
__host__ __device__ constexpr int ws_stage_bytes(int ks, int rb) { return 32 * rb * ws_stride_bytes(ks); }
constexpr int WS_STRIP_LD = 64 + 8;                            // epilogue strip row stride in elements
constexpr int WS_STRIP_BYTES = 4 * 32 * WS_STRIP_LD * 2;       // four waves
__host__ __device__ constexpr int ws_smem_bytes(int ks, int rb) { return 2 * ws_stage_bytes(ks, rb) + WS_STRIP_BYTES; }

template <int KS, int RB>
__device__ __forceinline__ void ws_down_item(const WsArgs& p, int g, int local, int seg0, int cnt, int64_t hoff, char* smem) {
  constexpr int K = KS * 16;
  constexpr int STRIDE = ws_stride_bytes(KS);
  constexpr int STAGE = ws_stage_bytes(KS, RB);
  constexpr int PR = 32 * RB;                                  // rows per piece
  constexpr int NDW = STAGE / 1024 / 4;                        // DMA instructions per wave and piece
  static_assert(STAGE % 4096 == 0, "a piece is a whole number of 1 KB transfers per wave");
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int n_strips = p.d / 256;
  const int strip = local % n_strips, chunk = local / n_strips;
  const int row0 = chunk * p.rc;
  const int rows = min(p.rc, cnt - row0);
  const int c0 = strip * 256 + wave * 64;
  const int n_pieces = (rows + PR - 1) / PR;

  // ---- per-lane sources of the piece transfers: LDS slot (transfer q, lane) -> (row, logical chunk) ----
  int a_off[NDW];                                              // element offset inside the piece, -1: padding
  int a_row[NDW];
#pragma unroll
  for (int j = 0; j < NDW; ++j) {
    const int off = (j * 4 + wave) * 1024 + lane * 16;
    const int row = off / STRIDE, within = off - row * STRIDE;
    const int grp = within >> 7, slot = (within & 127) >> 4;
    const int ch = grp * 8 + (slot ^ ((row >> 1) & 7));
    a_row[j] = row;
    a_off[j] = (ch * 8 < K) ? row * K + ch * 8 : -1;
  }
  const bf16_t* hbase = p.H + hoff + (int64_t)row0 * K;
  auto issue_piece = [&](int pc) {
    char* dst = smem + (pc & 1) * STAGE;
    const bf16_t* src0 = hbase + (int64_t)pc * PR * K;
#pragma unroll
    for (int j = 0; j < NDW; ++j) {
      const void* src = (a_off[j] >= 0 && pc * PR + a_row[j] < rows) ? (const void*)(src0 + a_off[j]) : (const void*)g_ws_zero_chunk;
      ws_dma16(src, dst + (j * 4 + wave) * 1024);
    }
  };
  auto lds_a = [&](int row, int ch) { return row * STRIDE + (ch >> 3) * 128 + (((ch & 7) ^ ((row >> 1) & 7)) << 4); };

  bf16_t* strip_lds = reinterpret_cast<bf16_t*>(smem + 2 * STAGE) + wave * 32 * WS_STRIP_LD;
  bf16_t* ybase = p.Y + (int64_t)(seg0 + row0) * p.d + c0;

  // The first piece's transfers go out first, then the weights in the order the MFMAs use them, then the second
  // piece: loads complete in order, so the first MFMAs can start as soon as the piece and the first weight
  // fragments are there while the rest of the weights is still arriving.
  issue_piece(0);
  // ---- this wave's 64 columns x K of Wdown as MFMA operands, resident for the whole item ----
  bf16x8_t breg[2][KS];
  {
    const bf16_t* wbase = p.W2 + p.groups[g].w2_off;
    constexpr int kt2 = K / TILE_K;
    const bf16_t* wc[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int c = c0 + nb * 32 + l32;
      wc[nb] = wbase + ((int64_t)(c / TILE_ROWS) * kt2) * TILE_ELEMS + (c % TILE_ROWS) * TILE_K + lh * 8;
    }
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        breg[nb][s] = *reinterpret_cast<const bf16x8_t*>(wc[nb] + (s / 2) * TILE_ELEMS + (s & 1) * 16);
  }
  if (n_pieces > 1) issue_piece(1);
  // piece 0 is older than every weight load: wait for everything but the second piece's transfers
  if (n_pieces > 1) ws_wait_vmcnt<NDW>();
  else ws_wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  for (int pc = 0; pc < n_pieces; ++pc) {
    const char* st = smem + (pc & 1) * STAGE;
    floatx16_t acc[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[rb][nb][i] = 0.0f;
    // A fragments are requested PD steps ahead of the MFMAs that use them (an LDS read takes longer than the
    // two or four MFMAs of a step), and the order is pinned: left to itself the compiler moves every read next
    // to its use and the matrix cores wait for the LDS at every step.
    constexpr int PD = (RB >= 2) ? 2 : 4;
    bf16x8_t af[PD + 1][RB];
#pragma unroll
    for (int s = 0; s < PD && s < KS; ++s)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) af[s][rb] = *reinterpret_cast<const bf16x8_t*>(st + lds_a(rb * 32 + l32, 2 * s + lh));
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      __builtin_amdgcn_sched_barrier(0);
      if (s + PD < KS) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          af[(s + PD) % (PD + 1)][rb] = *reinterpret_cast<const bf16x8_t*>(st + lds_a(rb * 32 + l32, 2 * (s + PD) + lh));
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          acc[rb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(breg[nb][s], af[s % (PD + 1)][rb], acc[rb][nb], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // every wave has read this stage: it may be refilled with the piece after next
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (pc + 2 < n_pieces) issue_piece(pc + 2);
    // This wave's transfers of the next piece have landed once at most the ones just issued are outstanding
    // (loads complete in order; the stores of the last epilogue were issued before them and do not matter).
    if (pc + 1 < n_pieces) {
      if (pc + 2 < n_pieces) ws_wait_vmcnt<NDW>();
      else ws_wait_vmcnt<0>();
    }
    // ---- epilogue of this piece ----
    // The weights are the first MFMA operand, so the product comes out transposed: lane l32 holds row l32 of the
    // piece and accumulator element i the column (i / 4) * 8 + lh * 4 + i % 4 of the 32-column block, i.e. four
    // consecutive columns per group of four elements.  They go as 8-byte pieces into a strip of LDS private to
    // the wave and leave it as 16-byte pieces along the rows (eight lanes write one 128-byte line; 8-byte
    // stores straight from the registers touch 32 lines per instruction and were measured slower).
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int j4 = 0; j4 < 4; ++j4) {
          bf16_t v[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = f32_to_bf16(acc[rb][nb][j4 * 4 + q]);
          *reinterpret_cast<uint2*>(strip_lds + l32 * WS_STRIP_LD + nb * 32 + j4 * 8 + lh * 4) = *reinterpret_cast<const uint2*>(v);
        }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the strip is private to this wave
#pragma unroll
      for (int q = lane; q < 32 * 8; q += 64) {
        const int rr = q >> 3, cc = q & 7;
        const int r = pc * PR + rb * 32 + rr;
        const uint4 v = *reinterpret_cast<const uint4*>(strip_lds + rr * WS_STRIP_LD + cc * 8);
        if (r < rows) *reinterpret_cast<uint4*>(ybase + (int64_t)r * p.d + cc * 8) = v;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    // all waves' parts of the next piece are in LDS
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1))) void ws_down_kernel(WsArgs p) {
  extern __shared__ __attribute__((aligned(16))) char ws_smem[];
  const int n_work = p.work[p.G];
  int wid = blockIdx.x;
  if (p.xcd_remap) {
    const int first = p.work[p.G + 1 + (wid & 7)], end = p.work[p.G + 2 + (wid & 7)];
    wid = first + (wid >> 3);
    if (wid >= end) return;
  }
  if (wid >= n_work) return;
  const int g = find_group(p.work, p.G, wid);
  const int local = wid - p.work[g];
  const int seg0 = p.seg_off[g];
  const int cnt = p.seg_off[g + 1] - seg0;
  const int64_t hoff = p.h_off[g];
  switch (p.groups[g].width_pad) {
    case 352: ws_down_item<22, 2>(p, g, local, seg0, cnt, hoff, ws_smem); break;
    case 448: ws_down_item<28, 2>(p, g, local, seg0, cnt, hoff, ws_smem); break;
    case 704: ws_down_item<44, 1>(p, g, local, seg0, cnt, hoff, ws_smem); break;
    default: break;                                            // the general kernel runs this group
  }
}

bool ws_down_handles(int width_pad) { return width_pad == 352 || width_pad == 448 || width_pad == 704; }

hipError_t launch_ws_down(const Engine& e, char* ws, const WsLayout& L, const void* y_slots, int rc, int n_blocks,
                          int xcd_remap, hipStream_t s) {
  static bool attr_done = false;
  constexpr int smem = ws_smem_bytes(22, 2) > ws_smem_bytes(28, 2)
                           ? (ws_smem_bytes(22, 2) > ws_smem_bytes(44, 1) ? ws_smem_bytes(22, 2) : ws_smem_bytes(44, 1))
                           : (ws_smem_bytes(28, 2) > ws_smem_bytes(44, 1) ? ws_smem_bytes(28, 2) : ws_smem_bytes(44, 1));
  if (!attr_done) {
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(ws_down_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (err != hipSuccess) return err;
    attr_done = true;
  }
  WsArgs a;
  a.H = reinterpret_cast<const bf16_t*>(ws + L.h);
  a.W2 = static_cast<const bf16_t*>(e.w2);
  a.Y = reinterpret_cast<bf16_t*>(const_cast<void*>(y_slots));
  a.groups = e.groups;
  a.seg_off = reinterpret_cast<const int32_t*>(ws + L.seg_off);
  a.work = reinterpret_cast<const int32_t*>(ws + L.work2);
  a.h_off = reinterpret_cast<const int64_t*>(ws + L.h_off);
  a.G = e.G;
  a.d = e.d;
  a.rc = rc;
  a.xcd_remap = xcd_remap;
  hipLaunchKernelGGL(ws_down_kernel, dim3((unsigned)n_blocks), dim3(256), smem, s, a);
  return hipGetLastError();
}

}  // namespace cmoe
