// Grouped SwiGLU expert kernels for bf16 layers (Eq. 3 restricted to an expert's neurons):
//   MODE 1  H_g = Swish(X_g Wgate_g) * (X_g Wup_g)     rows of X gathered through slot2tok, K = d
//   MODE 2  Y_g = H_g Wdown_g                          K = width_pad(g), N = d
// Both are C = A * B^T with K contiguous in A and in B, computed with v_mfma_f32_32x32x16_bf16 from
// LDS-staged, XOR-swizzled tiles filled by direct global->LDS loads.  A work item is (group, row tile, column tile); the list of work
// items is a device-side prefix array written by the permute kernel, so ragged, empty and skewed
// groups need no host round trip.  Workgroups whose index is past the list exit at once.
#include <algorithm>
#include <cstdlib>
#include <type_traits>
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
  int ldb;                   // elements per row of B in MODE 1 (packed gate/up rows)
  int b_tiled;               // 1: the weight matrices are tiled 16 x 32 (see cmoe_internal.h)
  int64_t T;
  int single;                // 1: one always-on group holding all T tokens; no device schedule is read
  int n_blocks;              // grid size (multiple of 8) before the K split
  int xcd_remap;             // 1: consecutive work items run on the same XCD
  int zero_pad;              // 1: tile rows past the end of a group read zeros instead of repeating its last row
  int ws_skip;               // 1 (down contraction): groups the weight-stationary kernel handles are left to it
  // K split: k_split > 1 workgroups share one tile, each multiplies a contiguous range of K tiles and
  // stores its fp32 partial sums to P [k_split][p_rows][ldp] (row = slot, column = column of the tile
  // grid); a finishing kernel adds the parts in order and applies the epilogue.  Used when a launch has
  // too few tiles to fill the chip (batches of a few hundred tokens).
  int k_split;
  float* P;
  int64_t p_rows;
  int ldp;
};

// ---- global->LDS loads and a ring of K tiles ------------------------------------------------------
// Each global_load_lds_dwordx4 moves 64 lanes x 16 bytes into 1 KB of consecutive LDS (8 tile rows);
// which global chunk a lane fetches is free, so the XOR swizzle is applied on the global side.  No
// VGPRs are spent on staging, and STAGES-1 tiles are in flight while one is multiplied.
__device__ __attribute__((aligned(16))) uint32_t g_zero_chunk[4] = {0, 0, 0, 0};
// A row of zeros as long as any K this file meets in practice.  Tile rows past the end of a group (ragged
// expert segments fill their last row tile to 50 % on average) read it instead of a real row: the result
// rows are discarded either way, but an MFMA whose operand is all zeros draws less power than one on real
// data, and on this part the clock under MFMA load is set by power.
constexpr int ZERO_ROW_ELEMS = 32768;
__device__ __attribute__((aligned(256))) bf16_t g_zero_row[ZERO_ROW_ELEMS];


template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ void dma16(const void* gsrc, bf16_t* lds_dst) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gsrc),
                                   (__attribute__((address_space(3))) void*)(lds_dst), 16, 0, 0);
}

// LDS tile [rows][BKT] of bf16, 16-byte chunks XOR-swizzled so that the 16 rows one quarter of a
// ds_read_b128 touches fall into 16 different 16-byte bank groups (256 bytes = all 64 banks).
template <int BKT>
__device__ __forceinline__ int lds_off_t(int row, int c) {
  if (BKT == 64) return row * 64 + ((c ^ ((row >> 1) & 7)) << 3);
  return row * 32 + ((c ^ ((row >> 2) & 3)) << 3);
}

// Waves per SIMD the register allocation has to leave room for: two when two four-wave workgroups fit a CU's
// 160 KB of LDS (the compiler otherwise spends up to 512 registers on a wave that is alone on its SIMD).
constexpr int min_waves_per_simd(int bm, int bn, int bkt, int stages, int nw) {
  return (stages >= 2 && nw == 4 && bm * bn >= 256 * 128 && stages * (bm + bn) * bkt * 2 <= 80 * 1024) ? 2 : 1;
}

// DYN: the number of 32-row blocks of the tile that hold rows of the segment is found at run time and the rest
// of the kernel runs in the instantiation for exactly that many blocks per wave (MI_ACT below; the blocks are
// dealt to the WGM wave rows in turn): blocks past the end of a ragged segment are neither fetched nor
// multiplied, so a tile costs what its rows cost, in steps of 32 * WGM rows.
template <int BM, int BN, int BKT, int STAGES, int WGM, int WGN, int MODE, bool DYN = false>
__global__ __launch_bounds__(WGM* WGN * 64)
__attribute__((amdgpu_waves_per_eu(min_waves_per_simd(BM, BN, BKT, STAGES, WGM* WGN)))) void grouped_gemm_bf16_dma(GemmArgs p) {
  constexpr int NW = WGM * WGN;
  constexpr int TM = BM / WGM, TN = BN / WGN, MI = TM / 32, NI = TN / 32;
  constexpr int CPR = BKT / 8;                                  // 16-byte chunks per tile row
  constexpr int RPI = 64 / CPR;                                 // tile rows one 1 KB DMA instruction fills
  constexpr int A_CH = BM / RPI / NW, B_CH = BN / RPI / NW;     // DMA instructions per wave and tile
  constexpr int LPT = A_CH + B_CH;
  constexpr int STAGE_ELEMS = (BM + BN) * BKT;
  constexpr int SWZ_SHIFT = (BKT == 64) ? 1 : 2;
  // STAGES >= 2: ring of whole K tiles (A part + B part).  STAGES == 0: ring of five half tiles in the order
  // A(0) B(0) A(1) B(1) ...: while tile kt is multiplied, B(kt+1) and A(kt+2) are fetched into the two
  // halves tile kt-1 just released, and A(kt+1) is already resident, so only half a tile has to land
  // within one K step although 2.5 tiles of LDS are in use.
  constexpr bool HR = (STAGES == 0);
  constexpr int HALF = (BM > BN ? BM : BN) * BKT;
  constexpr int RING_ELEMS = HR ? 5 * HALF : STAGES * STAGE_ELEMS;
  static_assert(BKT == 32 || BKT == 64, "K tile");
  static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "loader");
  static_assert(MODE != 1 || TN % 64 == 0, "gate/up pairs must stay inside a wave tile");
  static_assert(HR || (STAGES >= 2 && (STAGES - 2) * LPT < 64), "ring depth");
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: LDS destinations stay scalar
  const int wm = wave / WGN, wn = wave % WGN;
  const int l32 = lane & 31, lh = lane >> 5;

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
  // Workgroup b runs on XCD b % 8 (own L2).  Each XCD works through a contiguous range of the list so that
  // tiles sharing an operand meet in one L2: equal parts of a single-group problem, and for work lists the
  // shares of equal estimated cost that the permutation kernel left behind the prefix array.
  int wid = blockIdx.x;
  int k_part = 0;
  if (p.k_split > 1) {
    k_part = wid % p.k_split;
    wid /= p.k_split;
  }
  if (p.xcd_remap) {
    if (p.single) {
      const int chunk = (n_work + 7) >> 3;
      if ((wid >> 3) >= chunk) return;
      wid = (wid & 7) * chunk + (wid >> 3);
    } else {
      const int first = p.work[p.G + 1 + (wid & 7)], end = p.work[p.G + 2 + (wid & 7)];
      wid = first + (wid >> 3);
      if (wid >= end) return;
    }
  }
  if (wid >= n_work) return;
  int local = wid;
  if (!p.single) {
    g = find_group(p.work, p.G, wid);
    local = wid - p.work[g];
    seg0 = p.seg_off[g];
    cnt = p.seg_off[g + 1] - seg0;
    wp = p.groups[g].width_pad;
    hoff = p.h_off[g];
    if (MODE == 2 && p.ws_skip && (wp == 352 || wp == 448 || wp == 704)) return;
  }
  // this workgroup's range of K tiles (all of them without a K split); from here on K and the tile
  // index count from the start of that range and the source pointers are shifted accordingly
  const int K_full = (MODE == 1) ? p.d : wp;
  int K = K_full, k_first = 0;
  if (p.k_split > 1) {
    const int kt_all = (K_full + BKT - 1) / BKT;
    const int per = (kt_all + p.k_split - 1) / p.k_split;
    k_first = (k_part * per < kt_all ? k_part * per : kt_all) * BKT;
    const int k_end = ((k_part + 1) * per < kt_all) ? (k_part + 1) * per * BKT : K_full;
    K = k_end > k_first ? k_end - k_first : 0;
  }
  const int n_cols = (MODE == 1) ? 2 * wp : p.d;
  const int n_nt = (n_cols + BN - 1) / BN;
  const int n_mt = (cnt + BM - 1) / BM;
  constexpr int GM = 8;
  const int sr = local / (GM * n_nt);
  const int rem = local - sr * (GM * n_nt);
  const int rows_in_sr = (n_mt - sr * GM) < GM ? (n_mt - sr * GM) : GM;
  const int mt = sr * GM + rem % rows_in_sr;
  const int nt = rem / rows_in_sr;

  using std::integral_constant;
  using std::false_type;
  using std::true_type;
  auto body = [&](auto act_tag) {
  constexpr int MI_ACT = decltype(act_tag)::value;              // 32-row blocks per wave that are computed
  // tile rows that are fetched: with a dynamic height the 32-row blocks of the tile are dealt to the WGM wave
  // rows in turn (wave row wm owns blocks wm, wm + WGM, ...), so MI_ACT blocks per wave cover the first
  // MI_ACT * WGM blocks of the tile; DMA instructions per wave that cover them:
  constexpr int A_ACT = DYN ? (MI_ACT * WGM * 32 + RPI * NW - 1) / (RPI * NW) : A_CH;
  auto row_block = [&](int mi) { return DYN ? mi * WGM + wm : wm * MI + mi; };
  constexpr int LPT_ACT = A_ACT + B_CH;
  // every offset a row source is read at stays below K_full rounded up to a whole K tile
  const bool use_zero_row = p.zero_pad && K_full + BKT <= ZERO_ROW_ELEMS;
  // per-lane sources: transfer i of this wave covers tile rows rg*8 .. rg*8+7, rg = wave + i*NW; the lane
  // writes physical chunk lane%8 of row rg*8 + lane/8 and therefore fetches logical chunk (lane%8) ^ swz(row)
  const bf16_t* a_src[A_ACT];
  const bf16_t* b_src[B_CH];
  int a_coff[A_ACT], b_coff[B_CH];                      // element offset of the lane's chunk inside a 64-wide K tile
#pragma unroll
  for (int i = 0; i < A_ACT; ++i) {
    const int row = (wave + i * NW) * RPI + lane / CPR;
    a_coff[i] = (((lane % CPR) ^ ((row >> SWZ_SHIFT) & (CPR - 1))) << 3);
    int r = mt * BM + row;
    const bool past = r >= cnt;
    if (past) r = cnt - 1;
    if (MODE == 1) {
      const int64_t tok = p.slot2tok ? p.slot2tok[seg0 + r] : (seg0 + r);
      a_src[i] = p.A + tok * p.d + a_coff[i] + k_first;
    } else {
      a_src[i] = p.A + hoff + (int64_t)r * wp + a_coff[i] + k_first;
    }
    if (past && use_zero_row) a_src[i] = g_zero_row + a_coff[i] + k_first;
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int row = (wave + i * NW) * RPI + lane / CPR;
    b_coff[i] = (((lane % CPR) ^ ((row >> SWZ_SHIFT) & (CPR - 1))) << 3);
    int n = nt * BN + row;
    const bool past = n >= n_cols;
    if (past) n = n_cols - 1;
    if (p.b_tiled) {
      // the lane's chunk of K tile kt lies 64 / 32 = 2 tiles (BKT / TILE_K) further for every kt
      const int64_t rowg = (MODE == 1) ? (int64_t)p.groups[g].w1_row0 + n : n;
      const int64_t base = (MODE == 1) ? 0 : p.groups[g].w2_off;
      const int kt32 = (MODE == 1) ? p.ldb / TILE_K : wp / TILE_K;
      b_src[i] = p.B + base + tiled_offset(rowg, k_first + b_coff[i], kt32);
    } else {
      if (MODE == 1) b_src[i] = p.B + ((int64_t)p.groups[g].w1_row0 + n) * p.ldb + b_coff[i] + k_first;
      else b_src[i] = p.B + p.groups[g].w2_off + (int64_t)n * wp + b_coff[i] + k_first;
      if (past && use_zero_row) b_src[i] = g_zero_row + b_coff[i] + k_first;
    }
  }
  const int b_adv = p.b_tiled ? (BKT / TILE_K) * TILE_ELEMS : BKT;     // elements between a lane's chunks of two K tiles
  const int KT = (K + BKT - 1) / BKT;
  const bool k_ragged = (K % BKT) != 0;
  auto a_slot = [&](int kt) -> bf16_t* { return HR ? smem + ((2 * kt) % 5) * HALF : smem + (kt % (HR ? 1 : STAGES)) * STAGE_ELEMS; };
  auto b_slot = [&](int kt) -> bf16_t* {
    return HR ? smem + ((2 * kt + 1) % 5) * HALF : smem + (kt % (HR ? 1 : STAGES)) * STAGE_ELEMS + BM * BKT;
  };
  // one DMA instruction (index i of this wave's share) of the A or B part of tile kt
  // `maybe_last`: the tile may be the last one of a K that is not a multiple of the tile depth; its chunks
  // past K come from a block of zeros instead.  Steady-state steps never fetch the last tile and skip the test.
  auto issue_a = [&](int kt, int i, bool maybe_last) {
    const void* src = a_src[i] + kt * BKT;
    if (maybe_last && k_ragged && kt == KT - 1 && kt * BKT + a_coff[i] >= K) src = g_zero_chunk;
    dma16(src, a_slot(kt) + (wave + i * NW) * RPI * BKT);
  };
  auto issue_b = [&](int kt, int i, bool maybe_last) {
    const void* src = b_src[i] + kt * b_adv;
    if (maybe_last && k_ragged && kt == KT - 1 && kt * BKT + b_coff[i] >= K) src = g_zero_chunk;
    dma16(src, b_slot(kt) + (wave + i * NW) * RPI * BKT);
  };
  auto issue_tile_a = [&](int kt) {
#pragma unroll
    for (int i = 0; i < A_ACT; ++i) issue_a(kt, i, true);
  };
  auto issue_tile_b = [&](int kt) {
#pragma unroll
    for (int i = 0; i < B_CH; ++i) issue_b(kt, i, true);
  };

  floatx16_t acc[MI_ACT][NI];
#pragma unroll
  for (int mi = 0; mi < MI_ACT; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.0f;

  // prologue (a K part can be empty when the split does not divide the K tiles)
  if (HR) {
    if (KT > 0) {
      issue_tile_a(0);
      issue_tile_b(0);
    }
    if (KT > 1) issue_tile_a(1);
  } else {
#pragma unroll
    for (int st = 0; st < STAGES - 1; ++st)
      if (st < KT) { issue_tile_a(st); issue_tile_b(st); }
  }

  // One K tile: wait for it and multiply it while the loads that run ahead are issued.  AHEAD is a
  // compile-time count of what is still to be fetched, so the whole step is straight-line code:
  //   whole-tile ring: 1 = fetch tile kt+STAGES-1, 0 = nothing left
  //   half-tile ring : 2 = fetch B(kt+1) and A(kt+2), 1 = fetch B(kt+1) only, 0 = last tile
  // Instruction order inside the step is fixed by hand: memory instructions never follow one another.
  // After each MFMA comes at most one LDS fragment read of the next sub-step and at most one DMA
  // instruction, the DMA instructions spread evenly over all MFMAs of the step.  A wave that issues memory
  // instructions back to back waits for the queue to take them and cannot issue its MFMAs meanwhile
  // (measured on a skeleton of this loop: 3030 cycles per step with clustered reads, 2620 interleaved).
  auto k_tile = [&](int kt, auto ahead_tag, auto last_tag) {
    constexpr int AHEAD = decltype(ahead_tag)::value;
    constexpr bool MAYBE_LAST = decltype(last_tag)::value;   // a tile fetched in this step may be tile KT-1
    if (HR) {
      if (AHEAD >= 1) wait_vmcnt<A_ACT>();           // A(kt+1) may still be in flight; A(kt), B(kt) are older
      else wait_vmcnt<0>();
    } else {
      if (AHEAD >= 1) wait_vmcnt<HR ? 0 : (STAGES - 2) * LPT_ACT>();
      else wait_vmcnt<0>();
    }
    // Bare barrier: __syncthreads() would add a fence that drains every outstanding load (vmcnt(0)) and with
    // it the loads running ahead.  What the barrier has to order is covered by hand: this wave's parts of
    // tile kt have landed (vmcnt above), and its LDS reads of tile kt-1 were consumed by MFMAs already.
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");                   // all lanes' parts landed; the slots of tile kt-1 are free
    const bf16_t* as = a_slot(kt);
    const bf16_t* bs = b_slot(kt);
    constexpr int NKS = BKT / 16;                    // sub-steps (one MFMA depth each)
    constexpr int NMS = MI_ACT * NI;                 // MFMAs per sub-step
    constexpr int NM = NKS * NMS;                    // MFMAs per step
    // DMA instructions of this step, in issue order: half ring B(kt+1) then A(kt+2); whole ring A then B
    constexpr int N_FIRST = HR ? B_CH : A_ACT;
    constexpr int L = A_ACT + B_CH;
    auto issue_nth = [&](int i) {
      if (HR) {
        if (i < N_FIRST) issue_b(kt + 1, i, MAYBE_LAST);
        else if (AHEAD >= 2) issue_a(kt + 2, i - N_FIRST, MAYBE_LAST);
      } else {
        if (i < N_FIRST) issue_a(kt + STAGES - 1, i, MAYBE_LAST);
        else issue_b(kt + STAGES - 1, i - N_FIRST, MAYBE_LAST);
      }
    };
    // Fragments of a sub-step in the order of their first use by its MFMAs (row block mi is first needed by
    // MFMA mi * NI, column block ni by MFMA ni): A0, B0 .. B(NI-1), A1, A2, ...  LDS reads complete in issue
    // order, so the wait in front of an MFMA covers exactly the reads issued up to its own operands; with the
    // B fragments last, the first MFMA of every sub-step waited for all of them.
    bf16x8_t af[2][MI_ACT], bfr[2][NI];
    auto load_frag = [&](int ks, int k, int set) {
      const int mi = k == 0 ? 0 : k - NI;               // valid when k == 0 or k > NI
      if (k == 0 || k > NI) af[set][mi] = *reinterpret_cast<const bf16x8_t*>(as + lds_off_t<BKT>(row_block(mi) * 32 + l32, ks * 2 + lh));
      else bfr[set][k - 1] = *reinterpret_cast<const bf16x8_t*>(bs + lds_off_t<BKT>(wn * TN + (k - 1) * 32 + l32, ks * 2 + lh));
    };
#pragma unroll
    for (int f = 0; f < MI_ACT + NI; ++f) load_frag(0, f, 0);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const int cur = ks & 1;
#pragma unroll
      for (int j = 0; j < NMS; ++j) {
        const int mi = j / NI, ni = j % NI;
        __builtin_amdgcn_sched_barrier(0);
        // (down contraction: operands swapped, so that the accumulator block is the transpose: a lane then holds
        // four consecutive output columns of one row instead of one column of sixteen rows, and the epilogue
        // stages 8-byte pieces instead of single elements; same products, same order of accumulation)
        if constexpr (MODE == 2) acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][ni], af[cur][mi], acc[mi][ni], 0, 0, 0);
        else acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][mi], bfr[cur][ni], acc[mi][ni], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        // fragments of the next sub-step, spread over this sub-step's MFMAs (several per MFMA only when
        // a sub-step has fewer MFMAs than fragments)
#pragma unroll
        for (int f = 0; f < MI_ACT + NI; ++f)
          if (ks + 1 < NKS && f * NMS / (MI_ACT + NI) == j) load_frag(ks + 1, f, cur ^ 1);
        if (AHEAD >= 1) {
          const int m = ks * NMS + j;
          // (a skinny tile has more DMA instructions than MFMAs: then several follow one MFMA)
#pragma unroll
          for (int i = 0; i < L; ++i)
            if (L > NM ? (i * NM / L == m) : ((i + 1) * NM / L - 1 == m)) issue_nth(i);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  int kt = 0;
  if (HR) {
    for (; kt + 3 < KT; ++kt) k_tile(kt, integral_constant<int, 2>{}, false_type{});   // fetches B(kt+1), A(kt+2)
    for (; kt + 2 < KT; ++kt) k_tile(kt, integral_constant<int, 2>{}, true_type{});    // A(KT-1)
    for (; kt + 1 < KT; ++kt) k_tile(kt, integral_constant<int, 1>{}, true_type{});    // B(KT-1)
    for (; kt < KT; ++kt) k_tile(kt, integral_constant<int, 0>{}, false_type{});
  } else {
    constexpr int S1 = (HR ? 2 : STAGES) - 1;             // a step fetches tile kt+S1
    for (; kt + S1 + 1 < KT; ++kt) k_tile(kt, integral_constant<int, 1>{}, false_type{});
    for (; kt + S1 < KT; ++kt) k_tile(kt, integral_constant<int, 1>{}, true_type{});
    for (; kt < KT; ++kt) k_tile(kt, integral_constant<int, 0>{}, false_type{});
  }

  // ---- K split: the raw fp32 partial sums go to this part's slab; 32 consecutive lanes hold 32
  // consecutive columns of a row, so the stores are 128-byte segments ----
  if (p.k_split > 1) {
    float* slab = p.P + (int64_t)k_part * p.p_rows * p.ldp;
    if constexpr (MODE == 2) {
      // transposed accumulator blocks: element i of block (mi, ni) = row l32 of the row block, column
      // (i / 4) * 8 + lh * 4 + i % 4 of the column block; four consecutive columns per 16-byte store
      // (the slab's row stride is d, a multiple of 8)
#pragma unroll
      for (int mi = 0; mi < MI_ACT; ++mi) {
        const int r = mt * BM + row_block(mi) * 32 + l32;
        if (r >= cnt) continue;
        float* prow = slab + (int64_t)(seg0 + r) * p.ldp;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int col = nt * BN + wn * TN + ni * 32 + q * 8 + lh * 4;
            if (col < n_cols)
              *reinterpret_cast<float4*>(prow + col) =
                  make_float4(acc[mi][ni][4 * q], acc[mi][ni][4 * q + 1], acc[mi][ni][4 * q + 2], acc[mi][ni][4 * q + 3]);
          }
      }
      return;
    }
#pragma unroll
    for (int mi = 0; mi < MI_ACT; ++mi)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int r = mt * BM + row_block(mi) * 32 + (i / 4) * 8 + lh * 4 + (i % 4);
        if (r >= cnt) continue;
        float* prow = slab + (int64_t)(seg0 + r) * p.ldp;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
          const int col = nt * BN + wn * TN + ni * 32 + l32;
          if (col < n_cols) prow[col] = acc[mi][ni][i];
        }
      }
    return;
  }
  // ---- epilogue: through LDS, so that global stores are 16-byte vectors along the rows ----
  // Each wave stages 32 rows of its tile at a time in a private LDS strip (row stride padded by 16 bytes
  // against bank conflicts), then every lane copies 16-byte pieces of rows out to global memory.
  constexpr int TNO = (MODE == 1) ? TN / 2 : TN;          // output columns of a wave tile
  constexpr int LDO = TNO + 8;                            // strip row stride in elements
  constexpr int CPRO = TNO / 8;                           // 16-byte pieces per strip row
  static_assert(NW * 32 * LDO <= RING_ELEMS, "epilogue strip must fit in the tile ring");
  __syncthreads();                                        // every wave is done reading the last tile
  bf16_t* strip = smem + wave * 32 * LDO;
  const int out_col0 = (MODE == 1) ? (nt * BN + wn * TN) / 2 : nt * BN + wn * TN;
  const int out_cols = (MODE == 1) ? wp : p.d;
  bf16_t* out_base = (MODE == 1) ? p.C + hoff : p.C + (int64_t)seg0 * p.d;
  const int64_t out_ld = (MODE == 1) ? wp : p.d;
#pragma unroll
  for (int mi = 0; mi < MI_ACT; ++mi) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int rr = (i / 4) * 8 + lh * 4 + (i % 4);
      if constexpr (MODE == 1) {
#pragma unroll
        for (int pi = 0; pi < NI / 2; ++pi) {
          const float gt = acc[mi][2 * pi][i], up = acc[mi][2 * pi + 1][i];
          // Swish(g) * u with the hardware exponential: the result is rounded to bf16 right after
          const float sg = gt * __frcp_rn(1.0f + __expf(-gt));
          strip[rr * LDO + pi * 32 + l32] = f32_to_bf16(sg * up);
        }
      }
    }
    if constexpr (MODE == 2) {
      // transposed blocks (see the MFMA above): this lane's row of the strip is l32, and every group of four
      // accumulator elements is four consecutive columns: one 8-byte LDS write each
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          ushort4 v;
          v.x = f32_to_bf16(acc[mi][ni][4 * q]);
          v.y = f32_to_bf16(acc[mi][ni][4 * q + 1]);
          v.z = f32_to_bf16(acc[mi][ni][4 * q + 2]);
          v.w = f32_to_bf16(acc[mi][ni][4 * q + 3]);
          *reinterpret_cast<ushort4*>(strip + l32 * LDO + ni * 32 + q * 8 + lh * 4) = v;
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");    // the strip is private to this wave: no barrier
#pragma unroll
    for (int q = lane; q < 32 * CPRO; q += 64) {
      const int rr = q / CPRO, cc = q % CPRO;
      const int r = mt * BM + row_block(mi) * 32 + rr;
      const int col = out_col0 + cc * 8;
      const uint4 v = *reinterpret_cast<const uint4*>(strip + rr * LDO + cc * 8);
      if (r < cnt && col < out_cols) *reinterpret_cast<uint4*>(out_base + (int64_t)r * out_ld + col) = v;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");    // reads done before the strip is overwritten
  }
};   // body
  if constexpr (DYN) {
    const int rows_here = cnt - mt * BM;
    const int nb = rows_here >= BM ? MI : ((rows_here + 31) / 32 + WGM - 1) / WGM;      // blocks per wave row
    switch (nb) {
      case 1: body(integral_constant<int, 1>{}); break;
      case 2: if constexpr (MI >= 2) body(integral_constant<int, 2>{}); break;
      case 3: if constexpr (MI >= 3) body(integral_constant<int, 3>{}); break;
      case 4: if constexpr (MI >= 4) body(integral_constant<int, 4>{}); break;
      case 5: if constexpr (MI >= 5) body(integral_constant<int, 5>{}); break;
      case 6: if constexpr (MI >= 6) body(integral_constant<int, 6>{}); break;
      case 7: if constexpr (MI >= 7) body(integral_constant<int, 7>{}); break;
      default: body(integral_constant<int, MI>{}); break;
    }
  } else {
    body(integral_constant<int, MI>{});
  }
}

// ---- tile configurations ---------------------------------------------------------------------
// Tile shapes (the tuning switches gemm1_cfg / gemm2_cfg select one by index).
// stages >= 2: ring of whole K tiles; stages == 0: ring of five half tiles.
struct TileCfg { int bm, bn, wgm, wgn, stages, bk; };
static const TileCfg kCfgs[] = {
    {256, 256, 2, 4, 0, 64},   // 0: half-tile ring, eight waves of 128x64
    {128, 128, 2, 2, 2, 64},   // 1: two stages, two workgroups per CU
    {256, 256, 2, 4, 2, 64},   // 2
    {128, 128, 2, 2, 0, 64},   // 3
    {256, 128, 4, 2, 3, 64},   // 4
    {256, 256, 2, 4, 4, 32},   // 5
    {256, 256, 2, 2, 0, 64},   // 6: half-tile ring, four waves of 128x128, one per SIMD: a third less LDS read
                               //    traffic than 0, 5-8 % faster under the power limit (the large-tile default)
    {64, 128, 2, 2, 4, 64},    // 7: skinny tile for batches of tens of tokens per group, four whole K tiles deep: a
                               //    CU keeps 72 KB of loads in flight, two thirds of them weights (such a launch
                               //    is bound by HBM latency x bytes in flight, not by MFMA work).  Measured against
                               //    32x128 (2 waves; 3 and 7 stages), 32x256 and 64x128 with 3 and 6 stages.
    {128, 256, 2, 2, 3, 32},   // 8: four waves of 64x128, three K tiles of 32: 72 KB of LDS and at most 256 registers,
                               //    so two workgroups share a CU and one's epilogue overlaps the other's K loop
                               //    (the short-K down contraction; 256x128 in the same arrangement was slower)
    {224, 256, 1, 4, 0, 64},   // 9: four waves of 224x64 (all rows, a quarter of the columns each): 7/8 of the
                               //    MFMA work of 6 per tile, for segments that fill 256-row tiles poorly
    {192, 256, 1, 4, 0, 64},   // 10: four waves of 192x64
    {256, 256, 1, 4, 0, 64},   // 11: four waves of 256x64 with a dynamic tile height (DYN): a ragged segment's last tile
                               //     costs its rows in steps of 32, so the tallest tile wastes the least
    {128, 256, 1, 4, 3, 32},   // 12: the arrangement of 8 (two workgroups per CU, three K tiles of 32) with four waves
                               //     of 128x64 and a dynamic tile height
    {256, 256, 2, 2, 0, 64},   // 13: shape 6 (four waves of 128x128) with a dynamic tile height in steps of 64 rows: a
                               //     wave reads each A fragment for 128 columns, which the LDS keeps up with; four
                               //     waves of 256x64 (11) read a quarter more and are bound by it
    {128, 256, 2, 2, 3, 32},   // 14: shape 8 with a dynamic tile height in steps of 64 rows
    // 15-18: the weight-stationary down contraction (ws_down.hip): work items of 128 / 256 / 512 / 1024 rows x 256 columns,
    // cost in steps of 64 rows; groups it has no instantiation for run shape 8 (128 rows) or 6 (256 rows) over
    // the same list
    {128, 256, 2, 2, 3, 32},
    {256, 256, 2, 2, 0, 32},
    {512, 256, 2, 2, 0, 32},
    {1024, 256, 2, 2, 0, 32},  // 18: the same with 1024 rows per item
};
static bool cfg_is_ws(int ci) { return ci >= 15 && ci <= 18; }
static bool cfg_is_dyn(int ci) { return ci >= 11 && ci <= 18; }
bool ws_down_handles(int width_pad);
hipError_t launch_ws_down(const Engine& e, char* ws, const WsLayout& L, const void* y_slots, int rc, int n_blocks,
                          int xcd_remap, hipStream_t s);
constexpr int kNumCfgs = sizeof(kCfgs) / sizeof(kCfgs[0]);

// Which tile shape for contraction `which` (1: gate/up, 2: down) of a batch of T tokens: the tuning switches
// gemm1_cfg / gemm2_cfg when set, else the models below.
// Tile shape of the gate/up contraction: the one with the lowest estimated time = rounds x time per round,
// rounds = ceil(tiles / workgroup slots on the chip).  Relative times per round measured on the
// LLaMA-shaped layers (K = d for every shape, so the ratios carry over), in units of the eight-wave
// 256x256 tile: 256x256 with four waves 0.95 (one workgroup per CU), 256x128 0.58 (one per CU), 128x128
// 0.66 (two per CU), 64x128 0.30 (one per CU; it only wins while the launch is one or two rounds, i.e. up to
// 128 tokens for the dense FFN and about 200 for the 16-expert layer).  224x256 and 192x256 tiles (four waves
// side by side, each over all rows of the tile: a quarter more LDS reads per MFMA than 128x128 per wave) take
// 0.875 and 0.81: when ragged segments fill 256-row tiles poorly, a lower tile with the same number of rounds
// does less padded work (16 experts at 4096 tokens: 820 rows are four tiles either way, 204 -> 187 us).
// The model picks the measured best shape at every batch size from 33 to 8192 tokens or one within a few
// per cent of it.
static int gate_up_cfg(const Engine& e, int64_t T) {
  struct Cand { int cfg, bm, bn, slots; double t; };
  const bool single = e.G == 1 && e.n_always == 1;
  const Cand cands[] = {{3, 128, 128, 2, 0.66}, {4, 256, 128, 1, 0.58}, {6, 256, 256, 1, 0.95}, {7, 64, 128, 1, 0.30},
                        {9, 224, 256, 1, 0.875}, {10, 192, 256, 1, 0.81}};
  int best = 0;
  double best_t = 1e30;
  for (const Cand& c : cands) {
    // a tile of 192 rows or more for groups that average less than a quarter of it streams its weights at the
    // pace of a full tile (measured with 256 rows at 224-256 tokens on 16 experts: 61 us against 52 us with
    // 128x128)
    if (!single && c.bm >= 192 && T * e.S_dyn * 4 < (int64_t)std::min<int64_t>(e.G - e.n_always, T * e.S_dyn) * c.bm) continue;
    int64_t tiles = 0;
    for (int g = 0; g < e.n_always; ++g) tiles += ((T + c.bm - 1) / c.bm) * cdiv(2 * e.width_pad_host[g], c.bn);
    if (!single && e.G > e.n_always) {
      const int64_t entries = T * e.S_dyn;
      const int64_t touched = std::min<int64_t>(e.G - e.n_always, entries);
      const int64_t rows = std::max<int64_t>((entries + c.bm - 1) / c.bm + touched / 2, touched);
      tiles += rows * cdiv(2 * e.width_pad_host[e.n_always], c.bn);
    }
    // the routed groups' partial tiles are an estimate: average over the estimate and 8 % more
    const int64_t slots = 256 * c.slots, hi = single ? tiles : tiles + (tiles * 2 + 24) / 25;
    double t = 0.5 * c.t * (double)((tiles + slots - 1) / slots + (hi + slots - 1) / slots);
    // the skinny tile runs one workgroup per CU and its rounds are long: when the estimate is within 8 % of
    // spilling into a second, nearly empty round, count that round in full
    if (c.cfg == 7 && !single && tiles <= slots && hi > slots) t = 2.3 * c.t;      // (above one round of 128x128)
    if (t < best_t) {
      best_t = t;
      best = c.cfg;
    }
  }
  return best;
}

static int64_t est_tiles(const Engine& e, int64_t T, int which, int bm, int bn);

static int cfg_index(int which, const Engine& e, int64_t T) {
  int dflt = 0;
  if (which == 1) dflt = gate_up_cfg(e, T);
  if (which == 2) {
    const bool single = e.G == 1 && e.n_always == 1;
    int k_min = 1 << 30;
    for (int g = 0; g < e.G; ++g) k_min = std::min(k_min, e.width_pad_host[g]);
    if (!single && k_min < 2048) {
      // Short K (an expert's width, up to a few tens of K steps per tile; a wider merged shared group next to
      // such experts does not change the picture): rounds x time per round, rounds = ceil(tiles /
      // workgroup slots on the chip).  Measured on 8 to 64 experts of 352 to 1792 neurons, 128 to 8192 tokens:
      // a round of 256 tiles of 256x256 (eight waves, one workgroup per CU) and a round of 512 tiles of 128x256
      // (two per CU) take the same time, a round of 512 tiles of 128x128 two thirds of it.  The 128-row tiles
      // waste less of a ragged segment, and two workgroups on a CU overlap one's epilogue with the other's
      // K loop; a single round of the two-per-CU shape costs 1.4 (both workgroups of a CU start together).
      const int64_t n0 = est_tiles(e, T, 2, 256, 256), n9 = est_tiles(e, T, 2, 128, 256), n3 = est_tiles(e, T, 2, 128, 128);
      const int64_t r0 = (n0 + 255) / 256, r9 = (n9 + 511) / 512, r3 = (n3 + 511) / 512;
      const double t0 = (double)r0, t9 = (double)r9 + (r9 == 1 ? 0.4 : 0.0), t3 = 0.66 * (double)r3;
      dflt = (t3 < t9 && t3 < t0) ? 3 : (t9 <= t0 ? 8 : 0);
    } else {
      // Deep K (dense FFN, un-restructured experts): 256x256 tiles with four waves when every CU gets one;
      // below that 256x128, whose round takes 0.56 of the time, unless it would need a second round; 128x128
      // (two workgroups per CU) for batches of a few hundred tokens.
      const int64_t tiles_256 = ((T * e.S_all() + 255) / 256) * ((e.d + 255) / 256), tiles_4 = 2 * tiles_256;
      const int big = e.max_width_pad >= 2048 ? 6 : 0;
      const double t_big = (double)((tiles_256 + 255) / 256), t_4 = 0.56 * (double)((tiles_4 + 255) / 256);
      dflt = (2 * tiles_256 < 256) ? 3 : (t_big <= t_4 ? big : 4);
      if (dflt == 3 && est_tiles(e, T, 2, 128, 128) > 512 && tiles_256 <= 256) dflt = 0;
      // Batches of hundreds of tokens split K (see bf16_splitk); there 128x256 tiles with two workgroups per
      // CU stream the weights faster than 128x128 ones over part of the range (measured: dense FFN at 512 to
      // 1024 tokens 69-114 us against 83-142 us; eight experts of 14336 neurons up to 256 tokens 145-166 us
      // against 195-202 us; slower outside these ranges).
      if (dflt == 3) {
        const int64_t n8 = est_tiles(e, T, 2, 128, 256);
        if (single ? (n8 > 48 && n8 <= 160) : n8 <= 128) dflt = 8;
      }
    }
  }
  const int forced = which == 1 ? tuning().gemm1_cfg : tuning().gemm2_cfg;
  if (forced >= 0 && forced < kNumCfgs && !(which == 1 && cfg_is_ws(forced))) return forced;
  if (which == 2 && tuning().ws_down != 0 && !(e.G == 1 && e.n_always == 1) && e.w_tiled && e.d % 256 == 0) {
    // The weight-stationary kernel for the groups it handles, when the batch gives it enough work items to
    // fill the chip several times over: the largest row chunk that still leaves four rounds of items (a chunk
    // pays once for loading its strip of weights into registers).  Groups of other widths keep a 128- or
    // 256-row tile of the general kernel over the same list.
    bool any = false, all = true;
    for (int g = 0; g < e.G; ++g) {
      if (ws_down_handles(e.width_pad_host[g])) any = true;
      else all = false;
    }
    if (any) {
      if (all && est_tiles(e, T, 2, 1024, 256) >= 1024) return 18;
      if (all && est_tiles(e, T, 2, 512, 256) >= 1024) return 17;
      if (est_tiles(e, T, 2, 256, 256) >= 1024) return 16;
      if (est_tiles(e, T, 2, 128, 256) >= 768 || tuning().ws_down == 2) return 15;
    }
  }
  return dflt;
}

// which = 1: BM of gate/up, 2: BM of down, 3: BN of gate/up (packed rows), 4: BN of down,
// 5 / 6: rows per height step when the gate/up / down contraction runs tiles of dynamic height, else 0
int bf16_gemm_tile(int which, const Engine& e, int64_t T) {
  switch (which) {
    case 1: return kCfgs[cfg_index(1, e, T)].bm;
    case 2: return kCfgs[cfg_index(2, e, T)].bm;
    case 3: return kCfgs[cfg_index(1, e, T)].bn;
    case 4: return kCfgs[cfg_index(2, e, T)].bn;
    case 5: return cfg_is_dyn(cfg_index(1, e, T)) ? 32 * kCfgs[cfg_index(1, e, T)].wgm : 0;
    default: return cfg_is_dyn(cfg_index(2, e, T)) ? 32 * kCfgs[cfg_index(2, e, T)].wgm : 0;
  }
}

// Estimated number of tiles of contraction `which` (1 gate/up, 2 down) with bm x bn tiles: exact for the
// always-on groups, and for the routed groups the full row tiles plus half a tile per touched group.
static int64_t est_tiles(const Engine& e, int64_t T, int which, int bm, int bn) {
  auto cols = [&](int g) { return which == 1 ? cdiv(2 * e.width_pad_host[g], bn) : cdiv(e.d, bn); };
  int64_t tiles = 0;
  for (int g = 0; g < e.n_always; ++g) tiles += ((T + bm - 1) / bm) * cols(g);
  if (e.G > e.n_always && e.S_dyn > 0) {
    const int64_t entries = T * e.S_dyn;
    const int64_t touched = std::min<int64_t>(e.G - e.n_always, entries);
    const int64_t rows = std::max<int64_t>((entries + bm - 1) / bm + touched / 2, touched);
    tiles += rows * cols(e.n_always);
  }
  return tiles;
}

// K split of contraction `which`: with too few tiles to give every CU one (batches of a few hundred
// tokens) several workgroups share a tile.  Powers of two up to 8, at least four K tiles per part, at
// most 64 MB of partial sums.
constexpr size_t SPLITK_MAX_BYTES = 64u << 20;
static int64_t splitk_rows(const Engine& e, int64_t T) { return T * e.S_all(); }
static int splitk_ldp(const Engine& e, int which) { return which == 1 ? 2 * e.max_width_pad : e.d; }

int bf16_splitk(const Engine& e, int64_t T, int which) {
  if (T < 1 || T > 1024 || tuning().splitk == 0) return 1;
  if (cfg_is_ws(cfg_index(which, e, T))) return 1;
  const TileCfg& c = kCfgs[cfg_index(which, e, T)];
  const int64_t tiles = est_tiles(e, T, which, c.bm, c.bn);
  int k_min = e.d;
  if (which == 2) {
    k_min = 1 << 30;
    for (int g = 0; g < e.G; ++g) k_min = std::min(k_min, e.width_pad_host[g]);
  }
  const int kt = cdiv(k_min, c.bk);
  const size_t per_part = (size_t)splitk_rows(e, T) * splitk_ldp(e, which) * sizeof(float);
  int ks = 1;
  // Split only while the launch stays well inside one round of workgroups (two tiles of 128 rows fit a CU, one of
  // the larger shapes): measured at 64..512 tokens, splitting a launch that already has a tile for most
  // CUs costs more (partial sums, a second launch) than the shorter K loop saves.
  const int64_t slots = c.bm == 128 ? 2 : 1;
  while (ks < 8 && tiles * ks * 2 <= 192 * slots && kt / (ks * 2) >= 4 && per_part * ks * 2 <= SPLITK_MAX_BYTES) ks *= 2;
  return ks;
}

// Bytes to reserve for the partial sums in a workspace for up to T tokens: the cap, because a smaller
// batch may split further than the largest one does.
size_t bf16_splitk_bytes(const Engine& e, int64_t T) {
  (void)e;
  (void)T;
  return SPLITK_MAX_BYTES;
}

// The split a launch may use: the chosen one, unless the slabs would not fit what the workspace reserved.
static int splitk_that_fits(const Engine& e, int64_t T, int which, const WsLayout& L) {
  const int ks = bf16_splitk(e, T, which);
  const size_t per_part = (size_t)splitk_rows(e, T) * splitk_ldp(e, which) * sizeof(float);
  return (ks > 1 && per_part * ks <= L.splitk_bytes) ? ks : 1;
}

// Finish of a K-split gate/up contraction: one workgroup per slot row adds the parts in order and applies
// Swish(g) * u (Eq. 3, first line) with the same arithmetic as the fused epilogue.
__global__ __launch_bounds__(256) void splitk_finish_gate_up(const float* __restrict__ P, int k_split, int64_t p_rows,
                                                             int ldp, const GroupDev* __restrict__ groups,
                                                             const int32_t* __restrict__ seg_off,
                                                             const int64_t* __restrict__ h_off, int G, int single,
                                                             bf16_t* __restrict__ H) {
  const int64_t row = blockIdx.x;
  int g = 0, seg0 = 0;
  int64_t hoff = 0;
  if (!single) {
    g = find_group(seg_off, G, (int)row);       // the group whose slot segment holds this row
    seg0 = seg_off[g];
    hoff = h_off[g];
  }
  const int wp = groups[g].width_pad;
  for (int n = threadIdx.x; n < wp; n += 256) {
    const int gc = (n / IL) * 2 * IL + (n % IL);
    float gt = 0.0f, up = 0.0f;
    for (int k = 0; k < k_split; ++k) {
      const float* prow = P + ((int64_t)k * p_rows + row) * ldp;
      gt += prow[gc];
      up += prow[gc + IL];
    }
    const float sg = gt * __frcp_rn(1.0f + __expf(-gt));
    H[hoff + (row - seg0) * wp + n] = f32_to_bf16(sg * up);
  }
}

// Finish of a K-split down contraction: C[row][c] = sum of the parts, four columns per thread.
__global__ __launch_bounds__(256) void splitk_finish_down(const float* __restrict__ P, int k_split, int64_t p_rows,
                                                          int d, bf16_t* __restrict__ C) {
  const int64_t row = blockIdx.x;
  for (int c = threadIdx.x * 4; c < d; c += 1024) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k = 0; k < k_split; ++k) {
      const float4 v = *reinterpret_cast<const float4*>(P + ((int64_t)k * p_rows + row) * d + c);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    bf16_t out[4] = {f32_to_bf16(acc.x), f32_to_bf16(acc.y), f32_to_bf16(acc.z), f32_to_bf16(acc.w)};
    *reinterpret_cast<uint2*>(C + row * d + c) = *reinterpret_cast<const uint2*>(out);
  }
}

template <typename K>
static hipError_t launch_kernel(K kern, size_t smem, int threads, bool& attr_done, const GemmArgs& a, hipStream_t s) {
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)a.n_blocks * (unsigned)(a.k_split > 1 ? a.k_split : 1)), dim3(threads), smem, s, a);
  return hipGetLastError();
}

template <int BM, int BN, int BKT, int STAGES, int WGM, int WGN, int MODE, bool DYN = false>
static hipError_t launch_dma(const GemmArgs& a, hipStream_t s) {
  static bool attr_done = false;
  constexpr size_t smem = (STAGES == 0 ? 5 * (size_t)(BM > BN ? BM : BN) : STAGES * (size_t)(BM + BN)) * BKT * sizeof(bf16_t);
  return launch_kernel(grouped_gemm_bf16_dma<BM, BN, BKT, STAGES, WGM, WGN, MODE, DYN>, smem, WGM * WGN * 64, attr_done, a, s);
}

template <int MODE>
static hipError_t launch_cfg(int ci, const GemmArgs& a, hipStream_t s) {
  switch (ci) {
    case 0: return launch_dma<256, 256, 64, 0, 2, 4, MODE>(a, s);
    case 1: return launch_dma<128, 128, 64, 2, 2, 2, MODE>(a, s);
    case 2: return launch_dma<256, 256, 64, 2, 2, 4, MODE>(a, s);
    case 3: return launch_dma<128, 128, 64, 0, 2, 2, MODE>(a, s);
    case 4: return launch_dma<256, 128, 64, 3, 4, 2, MODE>(a, s);
    case 6: return launch_dma<256, 256, 64, 0, 2, 2, MODE>(a, s);
    case 7: return launch_dma<64, 128, 64, 4, 2, 2, MODE>(a, s);
    case 8: return launch_dma<128, 256, 32, 3, 2, 2, MODE>(a, s);
    case 9: return launch_dma<224, 256, 64, 0, 1, 4, MODE>(a, s);
    case 10: return launch_dma<192, 256, 64, 0, 1, 4, MODE>(a, s);
    case 11: return launch_dma<256, 256, 64, 0, 1, 4, MODE, true>(a, s);
    case 12: return launch_dma<128, 256, 32, 3, 1, 4, MODE, true>(a, s);
    case 13: return launch_dma<256, 256, 64, 0, 2, 2, MODE, true>(a, s);
    case 14: return launch_dma<128, 256, 32, 3, 2, 2, MODE, true>(a, s);
    default: return launch_dma<256, 256, 32, 4, 2, 4, MODE>(a, s);
  }
}

hipError_t launch_experts_bf16(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y,
                               hipStream_t s, int stage) {
  const int remap = tuning().xcd_remap;
  GemmArgs a;
  a.groups = e.groups;
  a.seg_off = reinterpret_cast<const int32_t*>(ws + L.seg_off);
  a.h_off = reinterpret_cast<const int64_t*>(ws + L.h_off);
  a.G = e.G;
  a.d = e.d;
  a.ldb = e.ldw1;
  a.b_tiled = e.w_tiled;
  a.T = T;
  a.single = (e.G == 1 && e.n_always == 1) ? 1 : 0;
  a.xcd_remap = remap;
  a.zero_pad = tuning().zero_pad;
  a.ws_skip = 0;
  // gate/up
  a.A = static_cast<const bf16_t*>(x);
  a.B = static_cast<const bf16_t*>(e.w1);
  a.C = reinterpret_cast<bf16_t*>(ws + L.h);
  a.work = reinterpret_cast<const int32_t*>(ws + L.work1);
  a.slot2tok = a.single ? nullptr : reinterpret_cast<const int32_t*>(ws + L.slot2tok);
  {
    // An XCD's share of a work list has equal estimated cost, not equal length (see place_tile): with tiles of
    // dynamic height the cheapest tile counts 3 blocks of 32 rows and a full one bm / 32, so the longest share
    // can hold that many times an eighth of the list.
    const int ci = cfg_index(1, e, T);
    const int64_t bound = gemm_work_bound(e, T, 1);
    int64_t share = (bound + 7) / 8;
    if (remap && !a.single) share = std::min<int64_t>(bound, share + 1);   // (a boundary inside a group is rounded)
    if (cfg_is_dyn(ci) && remap && !a.single) {
      const int full = kCfgs[ci].bm / 32, low = std::min(full, 3);
      share = std::min<int64_t>(bound, (bound * full + 8 * low - 1) / (8 * low) + 2);
    }
    a.n_blocks = (int)(8 * share);
  }
  a.P = reinterpret_cast<float*>(ws + L.splitk);
  a.p_rows = splitk_rows(e, T);
  a.k_split = splitk_that_fits(e, T, 1, L);
  a.ldp = splitk_ldp(e, 1);
  if (stage != 2) {
    hipError_t err = launch_cfg<1>(cfg_index(1, e, T), a, s);
    if (err == hipSuccess && a.k_split > 1) {
      hipLaunchKernelGGL(splitk_finish_gate_up, dim3((unsigned)a.p_rows), dim3(256), 0, s, a.P, a.k_split, a.p_rows, a.ldp,
                         a.groups, a.seg_off, a.h_off, a.G, a.single, a.C);
      err = hipGetLastError();
    }
    if (err != hipSuccess || stage == 1) return err;
  }
  // down
  a.A = reinterpret_cast<const bf16_t*>(ws + L.h);
  a.B = static_cast<const bf16_t*>(e.w2);
  a.C = e.direct_output() ? static_cast<bf16_t*>(y) : reinterpret_cast<bf16_t*>(ws + L.y_slots);
  a.work = reinterpret_cast<const int32_t*>(ws + L.work2);
  a.slot2tok = nullptr;
  {
    // An XCD's share of the down list has equal cost, not equal length: with groups of unequal width the
    // share made of the cheapest tiles is longer than an eighth of the list.
    const int64_t bound = gemm_work_bound(e, T, 2);
    int c_min = 1 << 30, c_max = 1;
    const int ci2 = cfg_index(2, e, T);
    const int full2 = kCfgs[ci2].bm / 32, low2 = cfg_is_dyn(ci2) ? std::min(full2, 3) : full2;
    for (int g = 0; g < e.G; ++g) {
      const int c = cdiv(e.width_pad_host[g], 64) + 4;
      c_min = std::min(c_min, c * low2);
      c_max = std::max(c_max, c * full2);
    }
    const int64_t share = std::min<int64_t>(bound, (bound * c_max + 8 * c_min - 1) / (8 * c_min) + 2);
    a.n_blocks = (int)(remap && !a.single ? 8 * share : round_up64(bound, 8));
  }
  a.k_split = splitk_that_fits(e, T, 2, L);
  a.ldp = splitk_ldp(e, 2);
  {
    const int ci2 = cfg_index(2, e, T);
    if (cfg_is_ws(ci2)) {
      bool wide = false;
      for (int g = 0; g < e.G; ++g) wide = wide || !ws_down_handles(e.width_pad_host[g]);
      hipError_t err = hipSuccess;
      if (wide) {
        a.ws_skip = 1;
        a.k_split = 1;
        err = launch_cfg<2>(kCfgs[ci2].bm == 128 ? 8 : 6, a, s);
      }
      if (err == hipSuccess) err = launch_ws_down(e, ws, L, a.C, kCfgs[ci2].bm, a.n_blocks, a.xcd_remap, s);
      return err;
    }
  }
  hipError_t err = launch_cfg<2>(cfg_index(2, e, T), a, s);
  if (err == hipSuccess && a.k_split > 1) {
    hipLaunchKernelGGL(splitk_finish_down, dim3((unsigned)a.p_rows), dim3(256), 0, s, a.P, a.k_split, a.p_rows, e.d, a.C);
    err = hipGetLastError();
  }
  return err;
}

}  // namespace cmoe
