// Internal declarations shared by the host side (packing, C ABI) and the HIP kernels of libcmoe.
// Not part of the public interface.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace cmoe {

// ---- packing constants ---------------------------------------------------------------------
// Gate and up rows of one expert are interleaved in blocks of IL neurons (IL gate rows, then the
// IL up rows of the same neurons) so that a 32x32 MFMA tile of gate pre-activations and the tile
// of up pre-activations of the same (token, neuron) pairs land in the same lanes.
constexpr int IL = 32;
// Expert widths are padded with zero neurons to a multiple of WPAD (zero gate/up rows give h = 0,
// zero down columns multiply it: the padded neurons contribute exactly nothing).
constexpr int WPAD = 32;
constexpr int MAX_TOPK = 16;       // N_k of a flat layer or of the sub-experts
constexpr int MAX_OUTER_TOPK = 8;  // outer_top_k of the hierarchy
constexpr int MAX_DYN = 24;        // routed slots per token (hierarchy: outer_top_k * (1 + N_k))
constexpr int MAX_SCORED = 64;     // routed experts scored by one router (one lane per expert)
constexpr int MAX_GROUPS = 128;    // expert groups of one engine
constexpr int TOK_TILE = 64;       // tokens per router / permute tile

__host__ __device__ static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
static inline int64_t round_up64(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
__host__ __device__ static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// ---- weight layout of the bf16 kernels ------------------------------------------------------------
// W1 and W2 are stored in tiles of 16 rows x 32 K elements (1 KB of consecutive memory), the tiles of a
// 16-row block one after the other along K.  A tile is exactly one A operand of v_mfma_f32_16x16x32_bf16, so
// a load instruction of the weight-streaming decode kernels covers 1 KB of consecutive bytes and a wave's
// K slice is one contiguous run; with row-major rows the same instruction would touch half of 16 different
// 128-byte lines (measured on a load-only skeleton: 3.6 against 5.2 TB/s).  The prefill kernels' 1 KB DMA
// transfers (8 rows x 64 K) are two 512-byte pieces of neighbouring tiles.  K is padded to a multiple of 32
// with zeros, rows to a multiple of 16.  fp32 layers keep row-major weights.
constexpr int TILE_ROWS = 16;
constexpr int TILE_K = 32;
constexpr int TILE_ELEMS = TILE_ROWS * TILE_K;
__host__ __device__ static inline int tiles_along_k(int K) { return (K + TILE_K - 1) / TILE_K; }
// Element offset of (row, k) in a tiled matrix whose rows are kt32 tiles long.
__host__ __device__ static inline int64_t tiled_offset(int64_t row, int k, int kt32) {
  return ((row / TILE_ROWS) * kt32 + k / TILE_K) * TILE_ELEMS + (row % TILE_ROWS) * TILE_K + (k % TILE_K);
}

// One expert group as the device kernels see it.
struct GroupDev {
  int32_t width_pad;    // neurons incl. zero padding (multiple of WPAD)
  int32_t w1_row0;      // first packed (interleaved gate/up) row of the group in W1
  int64_t w2_off;       // element offset of the group's down matrix [d][width_pad] in W2 (tiled: d padded to 16 rows)
};

// What the router kernel scores and selects.  Rows of the router matrix Wr [n_sw_rows + n_lin_rows][d]:
//   SwiGLU blocks of 2*IL rows (IL gate rows, IL up rows) scoring IL routed experts each (Eq. 8),
//   then n_lin_rows rows of plain linear logits (outer router of the hierarchical case).
struct RouterDev {
  int32_t n_scored;        // routed experts scored (flat: N_r; hierarchy: n_outer * N_r)
  int32_t n_sw_rows;       // 2 * IL * ceil(n_scored / IL)
  int32_t n_lin;           // linear logits in use (n_outer); 0 for a flat layer
  int32_t n_lin_rows;      // padded row count (0 or IL)
  int32_t top_k;           // N_k (0: the dense form of a hierarchy, outer routing only)
  int32_t outer_top_k;     // 0 for a flat layer
  int32_t n_r_sub;         // routed experts per outer expert (flat: N_r)
  int32_t n_always;        // always-on groups in front
  int32_t score_abs;       // rank by |s|
  int32_t use_gate;        // evaluate softmax / u / b (Eq. 9); 0 = binary gate of Eq. 4
  int32_t groups_per_outer;   // hierarchy: sub_has_shared + N_r
  int32_t sub_has_shared;     // hierarchy: each outer expert starts with a shared group
};

// Workspace carve-up for a batch of T tokens (byte offsets, 256-aligned).
struct WsLayout {
  size_t sel_group, sel_weight;      // [T][S_dyn] int32 / float   (router -> permute)
  size_t tile_counts;                // [n_tok_tiles][G] int32
  size_t seg_off, counts;            // [G+1] / [G] int32
  size_t work1, work2;               // [G+1] int32: prefix of work items of the two grouped GEMMs, then [9]: first
                                     // item of each XCD's contiguous share
  size_t h_off;                      // [G+1] int64: element offset of each group's rows in H
  size_t slot2tok;                   // [n_slots] int32
  size_t tok2slot, slot_w;           // [T][S_all] int32 / float
  size_t w_by_slot;                  // [n_slots] float: the combine weight of each slot (decode batches)
  size_t scores;                     // [8][T][router rows] float: K-slice partial pre-activations of the router
  size_t h;                          // hidden activations, ragged: rows of group g are width_pad(g) wide
  size_t y_slots;                    // [n_slots][d]; unused by a direct-output engine (written straight to y)
  size_t splitk;                     // fp32 partial sums of a K-split contraction (small batches only)
  size_t splitk_bytes;               // bytes reserved there (0: no contraction of this layout may split K)
  size_t total;
  int64_t n_slots;
  int n_tok_tiles;
  int skip_always;                   // 1: the gate/up work list leaves out the always-on group (the routing front end
                                     // runs its units itself, next to selection and placement)
  int gate_up_done;                  // 1: the routing front end ran every gate/up unit (up to 16 tokens): no gate/up launch
};

// A grouped SwiGLU problem on the device: router (optional) -> permute -> experts -> combine.
struct Engine {
  int dtype = 1;
  int d = 0;
  int G = 0;                 // groups
  int n_always = 0;          // leading groups every token visits (identity segments)
  int S_dyn = 0;             // routed slots per token
  int64_t h_per_token = 0;   // upper bound of hidden elements per token (sum of its groups' width_pad)
  int max_width_pad = 0;
  int ldw1 = 0;              // elements per row of W1 (row-major: the row stride; tiled: 32 * tiles along K)
  int w_tiled = 0;           // 1: W1 and W2 are tiled 16 x 32 (bf16 layers)
  int width_pad_host[MAX_GROUPS] = {0};   // host copy of the groups' padded widths
  RouterDev r{};
  // device pointers (inside the caller's weight buffer)
  const void* w1 = nullptr;        // [rows][d] interleaved gate/up rows of all groups
  const void* w2 = nullptr;        // per group [d][width_pad]
  const void* wr = nullptr;        // router rows
  const void* wr_tiled = nullptr;  // flat bf16 layers: the same rows in MFMA operand order [row block][K step][lane][8]
  const GroupDev* groups = nullptr;
  const float* gate_u = nullptr;   // [n_scored] or null
  const float* gate_b = nullptr;   // [n_scored] or null
  const float* lin_off = nullptr;  // [n_lin] or null
  // Neuron-level activation sparsity inside the routed groups (flat bf16 layers): a hidden activation h_n of a
  // routed group survives iff |h_n| * nscale[n] >= sparse_tau, nscale = 1 (mode 1) or the L2 norm of the
  // neuron's row of W_down (mode 2).  w2n: the routed groups' down matrices once more, neuron-major
  // [sum of routed width_pad][d], so that a dropped neuron's weights are never read.
  int sparse_mode = 0;             // 0: off
  float sparse_tau = 0.0f;
  const void* w2n = nullptr;
  const float* nscale = nullptr;   // [sum of all width_pad], indexed by w1_row0 / 2 + neuron
  int S_all() const { return n_always + S_dyn; }
  // One always-on group and nothing routed (the dense baseline): slot t is token t with weight 1, so the
  // down contraction writes y itself.  A routed layer with one slot per token (top-1, no shared expert) does
  // not qualify: its slots are permuted and carry a gate weight.
  bool direct_output() const { return S_dyn == 0 && n_always == 1; }
};

// Tuning switches: every field defaults to the measured best; the environment variables of the same
// names (CMOE_GEMM1_CFG, ...) are read once, when the library is first used, and cmoe_set_tuning changes a
// field afterwards (so that an A/B comparison can run inside one process).  The forward path reads plain ints.
struct Tuning {
  int gemm1_cfg = -1;      // tile shape of the gate/up contraction (index into the table of gemm_bf16.hip); -1: per batch
  int gemm2_cfg = -1;      // same for the down contraction
  int xcd_remap = 1;       // 0: workgroups take work items in launch order instead of per-XCD shares
  int splitk = 1;          // 0: never split K
  int zero_pad = 1;        // 0: tile rows past the end of a group repeat its last row instead of reading zeros
  int decode_fuse = 1;     // 0: separate down and combine kernels for batches of at most 32 tokens
  int front_shared = 1;    // 0: the shared expert's gate/up units stay in the gate/up launch at decode
  int front_all = 1;       // one token on a flat layer.  0: the routed gate/up units keep a launch of their own;
                           // 1: the selection launch runs them; 2: that launch also scores, every workgroup
                           // for itself, and there is no scoring launch (measured slower: 31.8 against 28.3 us
                           // per forward with 16 experts of 688, 34.0 against 30.7 with 32 of 448; the 300-odd
                           // workgroups each pull the router matrix through L2 at the same time)
  int front_tile = 0;      // 0: batches of 2-16 tokens keep a gate/up launch for the routed experts; 1: every
                           // routed unit runs in the selection launch, each workgroup selecting the batch itself
                           // (measured slower: the team selection of up to 16 tokens in 700 workgroups at once
                           // costs more than the launch it saves: 51.4 against 37.8 us at 2 tokens, 71.8 against
                           // 62.4 us at 16, 16 experts of 688)
  int force_simt = 0;      // 1: bf16 layers run the plain FMA kernels
  int ldpad = 0;           // extra elements in the row stride of a row-major (fp32) packed gate/up matrix
  int host_threads = 0;    // worker threads of the host-side construction (0: hardware threads, at most 16)
  int skip_rows = 1;       // 0: the gate/up contraction multiplies the 32-row blocks past the end of a segment too
  int decode_split = -1;   // K split of the decode gate/up units across workgroups (-1: chosen per batch)
  int ws_down = 0;         // 1: the weight-stationary down contraction where the batch gives it enough work items,
                           // 2: wherever it has an instantiation for the widths; 0 (default): never (measured slower)
  int skip_stage = 0;      // measurement aid: 3, 4 or 5 leaves out the gate/up, down or combine launch of every
                           // forward (outputs are then meaningless); the time a forward loses is that stage's
                           // cost inside the stream, launch gap included.  6: a batch that takes the decode front
                           // end runs its scoring launch and nothing else (such a loop is bound by the host's
                           // launch rate, not by the kernel).  Other values: nothing is skipped.
  int repeat_stage = 0;    // measurement aid: 3, 4 or 5 launches that stage twice (same inputs, same outputs); the
                           // time a forward gains is one more launch of it under the forward's own clocks.  At
                           // one token on a flat layer the gate/up stage is the selection launch, which 3 then
                           // issues twice (the second finds the weights in the cache: a lower bound).  6: the
                           // decode front end's scoring launch twice (small operands, cached either way), so
                           // that (loop without the down launch) - (this gain) is the selection launch's cost.
};
Tuning& tuning();

size_t elem_size(int dtype);
// Row stride of a row-major (fp32) packed gate/up matrix for model width d: d plus the optional pad of the
// CMOE_LDPAD tuning variable (rows a power of two apart all map to the same L2 channel).
int w1_row_stride(int d);

// Record the calling thread's error message (what cmoe_last_error returns) and hand `code` back.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
// splitk_cap: upper limit of the bytes reserved for the partial sums of a K-split contraction (a launch whose
// slabs would not fit what was reserved does not split).
WsLayout ws_layout(const Engine& e, int64_t T, size_t splitk_cap = ~(size_t)0);

// Kernel launchers (defined in the .hip files).  All enqueue on `s` and return the launch status.
hipError_t launch_router(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L,
                         int32_t* topk_out, int32_t* outer_out, float* scores_out, hipStream_t s);
hipError_t launch_permute(const Engine& e, int64_t T, char* ws, const WsLayout& L, int32_t* counts_out,
                          hipStream_t s);
// stage: 0 = gate/up GEMM then down GEMM, 1 = gate/up only, 2 = down only
hipError_t launch_experts(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y,
                          hipStream_t s, int stage = 0);
hipError_t launch_combine(const Engine& e, int64_t T, char* ws, const WsLayout& L, void* y, hipStream_t s);

// Tile sizes of the two grouped GEMMs (the permute kernel builds their work lists from them):
// which = 1: rows of a gate/up tile, 2: rows of a down tile, 3: packed gate/up rows (columns of the
// product) of a gate/up tile, 4: columns of a down tile, 5 / 6: rows per height step when the gate/up / down
// contraction runs tiles of dynamic height, else 0.
int gemm_tile(const Engine& e, int64_t T, int which);
bool use_simt_experts(int dtype);
int bf16_gemm_tile(int which, const Engine& e, int64_t T);
// K split of the bf16 contractions at small batches (1 = none) and the bytes of fp32 partial sums it needs.
int bf16_splitk(const Engine& e, int64_t T, int which);
size_t bf16_splitk_bytes(const Engine& e, int64_t T);
int simt_gemm_tile(int which);
hipError_t launch_experts_bf16(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y,
                               hipStream_t s, int stage);
hipError_t launch_experts_simt(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y,
                               hipStream_t s, int stage);
bool decode_front_ok(const Engine& e, int64_t T);
hipError_t launch_decode_front(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L,
                               int32_t* topk_out, int32_t* outer_out, float* scores_out, int32_t* counts_out,
                               hipStream_t s);
// Decode batches (bf16, T <= 16; the fused down + combine kernel up to 32): weight-streaming expert kernels,
// see decode.hip.
bool decode_path_ok(const Engine& e, int64_t T);
bool decode_front_runs_shared(const Engine& e, int64_t T);   // the front end's second launch also runs group 0's gate/up
bool decode_front_runs_all(const Engine& e, int64_t T);      // ... and every routed unit too (up to 16 tokens, flat layer)
bool decode_fuses_combine(const Engine& e, int64_t T);   // the down kernel also does the weighted sum over slots
hipError_t launch_decode_down_combine(const Engine& e, int64_t T, char* ws, const WsLayout& L, void* y, hipStream_t s);
// Neuron-level sparsity (Engine::sparse_mode): the down + combine kernel of one or two tokens that reads only the
// surviving neurons' rows, and for every other batch the kernel that zeroes the dropped activations in H.
bool decode_sparse_down_ok(const Engine& e, int64_t T);
hipError_t launch_decode_down_sparse(const Engine& e, int64_t T, char* ws, const WsLayout& L, void* y, hipStream_t s);
hipError_t launch_mask_hidden(const Engine& e, int64_t T, char* ws, const WsLayout& L, hipStream_t s);
hipError_t launch_experts_decode(const Engine& e, const void* x, int64_t T, char* ws, const WsLayout& L, void* y,
                                 hipStream_t s, int stage);
// Upper bound of work items of grouped GEMM `which` (1: gate/up, 2: down) for T tokens.
int64_t gemm_work_bound(const Engine& e, int64_t T, int which);

}  // namespace cmoe
