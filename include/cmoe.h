/*
 * cmoe.h - C ABI of libcmoe: a dense SwiGLU FFN restructured analytically into shared +
 * routed experts, and its forward pass on one MI355X (gfx950).
 *
 * Vocabulary follows the paper (arXiv 2502.04416):
 *   d      model width                      d_h   FFN hidden width (d_ff here)
 *   N      experts, m = d_h / N neurons each (Sec. 4.1)
 *   N_s    shared (always-active) experts   N_r = N - N_s routed experts
 *   N_k    routed experts selected per token (Eq. 4)
 *   K_a    how many top-|h| neurons count as "active" per calibration token (App. A.2)
 *   R_j    representative neuron of routed expert j (Eq. 7); the router is the pair of
 *          columns R_j of W_gate / W_up (Eq. 8)
 *   u, b   learnable gate scale and load-balance bias of Eq. 9 (both default to 0)
 *
 * Conventions
 *   - Every function returns 0 on success or a negative CMOE_E* code; cmoe_last_error()
 *     returns a thread-local message for the last failure.  Nothing aborts or throws
 *     across this boundary.  On failure output handles are left untouched.
 *   - "host" pointers are ordinary CPU memory, read during the call and not retained.
 *     "device" pointers are HIP device memory owned by the caller; they must stay valid
 *     until the work enqueued on the stream has finished.  The library owns only the
 *     opaque handle and its host-side metadata; the forward calls never allocate.
 *   - Matrices are row-major in the paper's orientation: W_gate, W_up are [d, d_h]
 *     (column i belongs to neuron i), W_down is [d_h, d] (row i belongs to neuron i),
 *     token batches are [T, d].
 *   - dtype CMOE_BF16: host weights arrive as fp32 and are rounded once to bf16
 *     (round-to-nearest-even); x and y on the device are bf16; products accumulate in fp32;
 *     router scores are fp32.  dtype CMOE_F32: everything is fp32.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  Forward
 *     calls only enqueue work; they do not synchronise.
 *   - Same inputs give bit-identical outputs from run to run (no floating-point atomics).
 */
#ifndef CMOE_H
#define CMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CMOE_OK       0
#define CMOE_EINVAL  -1   /* bad argument: null pointer, shape, workspace too small ...   */
#define CMOE_ENOMEM  -2   /* host allocation failed                                       */
#define CMOE_EHIP    -3   /* a HIP runtime call failed (message holds hipGetErrorString)  */
#define CMOE_ESTATE  -4   /* call out of order (e.g. forward before upload)               */

#define CMOE_F32   0
#define CMOE_BF16  1

typedef struct cmoe_layer cmoe_layer;   /* one restructured FFN (opaque)                       */
typedef struct cmoe_hier  cmoe_hier;    /* an MoE layer whose experts were each restructured   */

typedef struct {
  int32_t d_model;       /* d                                                               */
  int32_t d_ff;          /* d_h; must be a multiple of n_experts (m = d_h / N, Sec. 4.1)    */
  int32_t n_experts;     /* N                                                               */
  int32_t n_shared;      /* N_s, 0 <= N_s < N                                               */
  int32_t top_k;         /* N_k, 1 <= N_k <= min(N_r, 16); N_r <= 64                        */
  int32_t k_act;         /* K_a (the paper uses 10); only used by cmoe_build                */
  int32_t kmeans_iters;  /* assignment + centroid-update rounds, >= 1; only cmoe_build      */
  int32_t dtype;         /* CMOE_F32 or CMOE_BF16                                           */
  int32_t dist_mode;     /* 0: L2 distance with the square root (App. A.3 as printed),
                            1: squared L2 (= Hamming for binary vectors); only cmoe_build   */
  int32_t score_mode;    /* 0: rank experts by the signed score s of Eq. 8, 1: by |s|       */
} cmoe_config;

/* ---- construction (host side; Sec. 4.1-4.2, App. A.2-A.4) ------------------------------- */

/* build_moe: profile the calibration tokens (H, ATopK matrix A, rates mu), take the N_s*m
 * neurons of highest rate as the shared expert, cluster the rest into N_r balanced groups
 * (exact balanced assignment against the current centroids, then the mean update), pick the
 * representative neuron of each group (Eq. 7) and slice the experts and the router out of
 * the dense matrices.  All pointers are host fp32; calib_x is [q, d].  Ties go to the lowest
 * index everywhere.  *out receives a new handle (free with cmoe_destroy). */
int cmoe_build(const cmoe_config* cfg, const float* w_gate, const float* w_up, const float* w_down,
               const float* calib_x, int64_t q, cmoe_layer** out);

/* cmoe_build with App. A.2 steps 1-2 (hidden states of the calibration tokens and their per-token
 * top-K_a) computed on the current HIP device instead of the host: bf16 MFMA with fp32 accumulation,
 * same tie rule (lowest index).  Everything else, and every argument, as cmoe_build.  Needs a bf16 layer
 * with d_model a multiple of 64; allocates and frees its own device memory (about
 * 4*d_model*d_ff + 4*q*d_ff bytes) and synchronises.  A token whose K_a-th and (K_a+1)-th largest |h|
 * differ by less than fp32 accumulation error may get a different index set than on the host. */
int cmoe_build_gpu(const cmoe_config* cfg, const float* w_gate, const float* w_up, const float* w_down,
                   const float* calib_x, int64_t q, cmoe_layer** out);

/* App. A.2 steps 1-2 on their own: active_out [q, k_act] (host int32) receives, for every calibration
 * token, the k_act neurons of largest |h| in descending order of magnitude (ties to the lowest index);
 * on_gpu = 0 computes on the host (fp64 accumulation), 1 on the current HIP device as in cmoe_build_gpu.
 * Uses d_model, d_ff, k_act and dtype of the configuration. */
int cmoe_profile_activations(const cmoe_config* cfg, const float* w_gate, const float* w_up, const float* calib_x,
                             int64_t q, int on_gpu, int32_t* active_out);

/* The balanced assignment step of App. A.3 on its own: given dist [n, n_r] (host, row-major,
 * n = n_r * m) find label[i] in [0, n_r) minimising sum_i dist[i, label[i]] with exactly m rows per
 * cluster.  Exact (successive shortest paths on the transportation problem; same optimum as the
 * replicated-column assignment the paper describes).  label_out [n] int32, cost_out may be NULL. */
int cmoe_balanced_assignment(const double* dist, int32_t n, int32_t n_r, int32_t m, int32_t* label_out,
                             double* cost_out);

/* Same slicing and packing, but from a given partition instead of profiling:
 * neuron_order [d_h] lists dense neuron ids, the N_s*m shared ones first, then routed expert
 * 0, 1, ... with m ids each; rep_neuron [N_r] holds the dense neuron id R_j of each routed
 * expert (Eq. 7/8).  neuron_order must be a permutation of 0..d_h-1. */
int cmoe_build_from_partition(const cmoe_config* cfg, const float* w_gate, const float* w_up,
                              const float* w_down, const int32_t* neuron_order,
                              const int32_t* rep_neuron, cmoe_layer** out);

/* Copy the partition out: neuron_order [d_h], rep_neuron [N_r], mu [d_h] (activation rates;
 * zeros when the layer came from cmoe_build_from_partition).  Any pointer may be NULL.
 * cost (may be NULL) receives the objective of the last balanced assignment (App. A.3). */
int cmoe_export_partition(const cmoe_layer* layer, int32_t* neuron_order, int32_t* rep_neuron,
                          float* mu, double* cost);

/* Gate parameters of Eq. 9: u [N_r] (NULL = zeros), b [N_r] (NULL = zeros), host fp32.
 * With both zero the gate is the binary gate of Eq. 4 and no softmax is evaluated.
 * May be called before or after cmoe_upload; takes effect at the next forward.  On an uploaded layer
 * the call waits for the whole device (hipDeviceSynchronize) before it overwrites the device copy, so a
 * forward still in flight on any stream keeps the old values; it must not overlap a forward being
 * enqueued from another host thread. */
int cmoe_set_gate_params(cmoe_layer* layer, const float* u, const float* b);

/* Neuron-level activation sparsity inside the routed experts (Sec. 5 "Orthogonality with Activation
 * Sparsity": training-free activation sparsity applied within the routed experts; the shared experts are
 * never sparsified).  A hidden activation h_n of a selected routed expert contributes h_n w_n to the output
 * (Eq. 1) only if
 *     mode 1 (magnitude):        |h_n| >= tau
 *     mode 2 (weight-informed):  |h_n| * ||w_n||_2 >= tau,   w_n = row n of W_down (rounded to the layer dtype),
 * decided on the bf16 value of h_n the kernels hold (norm and product in fp32); mode 0 switches it off.  The
 * paper names the family of criteria and gives no formula; the threshold is the caller's (such methods
 * calibrate it offline for a target share of dropped neurons).  bf16 flat layers only (CMOE_EINVAL otherwise;
 * CMOE_ESTATE for a layer inside a hierarchy).  The first call with mode != 0 must come before cmoe_upload: it
 * adds a neuron-major copy of the routed experts' down matrices and the row norms to cmoe_packed_bytes (for
 * batches of one or two tokens the down projection reads only the surviving neurons' rows from it; larger
 * batches zero the dropped activations and run the usual kernels).  Later calls may change mode and tau at
 * any time; they take effect at the next forward. */
int cmoe_set_neuron_sparsity(cmoe_layer* layer, int mode, float tau);

/* Copies the current gate parameters to host arrays u [N_r], b [N_r] (either may be NULL). */
int cmoe_get_gate_params(const cmoe_layer* layer, float* u, float* b);

/* One load-balancing step of Sec. 4.3 (text after Eq. 9) from the per-expert token counts a forward
 * returned (host int32 [N_r], e.g. a copy of cmoe_forward's counts_dev): with p_i = counts_i / sum(counts)
 * and the uniform target p* = 1/N_r, b_i decreases by gamma where p_i > p*, increases by gamma where
 * p_i < p*, and is unchanged where they are equal or when no token was routed.  The paper uses
 * gamma = 1e-3.  u is kept.  Same rules as cmoe_set_gate_params (takes effect at the next forward;
 * not for layers inside a hierarchy).  CMOE_EINVAL on a negative count or a negative gamma. */
int cmoe_update_bias(cmoe_layer* layer, const int32_t* counts, float gamma);

/* The dense baseline F(x) of Eq. 3 needs a second, single-group copy of the layer's weights.  It is
 * kept by default (the speedup of the restructured layer is measured against it); enabled = 0 before
 * cmoe_upload / cmoe_hier_create releases the host copy and leaves it out of cmoe_packed_bytes and of the
 * upload: cmoe_dense_forward then returns CMOE_ESTATE.  It cannot be enabled again (CMOE_ESTATE). */
int cmoe_set_baseline(cmoe_layer* layer, int enabled);

/* Bytes of device memory cmoe_upload needs for the packed weights (expert-sliced copy for the
 * MoE forward, the router columns and, unless cmoe_set_baseline switched it off, an unpadded copy
 * for the dense baseline). */
size_t cmoe_packed_bytes(const cmoe_layer* layer);

/* Bytes of device workspace a forward call with up to max_tokens tokens needs. */
size_t cmoe_workspace_bytes(const cmoe_layer* layer, int64_t max_tokens);

/* Pack the weights (per-expert slices, gate/up rows interleaved, expert widths padded with
 * zero neurons to the MFMA tile) and copy them into dev_weights (>= cmoe_packed_bytes, 256-byte
 * aligned).  Synchronises the stream before returning (the host staging buffer is freed). */
int cmoe_upload(cmoe_layer* layer, void* dev_weights, void* hip_stream);

/* moe_ffn_forward (Eq. 4 with the router of Eq. 8 and the gate of Eq. 9):
 *   y[t] = E^s(x[t]) + sum over the N_k selected routed experts of g * E^r_j(x[t]).
 * x_dev, y_dev: device [T, d] in the layer's dtype.  Optional device outputs (NULL to skip):
 *   topk_idx_dev [T, N_k] int32  selected routed experts, descending key, ties to lowest id
 *   scores_dev   [T, N_r] fp32   router scores s of Eq. 8
 *   counts_dev   [N_r]    int32  tokens routed to each expert in this batch
 * T = 0 is a no-op.  Errors: CMOE_EINVAL (null x/y/workspace, T < 0, workspace_bytes too small),
 * CMOE_ESTATE (not uploaded), CMOE_EHIP (launch failure). */
int cmoe_forward(cmoe_layer* layer, const void* x_dev, int64_t T, void* y_dev,
                 int32_t* topk_idx_dev, float* scores_dev, int32_t* counts_dev,
                 void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* cmoe_forward for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and error rules as
 * cmoe_forward, but the workspace is a static device array inside the library (cmoe_static_scratch_bytes()
 * = 32 MiB, held by every GPU the library runs on until the process ends); the call allocates nothing and
 * frees nothing.  The device that holds the layer's weights must be current.  A batch whose workspace would
 * not fit is rejected with CMOE_EINVAL and a message that names the limit; cmoe_forward_static_max_tokens
 * gives the largest batch that fits for this layer (about 600 tokens for a 4096-wide layer with four slots
 * per token).  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two host threads) race; calls enqueued on one stream are ordered and safe.  Nothing in the array
 * has to be cleared between calls.  Partial sums of a K-split contraction get at most 8 MiB here, so a
 * batch of a few hundred tokens may split K differently than under cmoe_forward (same result within the
 * bf16 tolerance, not bit for bit). */
int cmoe_forward_static(cmoe_layer* layer, const void* x_dev, int64_t T, void* y_dev,
                        int32_t* topk_idx_dev, float* scores_dev, int32_t* counts_dev, void* hip_stream);
size_t cmoe_static_scratch_bytes(void);
int64_t cmoe_forward_static_max_tokens(const cmoe_layer* layer);

/* The dense FFN F(x) of Eq. 3 on the same layer, with kernels of the same quality as the MoE
 * path (one group, all tokens, all d_h neurons, no expert padding).  Same argument rules. */
int cmoe_dense_forward(cmoe_layer* layer, const void* x_dev, int64_t T, void* y_dev,
                       void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* Measurement aid: cmoe_forward (dense = 0) or cmoe_dense_forward (dense = 1) with HIP events recorded
 * on the stream between the stages; waits for the last event and writes the elapsed milliseconds of
 * the five stages to stage_ms[5] (host): router scoring + top-k (Eq. 8/9), permutation, gate/up
 * contraction with SwiGLU (Eq. 3 line 1), down contraction (Eq. 3 line 2), gate-weighted combine
 * (Eq. 4).  Stages a path does not run report ~0.  Synchronises; not for production use. */
int cmoe_forward_timed(cmoe_layer* layer, int dense, const void* x_dev, int64_t T, void* y_dev,
                       void* workspace_dev, size_t workspace_bytes, void* hip_stream, float* stage_ms);

void cmoe_destroy(cmoe_layer* layer);

/* ---- hierarchical case (Sec. 4.4, Eq. 10) ------------------------------------------------ */

/* An existing MoE layer with n_outer experts and a linear top-`outer_top_k` router
 * (logits = x W_router + logit_offset, weights = softmax over the selected logits, ties to the
 * lowest id), each of whose experts has been restructured into a cmoe_layer with the same
 * cmoe_config.  `experts` [n_outer] are handles built by cmoe_build / _from_partition; the
 * hierarchy borrows them (they must outlive it and must not be uploaded separately).
 * w_router: host fp32 [d, n_outer]; logit_offset: host fp32 [n_outer] or NULL. */
int cmoe_hier_create(cmoe_layer* const* experts, int32_t n_outer, int32_t outer_top_k,
                     const float* w_router, const float* logit_offset, cmoe_hier** out);

/* The same from the un-restructured MoE layer (Sec. 4.4): w_gate / w_up / w_down are arrays of n_outer host
 * pointers to the experts' dense matrices ([d, d_h], [d, d_h], [d_h, d] each, fp32), calib_x [q, d] one
 * calibration set for the whole layer.  The calibration tokens are routed by the outer router on the host
 * (double precision on the dtype-rounded operands, top-`outer_top_k`, ties to the lowest id); outer expert e
 * is then restructured as by cmoe_build (cmoe_build_gpu when on_gpu != 0) on the tokens whose selection
 * contains e, in their original order, or on the whole set when fewer than max(min_tokens, K_a) tokens reach
 * it (min_tokens <= 0 means 64).  The paper does not say which tokens profile which expert; this is the
 * reading taken.  with_baseline = 0 leaves out the un-restructured copy (cmoe_hier_dense_forward then
 * returns CMOE_ESTATE).  The hierarchy owns the experts it built: cmoe_hier_destroy frees them. */
int cmoe_hier_build(const cmoe_config* cfg, int32_t n_outer, int32_t outer_top_k, const float* const* w_gate,
                    const float* const* w_up, const float* const* w_down, const float* w_router,
                    const float* logit_offset, const float* calib_x, int64_t q, int32_t min_tokens, int on_gpu,
                    int with_baseline, cmoe_hier** out);

/* Outer expert e of a hierarchy as a borrowed handle (valid until cmoe_hier_destroy; use it with
 * cmoe_export_partition / cmoe_get_gate_params only), NULL if e is out of range.  calib_routed / calib_used
 * (either may be NULL) receive how many calibration tokens the outer router sent to the expert and how
 * many it was profiled on in cmoe_hier_build (-1 for a hierarchy made by cmoe_hier_create). */
const cmoe_layer* cmoe_hier_expert(const cmoe_hier* h, int32_t e, int64_t* calib_routed, int64_t* calib_used);

size_t cmoe_hier_packed_bytes(const cmoe_hier* h);
size_t cmoe_hier_workspace_bytes(const cmoe_hier* h, int64_t max_tokens);
int cmoe_hier_upload(cmoe_hier* h, void* dev_weights, void* hip_stream);

/* y[t] = sum over the selected outer experts e of w_e * (E^s_e(x) + sum_j g'_{e,j} E^r_{e,j}(x)).
 * Optional device outputs: outer_idx_dev [T, outer_top_k] int32; sub_idx_dev
 * [T, outer_top_k, N_k] int32 (sub-experts chosen inside each selected outer expert). */
int cmoe_hier_forward(cmoe_hier* h, const void* x_dev, int64_t T, void* y_dev,
                      int32_t* outer_idx_dev, int32_t* sub_idx_dev,
                      void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* The un-restructured MoE layer (every outer expert evaluated densely), the baseline of the
 * hierarchical case. */
int cmoe_hier_dense_forward(cmoe_hier* h, const void* x_dev, int64_t T, void* y_dev,
                            void* workspace_dev, size_t workspace_bytes, void* hip_stream);
/* Measurement aid, as cmoe_forward_timed (Eq. 10 path when dense = 0). */
int cmoe_hier_forward_timed(cmoe_hier* h, int dense, const void* x_dev, int64_t T, void* y_dev,
                            void* workspace_dev, size_t workspace_bytes, void* hip_stream, float* stage_ms);
void cmoe_hier_destroy(cmoe_hier* h);

/* ---- misc -------------------------------------------------------------------------------- */

/* Measurement aid for the roofline of the expert contractions (Eq. 3 restricted to neuron slices,
 * Sec. 4.1): the rate the matrix cores of the current device sustain when nothing else is in use.
 * One workgroup of eight waves per CU issues v_mfma_f32_32x32x16_bf16 back to back out of registers,
 * `iters` rounds of 8 per wave (1 <= iters <= 2^22), with all-zero operands (random_operands = 0) or
 * fixed normally distributed ones (1).  Writes the achieved TFLOP/s to *tflops (host) and, if
 * shader_mhz is not NULL, the shader clock observed meanwhile.  Allocates and frees 20 KB of device
 * memory, runs on the null stream and synchronises; not part of the forward path. */
int cmoe_probe_mfma(int random_operands, int iters, double* tflops, double* shader_mhz);

/* Measurement aid for the roofline of the weight-streaming decode kernels (the per-neuron form of the FFN,
 * Eq. 1, on the selected experts of Eq. 4): the rate at which the current device reads `bytes` of device
 * memory (rounded down to a multiple of 256 KB; choose more than the 256 MB last-level cache) when every
 * load instruction covers 1 KB of consecutive bytes and nothing else is done with the data.  Best of
 * `reps` launches after one warm-up, event-timed (the 4-5 us an event pair costs are inside), in GB/s to
 * *gbytes_per_s (host).  Allocates, zero-fills and frees the buffer, runs on the null stream and
 * synchronises; not part of the forward path. */
int cmoe_probe_hbm(size_t bytes, int reps, double* gbytes_per_s);

/* Tuning switch `name` (the names of the environment variables the library reads once at first use:
 * CMOE_GEMM1_CFG, CMOE_GEMM2_CFG, CMOE_XCD_REMAP, CMOE_SPLITK, CMOE_ZERO_PAD, CMOE_DECODE_FUSE,
 * CMOE_FRONT_SHARED, CMOE_FORCE_SIMT, CMOE_LDPAD, CMOE_HOST_THREADS, CMOE_SKIP_ROWS, CMOE_DECODE_SPLIT,
 * CMOE_WS_DOWN, CMOE_SKIP_STAGE, CMOE_REPEAT_STAGE, CMOE_FRONT_ALL, CMOE_FRONT_TILE) takes `value` from the next call on; -1
 * restores the per-batch choice of the tile-shape switches.  For A/B measurements and tests inside one process; every default is the measured best.  Not
 * synchronised against forwards being enqueued from other host threads.  CMOE_SKIP_STAGE = 3, 4 or 5 is a
 * measurement aid: every forward then leaves out its gate/up, down or combine launch (its output is
 * meaningless), and the time a loop of forwards loses is what that stage costs inside the stream, launch gap
 * included (6: a batch of at most 64 tokens runs its scoring launch and nothing else);
 * CMOE_REPEAT_STAGE = 3, 4 or 5 launches that stage twice instead (same inputs and outputs: the
 * result is unchanged), and the time a loop gains is one more launch of it under the forward's own clocks
 * (6: the scoring launch of a batch of at most 16 tokens twice).  0 restores the plain forward.  CMOE_EINVAL on an unknown name. */
int cmoe_set_tuning(const char* name, int value);

const char* cmoe_last_error(void);   /* thread-local, never NULL */
const char* cmoe_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CMOE_H */
