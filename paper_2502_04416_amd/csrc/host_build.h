// Host-side construction of the partition and the router (Sec. 4.1-4.2, App. A.2-A.4).
#pragma once
#include <cstdint>
#include <string>
#include "../../include/cmoe.h"
#include "host_pack.h"

namespace cmoe {

// Profile the calibration tokens, select the shared neurons, cluster the rest into balanced groups
// and pick the representative neurons.  Outputs: neuron_order [d_ff] (shared first, then routed expert
// 0.. with m ids each), rep_neuron [N_r], mu [d_ff], cost of the last assignment.  Returns false and a
// message on failure.
bool host_construct(const cmoe_config& cfg, const RoundedDense& rd, const float* calib_x, int64_t q,
                    int32_t* neuron_order, int32_t* rep_neuron, float* mu, double* cost, std::string* msg);

// The two halves of host_construct.  host_profile: App. A.2 steps 1-2, active [q][k_act] = the K_a neurons of
// largest |h| of every calibration token (descending magnitude, ties to the lowest index).
// host_construct_from_active: everything after that (rates, shared neurons, balanced clustering,
// representatives) from such a list, however it was obtained.
void host_profile(const cmoe_config& cfg, const RoundedDense& rd, const float* calib_x, int64_t q, int32_t* active);
bool host_construct_from_active(const cmoe_config& cfg, int64_t q, const int32_t* active, int32_t* neuron_order,
                                int32_t* rep_neuron, float* mu, double* cost, std::string* msg);

// App. A.2 steps 1-2 on the current HIP device (bf16 layers, d_model a multiple of 64): hidden states of
// the calibration tokens by bf16 MFMA with fp32 accumulation, then the per-token top-K_a of |h| (same tie
// rule).  Allocates and frees its own device memory and synchronises.  Returns a HIP error code as int
// (0 = success) and a message.
int gpu_profile(const cmoe_config& cfg, const RoundedDense& rd, const float* calib_x, int64_t q, int32_t* active,
                std::string* msg);

// Exact balanced assignment (App. A.3) on a dense distance matrix; see host_build.cpp.
bool solve_balanced_assignment(const double* dist, int n, int n_r, int m, int32_t* label_out, double* cost_out,
                               std::string* msg);

}  // namespace cmoe
