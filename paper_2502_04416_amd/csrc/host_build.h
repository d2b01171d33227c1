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

// Exact balanced assignment (App. A.3) on a dense distance matrix; see host_build.cpp.
bool solve_balanced_assignment(const double* dist, int n, int n_r, int m, int32_t* label_out, double* cost_out,
                               std::string* msg);

}  // namespace cmoe
