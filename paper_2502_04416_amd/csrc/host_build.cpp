// Host-side construction (one-off, off the GPU hot path): activation profiling, shared-neuron
// selection, balanced clustering of the remaining neurons and representative-neuron selection
// (Sec. 4.1-4.2, App. A.2-A.4).  All ties go to the lowest index.  Arithmetic is double precision on
// the dtype-rounded weights and calibration tokens.
#include "host_build.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <numeric>
#include <queue>
#include <string>
#include <vector>

namespace cmoe {

namespace {

inline float load_elem(const uint8_t* p, int dtype) {
  if (dtype == CMOE_BF16) {
    uint16_t b;
    std::memcpy(&b, p, 2);
    return host_bf16_to_f32(b);
  }
  float f;
  std::memcpy(&f, p, 4);
  return f;
}

// dot product of two float rows accumulated in double, eight independent partial sums
inline double dot_f32_f64(const float* a, const float* b, int n) {
  double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  int k = 0;
  for (; k + 8 <= n; k += 8)
    for (int l = 0; l < 8; ++l) acc[l] += (double)a[k + l] * (double)b[k + l];
  for (; k < n; ++k) acc[k & 7] += (double)a[k] * (double)b[k];
  return ((acc[0] + acc[4]) + (acc[1] + acc[5])) + ((acc[2] + acc[6]) + (acc[3] + acc[7]));
}

inline double swish(double z) { return z / (1.0 + std::exp(-z)); }

// ---- exact balanced assignment -----------------------------------------------------------------
// min sum_i d[i][label_i]  s.t. every cluster holds exactly m rows (App. A.3, 'Balanced Assignment').
// The paper solves it as a square assignment problem with every column repeated m times; this is the
// same transportation problem solved by successive shortest paths: start from the unconstrained
// optimum (every row at its nearest centroid) and, while some cluster is over-full, move one unit of
// excess along a shortest path of the cluster graph whose edge a->b costs the cheapest relabelling of
// a member of a to b.  The start has no negative cycle and shortest-path augmentation keeps it that
// way, so the final assignment is optimal.
struct HeapItem {
  double delta;
  int item;
  bool operator>(const HeapItem& o) const { return delta > o.delta || (delta == o.delta && item > o.item); }
};
using MinHeap = std::priority_queue<HeapItem, std::vector<HeapItem>, std::greater<HeapItem>>;

bool balanced_assignment(const std::vector<double>& dist, int n, int n_r, int m, std::vector<int>& label,
                         std::string* msg) {
  label.assign(n, 0);
  std::vector<int> count(n_r, 0);
  for (int i = 0; i < n; ++i) {
    int best = 0;
    for (int j = 1; j < n_r; ++j)
      if (dist[(size_t)i * n_r + j] < dist[(size_t)i * n_r + best]) best = j;
    label[i] = best;
    ++count[best];
  }
  if (n_r == 1) return true;
  // heap[a][b]: members of a keyed by the cost of relabelling them to b (lazy deletion)
  std::vector<MinHeap> heap((size_t)n_r * n_r);
  auto push_item = [&](int i) {
    const int a = label[i];
    const double* di = &dist[(size_t)i * n_r];
    for (int b = 0; b < n_r; ++b)
      if (b != a) heap[(size_t)a * n_r + b].push(HeapItem{di[b] - di[a], i});
  };
  for (int i = 0; i < n; ++i) push_item(i);
  auto top_edge = [&](int a, int b, HeapItem& out) -> bool {
    MinHeap& h = heap[(size_t)a * n_r + b];
    while (!h.empty()) {
      const HeapItem& t = h.top();
      if (label[t.item] == a) {
        out = t;
        return true;
      }
      h.pop();
    }
    return false;
  };
  int64_t excess = 0;
  for (int j = 0; j < n_r; ++j) excess += std::max(0, count[j] - m);
  const double INF = std::numeric_limits<double>::infinity();
  std::vector<double> w((size_t)n_r * n_r), dmin(n_r);
  std::vector<int> witem((size_t)n_r * n_r), pred(n_r);
  for (int64_t it = 0; it < excess; ++it) {
    for (int a = 0; a < n_r; ++a)
      for (int b = 0; b < n_r; ++b) {
        HeapItem e;
        if (a != b && top_edge(a, b, e)) {
          w[(size_t)a * n_r + b] = e.delta;
          witem[(size_t)a * n_r + b] = e.item;
        } else {
          w[(size_t)a * n_r + b] = INF;
          witem[(size_t)a * n_r + b] = -1;
        }
      }
    // Bellman-Ford from all over-full clusters
    for (int a = 0; a < n_r; ++a) {
      dmin[a] = count[a] > m ? 0.0 : INF;
      pred[a] = -1;
    }
    for (int round = 0; round < n_r; ++round) {
      bool changed = false;
      for (int a = 0; a < n_r; ++a) {
        if (dmin[a] == INF) continue;
        for (int b = 0; b < n_r; ++b) {
          const double wab = w[(size_t)a * n_r + b];
          if (wab == INF) continue;
          if (dmin[a] + wab < dmin[b] - 1e-13) {
            dmin[b] = dmin[a] + wab;
            pred[b] = a;
            changed = true;
          }
        }
      }
      if (!changed) break;
    }
    int sink = -1;
    for (int b = 0; b < n_r; ++b)
      if (count[b] < m && dmin[b] < INF && (sink < 0 || dmin[b] < dmin[sink])) sink = b;
    if (sink < 0) {
      if (msg) *msg = "balanced assignment: no augmenting path";
      return false;
    }
    // collect the path (sink back to a source) and move one member along every edge
    std::vector<int> path;
    for (int v = sink; v >= 0 && (int)path.size() <= n_r; v = pred[v]) path.push_back(v);
    if ((int)path.size() > n_r || count[path.back()] <= m) {
      if (msg) *msg = "balanced assignment: inconsistent shortest-path tree";
      return false;
    }
    std::vector<int> moved;
    for (size_t k = path.size() - 1; k >= 1; --k) {
      const int a = path[k], b = path[k - 1];
      const int i = witem[(size_t)a * n_r + b];
      label[i] = b;          // heap entries of i under a become stale (lazy deletion)
      moved.push_back(i);
    }
    --count[path.back()];
    ++count[sink];
    for (int i : moved) push_item(i);
  }
  for (int j = 0; j < n_r; ++j)
    if (count[j] != m) {
      if (msg) *msg = "balanced assignment: cluster sizes are not balanced";
      return false;
    }
  return true;
}

}  // namespace

// exposed for the unit tests of the solver
bool solve_balanced_assignment(const double* dist, int n, int n_r, int m, int32_t* label_out, double* cost_out,
                               std::string* msg) {
  if (n != n_r * m) {
    if (msg) *msg = "need n == n_r * m";
    return false;
  }
  std::vector<double> d(dist, dist + (size_t)n * n_r);
  std::vector<int> label;
  if (!balanced_assignment(d, n, n_r, m, label, msg)) return false;
  double c = 0.0;
  for (int i = 0; i < n; ++i) {
    label_out[i] = label[i];
    c += d[(size_t)i * n_r + label[i]];
  }
  if (cost_out) *cost_out = c;
  return true;
}

void host_profile(const cmoe_config& cfg, const RoundedDense& rd, const float* calib_x, int64_t q, int32_t* active) {
  const int d = cfg.d_model, d_ff = cfg.d_ff, k_act = cfg.k_act;

  // calibration tokens rounded to the layer dtype, weights as floats (exact for bf16)
  std::vector<float> xs((size_t)q * d);
  for (size_t i = 0; i < xs.size(); ++i)
    xs[i] = cfg.dtype == CMOE_BF16 ? host_bf16_to_f32(host_f32_to_bf16(calib_x[i])) : calib_x[i];
  std::vector<float> wg((size_t)d_ff * d), wu((size_t)d_ff * d);
  const size_t es = elem_size(cfg.dtype);
  parallel_for(d_ff, [&](int64_t i) {
    for (int k = 0; k < d; ++k) {
      wg[(size_t)i * d + k] = load_elem(rd.gate_row(i) + (size_t)k * es, cfg.dtype);
      wu[(size_t)i * d + k] = load_elem(rd.up_row(i) + (size_t)k * es, cfg.dtype);
    }
  });

  // (A) profiling: per token, the K_a neurons of largest |h| (App. A.2 steps 1-2); A kept as per-token lists
  parallel_for(q, [&](int64_t t) {
    const float* x = &xs[(size_t)t * d];
    std::vector<double> keep_v(k_act, -1.0);
    std::vector<int32_t> keep_i(k_act, -1);
    int kept = 0;
    for (int i = 0; i < d_ff; ++i) {
      const double a = dot_f32_f64(x, &wg[(size_t)i * d], d);
      const double b = dot_f32_f64(x, &wu[(size_t)i * d], d);
      const double mag = std::fabs(swish(a) * b);
      // keep the K_a largest magnitudes; an equal magnitude at a higher index never displaces a kept one
      if (kept < k_act) {
        int p = kept++;
        while (p > 0 && keep_v[p - 1] < mag) { keep_v[p] = keep_v[p - 1]; keep_i[p] = keep_i[p - 1]; --p; }
        keep_v[p] = mag;
        keep_i[p] = i;
      } else if (mag > keep_v[k_act - 1]) {
        int p = k_act - 1;
        while (p > 0 && keep_v[p - 1] < mag) { keep_v[p] = keep_v[p - 1]; keep_i[p] = keep_i[p - 1]; --p; }
        keep_v[p] = mag;
        keep_i[p] = i;
      }
    }
    for (int k = 0; k < k_act; ++k) active[(size_t)t * k_act + k] = keep_i[k];
  });
}

bool host_construct(const cmoe_config& cfg, const RoundedDense& rd, const float* calib_x, int64_t q,
                    int32_t* neuron_order, int32_t* rep_neuron, float* mu_out, double* cost_out, std::string* msg) {
  std::vector<int32_t> active((size_t)q * cfg.k_act);
  host_profile(cfg, rd, calib_x, q, active.data());
  return host_construct_from_active(cfg, q, active.data(), neuron_order, rep_neuron, mu_out, cost_out, msg);
}

bool host_construct_from_active(const cmoe_config& cfg, int64_t q, const int32_t* active, int32_t* neuron_order,
                                int32_t* rep_neuron, float* mu_out, double* cost_out, std::string* msg) {
  const int d_ff = cfg.d_ff, N = cfg.n_experts, m = d_ff / N;
  const int n_s = cfg.n_shared, n_r = N - n_s, k_act = cfg.k_act;
  const int n = n_r * m;
  // feature vectors c_i as sorted token lists; rates mu_i (App. A.2 step 3)
  std::vector<std::vector<int32_t>> feat(d_ff);
  for (int64_t t = 0; t < q; ++t)
    for (int k = 0; k < k_act; ++k) {
      // (a token with fewer than K_a comparable magnitudes, i.e. non-finite hidden states, has no valid list)
      const int32_t i = active[(size_t)t * k_act + k];
      if (i < 0 || i >= d_ff) {
        if (msg) *msg = "calibration token " + std::to_string(t) + " has no valid top-K_a list (non-finite hidden states?)";
        return false;
      }
      feat[i].push_back((int32_t)t);
    }
  std::vector<double> mu(d_ff);
  for (int i = 0; i < d_ff; ++i) {
    mu[i] = (double)feat[i].size() / (double)q;
    mu_out[i] = (float)mu[i];
  }

  // (B) shared neurons: the N_s*m highest rates, stable (App. A.2 step 4)
  std::vector<int32_t> by_rate(d_ff);
  std::iota(by_rate.begin(), by_rate.end(), 0);
  std::stable_sort(by_rate.begin(), by_rate.end(), [&](int32_t a, int32_t b) { return feat[a].size() > feat[b].size(); });
  std::vector<char> is_shared(d_ff, 0);
  for (int i = 0; i < n_s * m; ++i) {
    neuron_order[i] = by_rate[i];
    is_shared[by_rate[i]] = 1;
  }
  std::vector<int32_t> remaining;
  remaining.reserve(n);
  for (int i = 0; i < d_ff; ++i)
    if (!is_shared[i]) remaining.push_back(i);
  // initial centroids: the N_r remaining neurons of highest rate (App. A.3); by_rate is already stable
  std::vector<double> cent((size_t)n_r * q, 0.0);
  {
    int j = 0;
    for (int i = n_s * m; i < d_ff && j < n_r; ++i, ++j)
      for (int32_t t : feat[by_rate[i]]) cent[(size_t)j * q + t] = 1.0;
  }

  std::vector<int> label, prev_label;
  std::vector<double> dist((size_t)n * n_r);
  double cost = 0.0;
  auto distances = [&](bool squared, std::vector<double>& out) {
    // ||c_i - c^_j||^2 = |c_i| - 2 sum_{t in c_i} c^_j[t] + ||c^_j||^2 for binary c_i
    std::vector<double> cn(n_r, 0.0);
    for (int j = 0; j < n_r; ++j) {
      double s = 0.0;
      for (int64_t t = 0; t < q; ++t) s += cent[(size_t)j * q + t] * cent[(size_t)j * q + t];
      cn[j] = s;
    }
    parallel_for(n, [&](int64_t r) {
      const std::vector<int32_t>& f = feat[remaining[r]];
      for (int j = 0; j < n_r; ++j) {
        double cross = 0.0;
        for (int32_t t : f) cross += cent[(size_t)j * q + t];
        double d2 = (double)f.size() - 2.0 * cross + cn[j];
        if (d2 < 0.0) d2 = 0.0;
        out[(size_t)r * n_r + j] = squared ? d2 : std::sqrt(d2);
      }
    });
  };
  auto update_centroids = [&]() {
    std::vector<int> members(n_r, 0);
    std::vector<double> sum((size_t)n_r * q, 0.0);
    for (int r = 0; r < n; ++r) {
      ++members[label[r]];
      for (int32_t t : feat[remaining[r]]) sum[(size_t)label[r] * q + t] += 1.0;
    }
    for (int j = 0; j < n_r; ++j)
      if (members[j] > 0)
        for (int64_t t = 0; t < q; ++t) cent[(size_t)j * q + t] = sum[(size_t)j * q + t] / members[j];
  };
  for (int it = 0; it < cfg.kmeans_iters; ++it) {
    distances(cfg.dist_mode == 1, dist);
    if (!balanced_assignment(dist, n, n_r, m, label, msg)) return false;
    cost = 0.0;
    for (int r = 0; r < n; ++r) cost += dist[(size_t)r * n_r + label[r]];
    update_centroids();
    if (!prev_label.empty() && prev_label == label) break;
    prev_label = label;
  }
  if (cost_out) *cost_out = cost;

  // (C) representative neurons against the centroid of the final members (Eq. 7)
  std::vector<double> dfin((size_t)n * n_r);
  distances(false, dfin);
  std::vector<int> rep_pos(n_r, -1);
  for (int r = 0; r < n; ++r) {
    const int j = label[r];
    if (rep_pos[j] < 0 || dfin[(size_t)r * n_r + j] < dfin[(size_t)rep_pos[j] * n_r + j]) rep_pos[j] = r;
  }
  std::vector<int> fill(n_r, 0);
  for (int r = 0; r < n; ++r) {
    const int j = label[r];
    neuron_order[(size_t)(n_s + j) * m + fill[j]++] = remaining[r];
  }
  for (int j = 0; j < n_r; ++j) rep_neuron[j] = remaining[rep_pos[j]];
  return true;
}

}  // namespace cmoe
