"""CPU oracle for the analytical FFN-to-MoE restructuring and its forward pass.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 numpy implementation of
what the paper defines; it exists to check the HIP library and shares no code
with it.  Only the tests, the smoke check and the bench's cpu_baseline leg may
import it.  The product path never does.

Every function states the passage of the paper it follows.  All arithmetic is
fp64 on whatever (already dtype-rounded) inputs it is handed.  Matrix products
use numpy's matmul as a library step; nothing is blocked, fused or reordered.

Readings taken where the paper is silent (each is also listed in the design
notes of the repository):
  * Swish is SiLU, z * sigmoid(z) (beta = 1).
  * The selection key is the signed score s of Eq. 8/9 (option: |s|).
  * Every tie (ATopK, top-mu, centroid init, representative argmin, top-N_k)
    goes to the lowest index.
  * Distances are the L2 norm with the square root as printed in App. A.3
    (option: squared).
  * One assignment + one centroid update per K-means iteration; the
    representative neuron is taken against the mean of the final members.
  * Outer router of the hierarchical case: linear logits plus offsets, top-k,
    softmax over the selected logits; the outer weight multiplies the whole
    restructured expert (shared part included).

Parity unpinned by the paper (no printed example fixes them): the signed-score
reading, the iteration count, the centroid used for the representative neuron,
per-expert calibration in the hierarchical build (`hier_build`), the form of the
neuron-level sparsity criterion inside routed experts (`neuron_keep_mask`).  `build`,
`hier_build` and `hier_forward`'s outer gate therefore carry "parity unpinned"
for those choices: the code that implements each reading is pinned (hand-worked
examples, exhaustive search, loops written out in the tests), the choice of
reading is not.  Everything else is pinned by tests/test_oracle_pins.py.
"""
from __future__ import annotations

import itertools
from typing import Dict, Optional, Sequence, Tuple

import numpy as np
from scipy.optimize import linear_sum_assignment

F64 = np.float64


# --------------------------------------------------------------------------- dense FFN

def swish(z: np.ndarray) -> np.ndarray:
    """Swish / SiLU with beta = 1: z * sigmoid(z)  (Sec. 4.1, Eq. 3)."""
    z = np.asarray(z, dtype=F64)
    return z / (1.0 + np.exp(-z))


def hidden_states(x: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray) -> np.ndarray:
    """H = Swish(X W_gate) * (X W_up), shape [q, d_h]  (App. A.2 step 1; Eq. 3 first line)."""
    x = np.asarray(x, dtype=F64)
    return swish(x @ np.asarray(w_gate, dtype=F64)) * (x @ np.asarray(w_up, dtype=F64))


def dense_ffn(x: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray) -> np.ndarray:
    """F(x) = W_down^T h, rows of x are tokens  (Sec. 4.1, Eq. 3)."""
    return hidden_states(x, w_gate, w_up) @ np.asarray(w_down, dtype=F64)


def dense_ffn_by_neuron(x_row: np.ndarray, w_gate, w_up, w_down) -> np.ndarray:
    """F(x) = sum_i h_i w_i, one neuron at a time, for a single token  (Sec. 3.1, Eq. 1).
    Pure loop; only for small cases."""
    x_row = np.asarray(x_row, dtype=F64)
    d_h = w_gate.shape[1]
    out = np.zeros(w_down.shape[1], dtype=F64)
    for i in range(d_h):
        a = float(np.dot(x_row, np.asarray(w_gate[:, i], dtype=F64)))
        b = float(np.dot(x_row, np.asarray(w_up[:, i], dtype=F64)))
        h_i = a / (1.0 + np.exp(-a)) * b
        out += h_i * np.asarray(w_down[i, :], dtype=F64)
    return out


# --------------------------------------------------------------------------- (A) profiling

def _stable_top(values: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries, descending, ties to the lowest index."""
    order = np.argsort(-np.asarray(values, dtype=F64), kind="stable")
    return order[:k]


def atopk_matrix(h: np.ndarray, k_act: int) -> np.ndarray:
    """A[t, i] = 1 iff |h_i| is among the K_a largest magnitudes of token t  (App. A.2 step 2).
    Returns a boolean [q, d_h] matrix whose columns are the feature vectors c_i."""
    h = np.asarray(h, dtype=F64)
    a = np.zeros(h.shape, dtype=bool)
    for t in range(h.shape[0]):
        a[t, _stable_top(np.abs(h[t]), k_act)] = True
    return a


def activation_rates(a: np.ndarray) -> np.ndarray:
    """mu_i = (1/q) sum_t A[t, i]  (App. A.2 step 3)."""
    return a.astype(F64).sum(axis=0) / a.shape[0]


def select_shared(mu: np.ndarray, n_shared_neurons: int) -> np.ndarray:
    """The N_s * m neurons with the highest activation rate, in descending-rate order
    (Sec. 4.1 'Shared Experts'; App. A.2 step 4)."""
    return _stable_top(mu, n_shared_neurons)


# --------------------------------------------------------------------------- (B) balanced clustering

def init_centroids(a: np.ndarray, mu: np.ndarray, remaining: np.ndarray, n_routed: int) -> np.ndarray:
    """Initial centroids = feature vectors of the N_r remaining neurons with the highest
    rate (App. A.3 'Centroid Initialization').  Returns [N_r, q] float."""
    pick = remaining[_stable_top(mu[remaining], n_routed)]
    return a[:, pick].T.astype(F64)


def distance_matrix(feat: np.ndarray, centroids: np.ndarray, squared: bool = False) -> np.ndarray:
    """d_ij = || c_i - c^_j ||_2 over the q calibration tokens (App. A.3 'Distance Matrix').
    feat: [n, q] rows are the c_i; centroids: [N_r, q].  `squared=True` drops the root."""
    feat = np.asarray(feat, dtype=F64)
    centroids = np.asarray(centroids, dtype=F64)
    d2 = np.zeros((feat.shape[0], centroids.shape[0]), dtype=F64)
    for j in range(centroids.shape[0]):
        diff = feat - centroids[j][None, :]
        d2[:, j] = np.sum(diff * diff, axis=1)
    return d2 if squared else np.sqrt(d2)


def balanced_assignment(dist: np.ndarray, m: int) -> np.ndarray:
    """min sum T_ij d_ij  s.t. every cluster gets exactly m rows and every row one cluster
    (App. A.3 'Balanced Assignment').  Solved exactly as the paper states: every column is
    repeated m times and the square linear assignment problem is handed to a
    Jonker-Volgenant-type solver (scipy's linear_sum_assignment).  Returns label[i] in [0, N_r)."""
    n, n_r = dist.shape
    assert n == n_r * m, "balanced assignment needs exactly N_r * m rows"
    square = np.repeat(np.asarray(dist, dtype=F64), m, axis=1)      # column j*m + r  ->  cluster j
    rows, cols = linear_sum_assignment(square)
    label = np.empty(n, dtype=np.int64)
    label[rows] = cols // m
    return label


def balanced_assignment_bruteforce(dist: np.ndarray, m: int) -> Tuple[np.ndarray, float]:
    """Exhaustive search over all assignments with exactly m rows per cluster (tiny inputs
    only).  Returns (one optimal labelling, the optimal cost)."""
    n, n_r = dist.shape
    assert n == n_r * m and n <= 12
    best_cost, best = np.inf, None
    for label in itertools.product(range(n_r), repeat=n):
        if any(label.count(j) != m for j in range(n_r)):
            continue
        c = sum(dist[i, label[i]] for i in range(n))
        if c < best_cost:
            best_cost, best = c, label
    return np.array(best, dtype=np.int64), float(best_cost)


def assignment_cost(dist: np.ndarray, label: np.ndarray) -> float:
    return float(np.asarray(dist, dtype=F64)[np.arange(dist.shape[0]), label].sum())


def update_centroids(feat: np.ndarray, label: np.ndarray, prev: np.ndarray) -> np.ndarray:
    """c^_j <- mean of the assigned c_i, unchanged if the cluster is empty (App. A.3 'Cluster Update')."""
    new = np.array(prev, dtype=F64, copy=True)
    for j in range(prev.shape[0]):
        members = np.nonzero(label == j)[0]
        if members.size > 0:
            new[j] = np.asarray(feat[members], dtype=F64).sum(axis=0) / members.size
    return new


# --------------------------------------------------------------------------- (C) router

def representative_neurons(feat: np.ndarray, label: np.ndarray, centroids: np.ndarray) -> np.ndarray:
    """R_j = argmin over the members i of cluster j of ||c_i - c^_j||_2  (Sec. 4.2, Eq. 7).
    Returns positions into `feat` (ties to the lowest position)."""
    reps = np.empty(centroids.shape[0], dtype=np.int64)
    for j in range(centroids.shape[0]):
        members = np.nonzero(label == j)[0]
        diff = np.asarray(feat[members], dtype=F64) - centroids[j][None, :]
        d = np.sqrt(np.sum(diff * diff, axis=1))
        reps[j] = members[int(np.argmin(d))]      # argmin returns the first minimum
    return reps


def build(w_gate, w_up, calib_x, n_experts: int, n_shared: int, k_act: int = 10,
          kmeans_iters: int = 1, squared_dist: bool = False) -> Dict[str, np.ndarray]:
    """Stages (A)-(C) of Sec. 4 on one dense FFN: profile, split off the shared neurons,
    cluster the rest into N_r balanced groups, pick one representative neuron per group.

    Returns
      neuron_order [d_h]  dense neuron ids: the N_s*m shared ones first (descending rate),
                          then routed expert 0, 1, ... (m each, ascending neuron id inside)
      rep_neuron   [N_r]  dense neuron id of R_j
      mu           [d_h]  activation rates
      label        [N_r*m] cluster of each remaining neuron (remaining in ascending id)
      cost         float  objective of the last assignment
      label_history, cost_history   the same for every round that ran, in order
    """
    d_h = w_gate.shape[1]
    assert d_h % n_experts == 0
    m = d_h // n_experts
    n_routed = n_experts - n_shared
    h = hidden_states(calib_x, w_gate, w_up)
    a = atopk_matrix(h, k_act)
    mu = activation_rates(a)
    shared = select_shared(mu, n_shared * m)
    is_shared = np.zeros(d_h, dtype=bool)
    is_shared[shared] = True
    remaining = np.nonzero(~is_shared)[0]                       # ascending neuron id
    feat = a[:, remaining].T.astype(F64)                        # [N_r*m, q]
    centroids = init_centroids(a, mu, remaining, n_routed)
    label, cost, prev_label = None, np.nan, None
    label_history, cost_history = [], []
    for _ in range(max(1, kmeans_iters)):
        dist = distance_matrix(feat, centroids, squared=squared_dist)
        label = balanced_assignment(dist, m)
        cost = assignment_cost(dist, label)
        label_history.append(label)
        cost_history.append(cost)
        centroids = update_centroids(feat, label, centroids)
        if prev_label is not None and np.array_equal(prev_label, label):
            break
        prev_label = label
    reps_pos = representative_neurons(feat, label, centroids)
    order = [shared]
    for j in range(n_routed):
        order.append(remaining[label == j])
    return {
        "neuron_order": np.concatenate(order).astype(np.int32),
        "rep_neuron": remaining[reps_pos].astype(np.int32),
        "mu": mu,
        "label": label,
        "cost": cost,
        "remaining": remaining,
        "label_history": label_history,
        "cost_history": cost_history,
    }


# --------------------------------------------------------------------------- MoE forward

def router_scores(x: np.ndarray, w_gate, w_up, rep_neuron: Sequence[int]) -> np.ndarray:
    """s = Swish(W_gate^R^T x) * (W_up^R^T x) with W^R the columns of the representative
    neurons  (Sec. 4.2, Eq. 8).  Returns [T, N_r]."""
    rep = np.asarray(rep_neuron, dtype=np.int64)
    return hidden_states(x, np.asarray(w_gate)[:, rep], np.asarray(w_up)[:, rep])


def softmax_rows(s: np.ndarray) -> np.ndarray:
    s = np.asarray(s, dtype=F64)
    e = np.exp(s - s.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def select_top_k(key: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Per row: the k largest keys in descending order (ties to the lowest index) and the
    gap between the k-th and (k+1)-th largest key (inf when k equals the row length)."""
    key = np.asarray(key, dtype=F64)
    t, n = key.shape
    sel = np.empty((t, k), dtype=np.int64)
    gap = np.full(t, np.inf, dtype=F64)
    for r in range(t):
        order = np.argsort(-key[r], kind="stable")
        sel[r] = order[:k]
        if k < n:
            gap[r] = key[r, order[k - 1]] - key[r, order[k]]
    return sel, gap


def expert_output(x: np.ndarray, w_gate, w_up, w_down, neurons: np.ndarray) -> np.ndarray:
    """One expert = the SwiGLU FFN of Eq. 3 restricted to a set of neurons: columns of
    W_gate/W_up and rows of W_down sliced by neuron index  (Sec. 4.1 'Shared Experts')."""
    idx = np.asarray(neurons, dtype=np.int64)
    return dense_ffn(x, np.asarray(w_gate)[:, idx], np.asarray(w_up)[:, idx], np.asarray(w_down)[idx, :])


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 value of every entry, ties to even, returned as float64 (finite inputs).
    bfloat16 keeps the upper 16 bits of the IEEE single-precision pattern."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(f.shape).astype(F64)


def neuron_keep_mask(h: np.ndarray, w_down_rows: np.ndarray, tau: float, weight_informed: bool = False,
                     decide_in_bf16: bool = False) -> np.ndarray:
    """Which hidden activations of a routed expert survive neuron-level activation sparsity (Sec. 5,
    'Orthogonality with Activation Sparsity'; Broader-impact paragraph: training-free activation sparsity
    applied inside the routed experts).  The paper names the family (magnitude- or weight-informed
    thresholds) and gives no formula; the reading taken (parity unpinned by the paper):
      magnitude        keep h_n  iff  |h_n| >= tau
      weight-informed  keep h_n  iff  |h_n| * ||w_n||_2 >= tau,  w_n = row n of W_down (the neuron's output direction)
    A dropped neuron contributes nothing to F(x) = sum_n h_n w_n (Eq. 1).  decide_in_bf16: the comparison is
    made on h rounded to bfloat16 (and the norm rounded to single precision), the precision in which the
    device kernels of a bf16 layer hold h when they take the same decision; the surviving h_n keep their
    full-precision value either way."""
    h = np.asarray(h, dtype=F64)
    key = np.abs(round_to_bf16(h)) if decide_in_bf16 else np.abs(h)
    if weight_informed:
        norm = np.sqrt(np.sum(np.asarray(w_down_rows, dtype=F64) ** 2, axis=1))
        if decide_in_bf16:
            norm = norm.astype(np.float32).astype(F64)
            key = (key.astype(np.float32) * norm.astype(np.float32)[None, :]).astype(F64)      # one fp32 product
        else:
            key = key * norm[None, :]
    return key >= tau


def sparse_expert_output(x, w_gate, w_up, w_down, neurons, tau: float, weight_informed: bool = False,
                         decide_in_bf16: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """One routed expert with neuron-level sparsity: sum over the surviving neurons of h_n w_n (Eq. 1 on the
    expert's slice, Eq. 3 otherwise).  Returns (output [T, d], keep mask [T, m])."""
    idx = np.asarray(neurons, dtype=np.int64)
    h = hidden_states(x, np.asarray(w_gate)[:, idx], np.asarray(w_up)[:, idx])
    wd = np.asarray(w_down, dtype=F64)[idx, :]
    keep = neuron_keep_mask(h, wd, tau, weight_informed, decide_in_bf16)
    return (h * keep) @ wd, keep


def moe_forward(x, w_gate, w_up, w_down, neuron_order, rep_neuron, n_experts: int, n_shared: int,
                top_k: int, u: Optional[np.ndarray] = None, b: Optional[np.ndarray] = None,
                abs_score: bool = False, sel_override: Optional[np.ndarray] = None,
                neuron_tau: Optional[float] = None, neuron_weight_informed: bool = False,
                neuron_decide_in_bf16: bool = False) -> Dict[str, np.ndarray]:
    """F_MoE(x) = E^s(x) + sum_i g_i E^r_i(x)  (Eq. 4) with the gate of Eq. 9:
    g_i = 1 + s'_i u_i if s'_i + b_i is among the top N_k, else 0; s' = Softmax(s), s from Eq. 8.

    With u = b = None (both zero) the selection key is s itself: Softmax is strictly
    monotone per row, so the ordering is the same and no rounding of exp() can create a tie.
    `sel_override` [T, N_k] replaces the selection (used to evaluate a different but equally
    valid choice at near-ties).  neuron_tau (not None) applies neuron-level activation sparsity inside the
    routed experts, never the shared ones (see neuron_keep_mask).
    Returns y, scores, sel (descending key), gap, gate [T, N_k], kept (surviving / evaluated routed neurons).
    """
    x = np.asarray(x, dtype=F64)
    order = np.asarray(neuron_order, dtype=np.int64)
    d_h = order.shape[0]
    m = d_h // n_experts
    n_routed = n_experts - n_shared
    s = router_scores(x, w_gate, w_up, rep_neuron)
    s_key = np.abs(s) if abs_score else s
    plain = u is None and b is None
    if plain:
        key = s_key
        s_prime = None
    else:
        s_prime = softmax_rows(s_key)
        key = s_prime + (0.0 if b is None else np.asarray(b, dtype=F64)[None, :])
    sel, gap = select_top_k(key, top_k)
    if sel_override is not None:
        sel = np.asarray(sel_override, dtype=np.int64)
    t = x.shape[0]
    gate = np.ones((t, top_k), dtype=F64)
    if not plain and u is not None:
        uu = np.asarray(u, dtype=F64)
        for r in range(t):
            gate[r] = 1.0 + s_prime[r, sel[r]] * uu[sel[r]]
    y = expert_output(x, w_gate, w_up, w_down, order[: n_shared * m])          # E^s
    kept, evaluated = 0, 0
    for j in range(n_routed):
        neurons = order[(n_shared + j) * m: (n_shared + j + 1) * m]
        rows, slot = np.nonzero(sel == j)
        if rows.size == 0:
            continue
        if neuron_tau is None:
            e_out = expert_output(x[rows], w_gate, w_up, w_down, neurons)
        else:
            e_out, keep = sparse_expert_output(x[rows], w_gate, w_up, w_down, neurons, neuron_tau,
                                               neuron_weight_informed, neuron_decide_in_bf16)
            kept += int(keep.sum())
            evaluated += keep.size
        y[rows] += gate[rows, slot][:, None] * e_out
    return {"y": y, "scores": s, "sel": sel, "gap": gap, "gate": gate,
            "kept": (kept / evaluated) if evaluated else 1.0}


def moe_forward_one_token(x_row, w_gate, w_up, w_down, neuron_order, rep_neuron, n_experts, n_shared,
                          top_k, u=None, b=None, sel_override=None, abs_score: bool = False) -> Dict[str, np.ndarray]:
    """The same computation for a single token (used to sample outputs of large batches)."""
    so = None if sel_override is None else np.asarray(sel_override).reshape(1, -1)
    out = moe_forward(np.asarray(x_row)[None, :], w_gate, w_up, w_down, neuron_order, rep_neuron,
                      n_experts, n_shared, top_k, u=u, b=b, abs_score=abs_score, sel_override=so)
    return {k: (v[0] if isinstance(v, np.ndarray) else v) for k, v in out.items()}


def bias_update(b: np.ndarray, counts: np.ndarray, gamma: float = 1e-3) -> np.ndarray:
    """One load-balancing step (Sec. 4.3, text after Eq. 9): with p_i = counts_i / sum(counts) the
    utilisation of routed expert i and p* = 1/N_r, b_i decreases by gamma where p_i > p*, increases by
    gamma where p_i < p*, and stays where p_i = p*.  Nothing changes when no token was routed.
    The comparison is done on integers (counts_i * N_r against sum(counts)), which is the same test."""
    b = np.asarray(b, dtype=F64).copy()
    c = np.asarray(counts, dtype=np.int64)
    total = int(c.sum())
    if total == 0:
        return b
    n_r = c.shape[0]
    b[c * n_r > total] -= gamma
    b[c * n_r < total] += gamma
    return b


# --------------------------------------------------------------------------- hierarchical

def outer_route(x, w_router, offsets, outer_top_k: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Top-level router of an existing MoE layer (Sec. 4.4): logits = x W_router + offsets,
    top-k experts (ties to the lowest index), weights = softmax over the selected logits.
    Returns (sel [T,k], weight [T,k], gap [T])."""
    logits = np.asarray(x, dtype=F64) @ np.asarray(w_router, dtype=F64) + np.asarray(offsets, dtype=F64)[None, :]
    sel, gap = select_top_k(logits, outer_top_k)
    picked = np.take_along_axis(logits, sel, axis=1)
    return sel, softmax_rows(picked), gap


def hier_forward(x, w_router, offsets, outer_top_k: int, experts: Sequence[dict], n_sub: int,
                 n_shared: int, top_k: int, outer_sel_override=None, sub_sel_override=None,
                 abs_score: bool = False) -> Dict[str, np.ndarray]:
    """Existing MoE layer whose every expert E_e has been restructured into
    E^s_e + sum_j g'_{e,j} E^r_{e,j}  (Sec. 4.4, Eq. 10):
        y = sum_{e in outer top-k} w_e * F_MoE^{(e)}(x).
    `experts[e]` holds w_gate, w_up, w_down, neuron_order, rep_neuron (and optional u, b).
    sub_sel_override: [T, outer_top_k, top_k] sub-expert choice per outer slot.
    Returns y, outer_sel, outer_weight, outer_gap, sub_sel [T, outer_top_k, top_k], sub_gap [T, outer_top_k]."""
    x = np.asarray(x, dtype=F64)
    t = x.shape[0]
    o_sel, o_w, o_gap = outer_route(x, w_router, offsets, outer_top_k)
    if outer_sel_override is not None:
        o_sel = np.asarray(outer_sel_override, dtype=np.int64)
        logits = x @ np.asarray(w_router, dtype=F64) + np.asarray(offsets, dtype=F64)[None, :]
        o_w = softmax_rows(np.take_along_axis(logits, o_sel, axis=1))
    y = np.zeros((t, experts[0]["w_down"].shape[1]), dtype=F64)
    sub_sel = np.full((t, outer_top_k, top_k), -1, dtype=np.int64)
    sub_gap = np.full((t, outer_top_k), np.inf, dtype=F64)
    for e, ex in enumerate(experts):
        rows, slot = np.nonzero(o_sel == e)
        if rows.size == 0:
            continue
        so = None if sub_sel_override is None else np.asarray(sub_sel_override)[rows, slot]
        out = moe_forward(x[rows], ex["w_gate"], ex["w_up"], ex["w_down"], ex["neuron_order"],
                          ex["rep_neuron"], n_sub, n_shared, top_k, u=ex.get("u"), b=ex.get("b"),
                          abs_score=abs_score, sel_override=so)
        y[rows] += o_w[rows, slot][:, None] * out["y"]
        sub_sel[rows, slot] = out["sel"]
        sub_gap[rows, slot] = out["gap"]
    return {"y": y, "outer_sel": o_sel, "outer_weight": o_w, "outer_gap": o_gap,
            "sub_sel": sub_sel, "sub_gap": sub_gap}


def hier_build(expert_weights: Sequence[Tuple[np.ndarray, np.ndarray]], w_router, offsets, outer_top_k: int,
               calib_x, n_sub: int, n_shared: int, k_act: int = 10, kmeans_iters: int = 1,
               squared_dist: bool = False, min_tokens: int = 64) -> Dict[str, list]:
    """Restructuring of every expert of an existing MoE layer (Sec. 4.4): stages (A)-(C) of Sec. 4 are
    applied to each expert E_e on its own.  The paper does not say which calibration tokens profile
    which expert; the reading taken here (parity unpinned): expert e is profiled on the calibration
    tokens whose outer top-k contains e, in their original order, and on the whole calibration set when
    fewer than max(min_tokens, K_a) tokens reach it.
    expert_weights[e] = (w_gate_e, w_up_e).  Returns per expert: parts (the dict of `build`),
    tokens (indices of the calibration tokens used), routed (how many tokens the outer router sent)."""
    calib_x = np.asarray(calib_x, dtype=F64)
    o_sel, _, _ = outer_route(calib_x, w_router, offsets, outer_top_k)
    parts, tokens, routed = [], [], []
    for e, (wg, wu) in enumerate(expert_weights):
        rows = np.nonzero((o_sel == e).any(axis=1))[0]
        routed.append(int(rows.size))
        if rows.size < max(min_tokens, k_act):
            rows = np.arange(calib_x.shape[0])
        tokens.append(rows)
        parts.append(build(wg, wu, calib_x[rows], n_sub, n_shared, k_act, kmeans_iters, squared_dist))
    return {"parts": parts, "tokens": tokens, "routed": routed}


def moe_layer_dense_experts(x, w_router, offsets, outer_top_k: int, experts: Sequence[dict]) -> np.ndarray:
    """The un-restructured MoE layer: y = sum_{e in top-k} w_e E_e(x), each E_e a dense SwiGLU FFN."""
    x = np.asarray(x, dtype=F64)
    o_sel, o_w, _ = outer_route(x, w_router, offsets, outer_top_k)
    y = np.zeros((x.shape[0], experts[0]["w_down"].shape[1]), dtype=F64)
    for e, ex in enumerate(experts):
        rows, slot = np.nonzero(o_sel == e)
        if rows.size:
            y[rows] += o_w[rows, slot][:, None] * dense_ffn(x[rows], ex["w_gate"], ex["w_up"], ex["w_down"])
    return y


# --------------------------------------------------------------------------- bookkeeping

def layer_flops_per_token(d: int, m: int, n_shared: int, n_routed: int, top_k: int) -> Tuple[int, int]:
    """(MoE flops, dense flops) per token: 6 d m per active expert of m neurons plus
    4 d N_r for the router; dense = 6 d d_h  (bookkeeping behind the paper's FLOPs table)."""
    moe = 6 * d * m * (n_shared + top_k) + 4 * d * n_routed
    dense = 6 * d * m * (n_shared + n_routed)
    return moe, dense
