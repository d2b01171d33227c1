"""Host-side construction in libcmoe (cmoe_build, cmoe_balanced_assignment) against the CPU oracle.
No GPU is involved: construction is host code by design.

Several balanced assignments can be optimal (ties are generic with sparse binary feature vectors), so
partitions are compared through what is unique: rates, the shared set, the optimal cost, the
constraints, and the validity of each representative neuron inside the library's own clusters."""
import numpy as np
import pytest

from oracle import cmoe_oracle as O
from paper_2502_04416_amd import binding, synth


@pytest.fixture(scope="module", autouse=True)
def lib():
    return binding.load()


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


@pytest.mark.parametrize("n_r,m", [(3, 2), (2, 4), (3, 3), (4, 2), (2, 5)])
def test_solver_matches_bruteforce(n_r, m):
    r = _rng(10 * n_r + m)
    for trial in range(8):
        dist = r.random((n_r * m, n_r)) if trial % 2 == 0 else np.sqrt(r.integers(0, 4, size=(n_r * m, n_r)).astype(float))
        label, cost = binding.cmoe_balanced_assignment(dist, m)
        assert np.bincount(label, minlength=n_r).tolist() == [m] * n_r
        assert cost == pytest.approx(O.assignment_cost(dist, label), rel=1e-12, abs=1e-12)
        _, best = O.balanced_assignment_bruteforce(dist, m)
        assert cost == pytest.approx(best, rel=1e-12, abs=1e-12)


@pytest.mark.parametrize("n_r,m", [(5, 12), (7, 128), (15, 100), (30, 40)])
def test_solver_matches_replicated_column_assignment(n_r, m):
    """Same optimum as the paper's formulation (columns repeated m times, Jonker-Volgenant solver)."""
    r = _rng(1000 + n_r)
    for trial in range(2):
        n = n_r * m
        dist = r.random((n, n_r)) if trial == 0 else np.sqrt(r.integers(0, 6, size=(n, n_r)).astype(float))
        label, cost = binding.cmoe_balanced_assignment(dist, m)
        assert np.bincount(label, minlength=n_r).tolist() == [m] * n_r
        ref = O.assignment_cost(dist, O.balanced_assignment(dist, m))
        assert cost == pytest.approx(ref, rel=1e-9)


def test_solver_exchange_certificate_large():
    """At a size the replicated-column solver is slow for: optimal iff the cluster graph with edge costs
    min over members (d_ib - d_ia) has no negative cycle."""
    r = _rng(7)
    n_r, m = 28, 448
    n = n_r * m
    dist = np.sqrt(r.integers(0, 12, size=(n, n_r)).astype(float)) + 1e-3 * r.random((n, n_r))
    label, cost = binding.cmoe_balanced_assignment(dist, m)
    assert np.bincount(label, minlength=n_r).tolist() == [m] * n_r
    w = np.full((n_r, n_r), np.inf)
    for a in range(n_r):
        mem = np.nonzero(label == a)[0]
        for b in range(n_r):
            if a != b:
                w[a, b] = (dist[mem, b] - dist[mem, a]).min()
    for k in range(n_r):
        w = np.minimum(w, w[:, k:k + 1] + w[k:k + 1, :])
    assert np.diag(w).min() >= -1e-9


def test_solver_rejects_bad_shapes():
    with pytest.raises(binding.CmoeError):
        binding.cmoe_balanced_assignment(np.zeros((5, 2)), 2)


def _check_build(cfg, weights, calib, kmeans_iters=1, dist_mode=0):
    h = binding.cmoe_build(binding.make_config(cfg, kmeans_iters, dist_mode), *weights, calib)
    e = binding.cmoe_export_partition(h, cfg.d_ff, cfg.n_routed)
    binding.cmoe_destroy(h)
    wg, wu, _ = weights
    p = O.build(wg, wu, calib, cfg.n_experts, cfg.n_shared, cfg.k_act, kmeans_iters=kmeans_iters,
                squared_dist=bool(dist_mode))
    m, n_s, n_r = cfg.m, cfg.n_shared, cfg.n_routed
    order = e["neuron_order"]
    # rates, shared experts: unique, must match exactly (ties to the lowest index on both sides)
    assert np.array_equal(e["mu"], p["mu"].astype(np.float32))
    assert np.array_equal(order[: n_s * m], p["neuron_order"][: n_s * m])
    # partition
    assert sorted(order.tolist()) == list(range(cfg.d_ff))
    # the cost of the first assignment is unique even where the assignment is not; later rounds start from
    # centroids that depend on which optimal assignment was taken (see test_build_rounds_chain)
    if kmeans_iters == 1:
        assert e["cost"] == pytest.approx(p["cost"], rel=1e-9)
    # representative neurons: valid under the library's own final clusters (Eq. 7)
    a = O.atopk_matrix(O.hidden_states(calib, wg, wu), cfg.k_act)
    for j in range(n_r):
        members = np.sort(order[(n_s + j) * m:(n_s + j + 1) * m])
        feat = a[:, members].T.astype(float)
        cent = feat.mean(axis=0)
        dd = np.sqrt(((feat - cent[None, :]) ** 2).sum(axis=1))
        rep = e["rep_neuron"][j]
        assert rep in members
        assert dd[list(members).index(rep)] <= dd.min() + 1e-9
    return e, p


def test_build_cfg0_matches_oracle():
    cfg = synth.CONFIGS[0]
    weights = synth.make_weights(cfg)
    calib = synth.make_token_source(cfg).calibration()
    _check_build(cfg, weights, calib)


def test_build_first_assignment_is_optimal_for_the_oracles_distances():
    """The library's clusters, priced with the oracle's distance matrix, reach the oracle's optimum."""
    cfg = synth.CONFIGS[0]
    wg, wu, wd = synth.make_weights(cfg)
    calib = synth.make_token_source(cfg).calibration()
    h = binding.cmoe_build(binding.make_config(cfg), wg, wu, wd, calib)
    e = binding.cmoe_export_partition(h, cfg.d_ff, cfg.n_routed)
    binding.cmoe_destroy(h)
    p = O.build(wg, wu, calib, cfg.n_experts, cfg.n_shared, cfg.k_act)
    a = O.atopk_matrix(O.hidden_states(calib, wg, wu), cfg.k_act)
    remaining = p["remaining"]
    dist = O.distance_matrix(a[:, remaining].T.astype(float), O.init_centroids(a, p["mu"], remaining, cfg.n_routed))
    pos = {int(nid): k for k, nid in enumerate(remaining)}
    label = np.empty(len(remaining), dtype=np.int64)
    for j in range(cfg.n_routed):
        for nid in e["neuron_order"][(cfg.n_shared + j) * cfg.m:(cfg.n_shared + j + 1) * cfg.m]:
            label[pos[int(nid)]] = j
    assert O.assignment_cost(dist, label) == pytest.approx(p["cost"], rel=1e-9)


@pytest.mark.parametrize("dtype,iters,dist_mode", [("bf16", 1, 0), ("bf16", 3, 1), ("fp32", 2, 0)])
def test_build_reduced_configs(dtype, iters, dist_mode):
    cfg = synth.scaled(synth.CONFIGS[1], d_model=128, d_ff=768, n_experts=12, n_shared=2, top_k=3, dtype=dtype,
                       n_centres=8, n_calib=100, k_act=20)
    weights = synth.make_weights(cfg)
    calib = synth.make_token_source(cfg).calibration()
    e, _ = _check_build(cfg, weights, calib, kmeans_iters=iters, dist_mode=dist_mode)
    assert e["cost"] > 1.0                              # the routed neurons' feature vectors are not all zero


@pytest.mark.parametrize("dtype,dist_mode", [("bf16", 1), ("fp32", 0)])
def test_build_rounds_chain(dtype, dist_mode):
    """Several K-means rounds (App. A.3: assignment, cluster update, repeated).  Optimal assignments are not
    unique, so the library's round k cannot be compared with the oracle's round k label by label.  What is
    unique: a build with k rounds starts from the result of the build with k - 1 rounds (the library is
    deterministic), so the labels of k - 1 rounds give the centroids of round k (means of their members,
    computed here by the oracle's update), the oracle's distance matrix against those centroids prices the
    labels of k rounds, and that price must equal both the cost the library reports and the optimum of that
    matrix (the oracle's replicated-column assignment).  A library that skipped the update, updated from
    other labels, or stopped early without reason fails the cost equality."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=128, d_ff=768, n_experts=12, n_shared=2, top_k=3, dtype=dtype,
                       n_centres=8, n_calib=100, k_act=20)
    wg, wu, wd = synth.make_weights(cfg)
    calib = synth.make_token_source(cfg).calibration()
    m, n_s, n_r = cfg.m, cfg.n_shared, cfg.n_routed
    a = O.atopk_matrix(O.hidden_states(calib, wg, wu), cfg.k_act)
    mu = O.activation_rates(a)
    shared = O.select_shared(mu, n_s * m)
    remaining = np.setdiff1d(np.arange(cfg.d_ff), shared)
    feat = a[:, remaining].T.astype(float)
    pos = {int(nid): k for k, nid in enumerate(remaining)}
    cent = O.init_centroids(a, mu, remaining, n_r)
    prev_label, moved, stopped = None, 0, False
    for k in range(1, 8):
        h = binding.cmoe_build(binding.make_config(cfg, k, dist_mode), wg, wu, wd, calib)
        e = binding.cmoe_export_partition(h, cfg.d_ff, n_r)
        binding.cmoe_destroy(h)
        assert np.array_equal(np.sort(e["neuron_order"][: n_s * m]), np.sort(shared))
        label = np.empty(len(remaining), dtype=np.int64)
        for j in range(n_r):
            for nid in e["neuron_order"][(n_s + j) * m:(n_s + j + 1) * m]:
                label[pos[int(nid)]] = j
        dist = O.distance_matrix(feat, cent, squared=bool(dist_mode))
        assert O.assignment_cost(dist, label) == pytest.approx(e["cost"], rel=1e-9)
        assert e["cost"] == pytest.approx(O.assignment_cost(dist, O.balanced_assignment(dist, m)), rel=1e-9)
        if prev_label is not None and np.array_equal(prev_label, label):
            stopped = True                          # the library stops when a round moves nothing
            break
        moved += prev_label is not None
        prev_label = label
        cent = O.update_centroids(feat, label, cent)
    assert moved >= 1 and stopped                   # later rounds did change the assignment, then it settled


def test_build_argument_errors():
    cfg = synth.scaled(synth.CONFIGS[0], d_model=16, d_ff=32, n_experts=4, n_shared=1, top_k=1)
    w = synth.make_weights(cfg)
    x = synth.make_token_source(cfg).calibration(n=20)
    c = binding.make_config(cfg)
    c.k_act = 33
    with pytest.raises(binding.CmoeError, match="k_act"):
        binding.cmoe_build(c, *w, x)
    c = binding.make_config(cfg)
    c.kmeans_iters = 0
    with pytest.raises(binding.CmoeError, match="kmeans_iters"):
        binding.cmoe_build(c, *w, x)
    with pytest.raises(binding.CmoeError, match="empty"):
        binding.cmoe_build(binding.make_config(cfg), *w, np.zeros((0, 16), dtype=np.float32))


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_profile_activations_on_the_host_matches_the_oracle(dtype):
    """App. A.2 steps 1-2 on their own: the per-token index sets are the rows of the oracle's ATopK matrix."""
    cfg = synth.scaled(synth.CONFIGS[0], d_model=64, d_ff=384, n_experts=8, n_shared=1, top_k=2, dtype=dtype,
                       n_calib=96, k_act=7)
    wg, wu, _ = synth.make_weights(cfg)
    x = synth.make_token_source(cfg).calibration()
    active = binding.cmoe_profile_activations(binding.make_config(cfg), wg, wu, x, on_gpu=False)
    a = O.atopk_matrix(O.hidden_states(x, wg, wu), cfg.k_act)
    assert active.shape == (x.shape[0], cfg.k_act)
    for t in range(x.shape[0]):
        assert set(active[t].tolist()) == set(np.nonzero(a[t])[0].tolist())


def _hier_inputs(dtype="bf16", n_outer=4, n_calib=400):
    cfg = synth.scaled(synth.CONFIGS[4], d_model=64, d_ff=384, n_experts=8, n_shared=2, top_k=2, dtype=dtype,
                       n_centres=8, n_calib=n_calib, k_act=12, n_outer=n_outer, outer_top_k=2)
    w_router, offsets = synth.make_outer_router(cfg)
    ws = [synth.make_outer_expert_weights(cfg, e) for e in range(n_outer)]
    calib = synth.make_token_source(cfg).calibration()
    return cfg, w_router, offsets, ws, calib


@pytest.mark.parametrize("dtype,min_tokens", [("bf16", 64), ("fp32", 150)])
def test_hier_build_matches_the_oracle_per_outer_expert(dtype, min_tokens):
    """cmoe_hier_build (Sec. 4.4): the library routes the calibration tokens through the outer router and
    restructures each outer expert on the tokens it receives.  Against the oracle's hier_build: the same
    number of tokens per expert (Zipf-skewed offsets; with min_tokens = 150 the least loaded experts fall back
    to the whole set), and per expert what is unique in a construction: rates, the shared set, the cost of
    the optimal assignment, representatives that are valid in the library's own clusters."""
    cfg, w_router, offsets, ws, calib = _hier_inputs(dtype)
    h = binding.cmoe_hier_build(binding.make_config(cfg), cfg.outer_top_k, [w[0] for w in ws], [w[1] for w in ws],
                                [w[2] for w in ws], w_router, offsets, calib, min_tokens=min_tokens)
    ref = O.hier_build([(w[0], w[1]) for w in ws], w_router, offsets, cfg.outer_top_k, calib, cfg.n_experts,
                       cfg.n_shared, cfg.k_act, min_tokens=min_tokens)
    assert sum(ref["routed"]) == calib.shape[0] * cfg.outer_top_k
    fell_back = 0
    m, n_s, n_r = cfg.m, cfg.n_shared, cfg.n_routed
    for e in range(cfg.n_outer):
        layer, routed, used = binding.cmoe_hier_expert(h, e)
        assert routed == ref["routed"][e] and used == len(ref["tokens"][e])
        fell_back += used != routed
        part = binding.cmoe_export_partition(layer, cfg.d_ff, n_r)
        p = ref["parts"][e]
        assert np.array_equal(part["mu"], p["mu"].astype(np.float32))
        assert np.array_equal(part["neuron_order"][: n_s * m], p["neuron_order"][: n_s * m])
        assert sorted(part["neuron_order"].tolist()) == list(range(cfg.d_ff))
        assert part["cost"] == pytest.approx(p["cost"], rel=1e-9)
        a = O.atopk_matrix(O.hidden_states(calib[ref["tokens"][e]], ws[e][0], ws[e][1]), cfg.k_act)
        for j in range(n_r):
            members = np.sort(part["neuron_order"][(n_s + j) * m:(n_s + j + 1) * m])
            feat = a[:, members].T.astype(float)
            dd = np.sqrt(((feat - feat.mean(axis=0)[None, :]) ** 2).sum(axis=1))
            rep = part["rep_neuron"][j]
            assert rep in members and dd[list(members).index(rep)] <= dd.min() + 1e-9
    assert (fell_back > 0) == (min_tokens == 150)
    binding.cmoe_hier_destroy(h)


def test_hier_build_argument_errors():
    cfg, w_router, offsets, ws, calib = _hier_inputs(n_outer=2, n_calib=80)
    args = ([w[0] for w in ws], [w[1] for w in ws], [w[2] for w in ws], w_router, offsets)
    with pytest.raises(binding.CmoeError, match="outer_top_k"):
        binding.cmoe_hier_build(binding.make_config(cfg), 3, *args, calib)
    bad = calib.copy()
    bad[5, 0] = np.nan
    with pytest.raises(binding.CmoeError, match="token 5"):
        binding.cmoe_hier_build(binding.make_config(cfg), 2, *args, bad)
    c = binding.make_config(cfg)
    c.k_act = cfg.d_ff + 1
    with pytest.raises(binding.CmoeError, match="k_act"):
        binding.cmoe_hier_build(c, 2, *args, calib)
    with pytest.raises(binding.CmoeError):
        binding.cmoe_hier_expert(None, 0)
