"""GPU parity of the hierarchical case (Sec. 4.4, Eq. 10): an MoE layer whose experts were each
restructured into shared + routed sub-experts, against the CPU oracle."""
import numpy as np
import pytest

from oracle import cmoe_oracle as O
from paper_2502_04416_amd import synth
from parity_utils import GAP_EPS, TOL, tail_tokens, tokenwise_rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2502_04416_amd import binding as b
    b.load()
    return b


def _make(binding, cfg, gate=False, tie_reps=False, score_mode=0):
    """A hierarchy over seeded outer experts with arbitrary partitions.  gate: every sub-layer gets its own
    seeded (u, b) of Eq. 9.  tie_reps: sub-experts 1 and 4 of every outer expert share a representative neuron."""
    w_router, offsets = synth.make_outer_router(cfg)
    experts, layers = [], []
    for e in range(cfg.n_outer):
        wg, wu, wd = synth.make_outer_expert_weights(cfg, e)
        part = synth.trivial_partition(cfg, seed=e)
        reps = part["rep_neuron"].copy()
        if tie_reps:
            reps[4] = reps[1]
        ex = {"w_gate": wg, "w_up": wu, "w_down": wd, "neuron_order": part["neuron_order"], "rep_neuron": reps}
        layer = binding.Layer.from_partition(cfg, wg, wu, wd, part["neuron_order"], reps, upload=False, score_mode=score_mode)
        if gate:
            u, b = synth.make_gate_params(cfg, seed=7300 + e)
            if tie_reps:
                b[4] = b[1]
            layer.set_gate_params(u, b)
            ex["u"], ex["b"] = u, b
        experts.append(ex)
        layers.append(layer)
    hier = binding.Hierarchy(layers, cfg.outer_top_k, w_router, offsets)
    return hier, experts, w_router, offsets


def _check(cfg, experts, w_router, offsets, x, out, dense_y, sample, exact_ties_strict=False, abs_score=False):
    T = x.shape[0]
    ok, okw, ogap = O.outer_route(x, w_router, offsets, cfg.outer_top_k)
    strict = (ogap >= GAP_EPS) | ((ogap == 0.0) if exact_ties_strict else False)
    assert np.array_equal(out["outer"][strict], ok[strict]), "outer expert indices differ"
    # sub-expert routing of every token under the GPU's outer choice
    n_r = cfg.n_routed
    sub_excused = exact = 0
    for e in range(cfg.n_outer):
        rows, slot = np.nonzero(out["outer"] == e)
        if rows.size == 0:
            continue
        s = O.router_scores(x[rows], experts[e]["w_gate"], experts[e]["w_up"], experts[e]["rep_neuron"])
        if abs_score:
            s = np.abs(s)
        if experts[e].get("u") is not None or experts[e].get("b") is not None:      # key of Eq. 9
            s = O.softmax_rows(s) + np.asarray(experts[e]["b"], dtype=np.float64)[None, :]
        sel, gap = O.select_top_k(s, cfg.top_k)
        good = gap >= GAP_EPS
        if exact_ties_strict:
            good |= gap == 0.0
            exact += int((gap == 0.0).sum())
        got = out["sub"][rows, slot]
        assert np.array_equal(got[good], sel[good]), "sub-expert indices differ in outer expert %d" % e
        sub_excused += int((~good).sum())
        for r in np.nonzero(~good)[0]:
            kth = s[r, sel[r, -1]]
            assert len(set(got[r].tolist())) == cfg.top_k and (s[r, got[r]] >= kth - GAP_EPS).all()
        assert got.min() >= 0 and got.max() < n_r
    idx = np.asarray(sample)
    ref = O.hier_forward(x[idx], w_router, offsets, cfg.outer_top_k, experts, cfg.n_experts, cfg.n_shared, cfg.top_k,
                         outer_sel_override=out["outer"][idx], sub_sel_override=out["sub"][idx], abs_score=abs_score)
    err = tokenwise_rel_err(out["y"][idx], ref["y"])
    assert err.max() <= TOL[cfg.dtype], "hier: max per-token relative error %g" % err.max()
    dref = O.moe_layer_dense_experts(x[idx[:16]], w_router, offsets, cfg.outer_top_k, experts)
    # the dense form routes with the GPU's own outer choice; compare only tokens whose outer choice is strict
    keep = strict[idx[:16]]
    derr = tokenwise_rel_err(dense_y[idx[:16]][keep], dref[keep])
    assert derr.max() <= TOL[cfg.dtype], "hier dense: max per-token relative error %g" % derr.max()
    load = np.bincount(out["outer"].ravel(), minlength=cfg.n_outer)
    return {"outer_near_ties": int((~strict).sum()), "sub_near_ties": sub_excused, "sub_exact_ties": exact,
            "checked_tokens": int(len(idx)), "max_rel_err": float(err.max()),
            "dense_rel_err": float(derr.max()), "outer_load": load.tolist()}


def test_hier_small(binding):
    cfg = synth.scaled(synth.CONFIGS[4], d_model=512, d_ff=1408, n_experts=8, n_shared=2, top_k=2, n_outer=4,
                       outer_top_k=2, n_centres=16)
    hier, experts, w_router, offsets = _make(binding, cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=500)
    out = hier.forward(x)
    rep = _check(cfg, experts, w_router, offsets, x, out, hier.dense_forward(x), np.arange(500))
    print("\n[parity] hier small: %s" % rep, flush=True)
    out2 = hier.forward(x)
    assert np.array_equal(out["y"], out2["y"])
    # every sub-expert active: the hierarchy reproduces the un-restructured layer (Eq. 10 + Eq. 5)
    hier.close()


@pytest.mark.parametrize("T", [1, 7, 20, 32, 33, 64, 65])
def test_hier_decode_batches(binding, T):
    """Small batches: the weight-streaming kernels up to 16 tokens, the one-tile routing front end up to 64,
    the fused down + combine kernel up to 32; 65 tokens is the first size on the general path."""
    cfg = synth.scaled(synth.CONFIGS[4], d_model=512, d_ff=1408, n_experts=8, n_shared=2, top_k=2, n_outer=4,
                       outer_top_k=2, n_centres=16)
    hier, experts, w_router, offsets = _make(binding, cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    for rep_i in range(2):                      # twice: nothing may depend on what the last call left behind
        out = hier.forward(x)
        rep = _check(cfg, experts, w_router, offsets, x, out, hier.dense_forward(x), np.arange(T))
    print("\n[parity] hier decode T=%d: %s" % (T, rep), flush=True)
    hier.close()


@pytest.mark.parametrize("T", [1, 9, 40, 300])
def test_hier_gate_params_inside_the_hierarchy(binding, T):
    """Eq. 9 inside Eq. 10: every restructured outer expert has its own learnable scale u and load-balance
    bias b.  The sub-expert selection key is Softmax(s) + b, the combine weight w_e * (1 + Softmax(s) * u).
    Sizes: the one-token path, the team selection of the one-tile front end, and the tile router."""
    cfg = synth.scaled(synth.CONFIGS[4], d_model=512, d_ff=1408, n_experts=8, n_shared=2, top_k=2, n_outer=4,
                       outer_top_k=2, n_centres=16)
    hier, experts, w_router, offsets = _make(binding, cfg, gate=True)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    out = hier.forward(x)
    rep = _check(cfg, experts, w_router, offsets, x, out, hier.dense_forward(x), np.arange(T))
    print("\n[parity] hier gate T=%d: %s" % (T, rep), flush=True)
    # the gate does change the result: the same hierarchy without it differs
    plain, *_ = _make(binding, cfg)
    if T >= 9:
        assert not np.array_equal(plain.forward(x)["y"], out["y"])
    plain.close()
    hier.close()


@pytest.mark.parametrize("T", [1, 20, 300])
@pytest.mark.parametrize("gate", [False, True])
def test_hier_exact_ties_go_to_the_lower_id(binding, T, gate):
    """Sub-experts 1 and 4 of every outer expert share a representative neuron (equal scores, bit for bit) and
    outer experts 1 and 2 share a router column and offset (equal logits): wherever such a pair straddles a
    selection boundary the lower id has to win, at both levels."""
    cfg = synth.scaled(synth.CONFIGS[4], d_model=512, d_ff=1408, n_experts=8, n_shared=2, top_k=2, n_outer=4,
                       outer_top_k=2, n_centres=16)
    w_router, offsets = synth.make_outer_router(cfg)
    w_router = w_router.copy()
    offsets = offsets.copy()
    w_router[:, 2] = w_router[:, 1]
    offsets[2] = offsets[1]
    hier, experts, _, _ = _make(binding, cfg, gate=gate, tie_reps=True)
    hier.close()
    # rebuild with the tied outer router (the helper draws its own)
    layers = []
    for e, ex in enumerate(experts):
        layer = binding.Layer.from_partition(cfg, ex["w_gate"], ex["w_up"], ex["w_down"], ex["neuron_order"], ex["rep_neuron"],
                                             upload=False)
        if gate:
            layer.set_gate_params(ex["u"], ex["b"])
        layers.append(layer)
    hier = binding.Hierarchy(layers, cfg.outer_top_k, w_router, offsets)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    out = hier.forward(x)
    rep = _check(cfg, experts, w_router, offsets, x, out, hier.dense_forward(x), np.arange(T), exact_ties_strict=True)
    print("\n[parity] hier exact ties T=%d gate=%s: %s" % (T, gate, rep), flush=True)
    has1, has2 = (out["outer"] == 1).any(axis=1), (out["outer"] == 2).any(axis=1)
    assert not (has2 & ~has1).any()
    if T >= 300:
        assert (has1 & ~has2).any() or (has1 & has2).any()
        assert rep["sub_exact_ties"] > 0
    hier.close()


def test_hier_abs_score_mode(binding):
    cfg = synth.scaled(synth.CONFIGS[4], d_model=512, d_ff=1408, n_experts=8, n_shared=2, top_k=2, n_outer=4,
                       outer_top_k=2, n_centres=16)
    hier, experts, w_router, offsets = _make(binding, cfg, score_mode=1)
    x = synth.make_token_source(cfg).eval_batch(0, n=200)
    out = hier.forward(x)
    rep = _check(cfg, experts, w_router, offsets, x, out, hier.dense_forward(x), np.arange(200), abs_score=True)
    print("\n[parity] hier |s|: %s" % rep, flush=True)
    hier.close()


@pytest.mark.parametrize("on_gpu", [False, True])
def test_hier_build_then_forward(binding, on_gpu):
    """cmoe_hier_build end to end (Sec. 4.4): the library routes the calibration tokens, restructures every
    outer expert on its own tokens (profiling on the host or on the device) and the forward on the result
    matches the oracle evaluated on the exported partitions."""
    cfg = synth.scaled(synth.CONFIGS[4], d_model=512, d_ff=1408, n_experts=8, n_shared=2, top_k=2, n_outer=4,
                       outer_top_k=2, n_centres=16, n_calib=600, k_act=24)
    w_router, offsets = synth.make_outer_router(cfg)
    ws = [synth.make_outer_expert_weights(cfg, e) for e in range(cfg.n_outer)]
    src = synth.make_token_source(cfg)
    calib = src.calibration()
    hier = binding.Hierarchy.build(cfg, cfg.outer_top_k, [w[0] for w in ws], [w[1] for w in ws], [w[2] for w in ws],
                                   w_router, offsets, calib, on_gpu=on_gpu)
    ref = O.hier_build([(w[0], w[1]) for w in ws], w_router, offsets, cfg.outer_top_k, calib, cfg.n_experts, cfg.n_shared,
                       cfg.k_act)
    experts = []
    for e in range(cfg.n_outer):
        part = hier.expert_partition(e)
        assert part["calib_routed"] == ref["routed"][e] and part["calib_used"] == len(ref["tokens"][e])
        assert np.array_equal(part["mu"], ref["parts"][e]["mu"].astype(np.float32))
        assert part["cost"] == pytest.approx(ref["parts"][e]["cost"], rel=1e-9)
        experts.append({"w_gate": ws[e][0], "w_up": ws[e][1], "w_down": ws[e][2], "neuron_order": part["neuron_order"],
                        "rep_neuron": part["rep_neuron"]})
    x = src.eval_batch(0, n=400)
    out = hier.forward(x)
    rep = _check(cfg, experts, w_router, offsets, x, out, hier.dense_forward(x), np.arange(400))
    print("\n[parity] hier_build on_gpu=%s: %s routed %s" % (on_gpu, rep, ref["routed"]), flush=True)
    hier.close()


def _random_hier_shapes(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        d = int(rng.choice([256, 512, 768]))
        n_outer = int(rng.choice([2, 3, 4, 8]))
        otk = int(rng.integers(1, min(n_outer, 3) + 1))
        N = int(rng.choice([4, 8]))
        N_s = int(rng.integers(0, 3))
        N_k = int(rng.integers(1, min(N - N_s, 3) + 1))
        m = int(rng.choice([64, 100, 176]))
        T = int(rng.choice([1, 7, 33, 100, 300]))
        out.append((i, d, n_outer, otk, N, N_s, N_k, m, T))
    return out


@pytest.mark.parametrize("i,d,n_outer,otk,N,N_s,N_k,m,T", _random_hier_shapes(10, 20250212))
def test_hier_random_shapes(binding, i, d, n_outer, otk, N, N_s, N_k, m, T):
    """Seeded hierarchy shapes inside the documented limits, including a single outer expert per token and
    sub-layers without a shared expert."""
    cfg = synth.scaled(synth.CONFIGS[4], d_model=d, d_ff=N * m, n_experts=N, n_shared=N_s, top_k=N_k, n_outer=n_outer,
                       outer_top_k=otk, n_centres=8)
    hier, experts, w_router, offsets = _make(binding, cfg)
    x = synth.make_token_source(cfg).eval_batch(i, n=T)
    out = hier.forward(x)
    rep = _check(cfg, experts, w_router, offsets, x, out, hier.dense_forward(x), np.arange(T))
    print("\n[parity] hier random %d: d=%d outer %d/%d sub S%dA%dE%d m=%d T=%d: %s" % (i, d, otk, n_outer, N_s, N_k, N, m, T, rep), flush=True)
    assert np.array_equal(out["y"], hier.forward(x)["y"])
    hier.close()


def test_hier_all_subexperts_active_equals_dense_layer(binding):
    cfg = synth.scaled(synth.CONFIGS[4], d_model=256, d_ff=1024, n_experts=8, n_shared=2, top_k=6, n_outer=3,
                       outer_top_k=2, n_centres=8)
    hier, experts, w_router, offsets = _make(binding, cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=130)
    out = hier.forward(x)
    dense = hier.dense_forward(x)
    ref = O.moe_layer_dense_experts(x, w_router, offsets, cfg.outer_top_k, experts)
    assert tokenwise_rel_err(out["y"], ref).max() <= TOL["bf16"]
    assert tokenwise_rel_err(dense, ref).max() <= TOL["bf16"]
    hier.close()


def test_hier_cfg4_full(binding):
    """Mixtral-8x7B-shaped layer: 8 outer experts of 14336 neurons, each split into 8 sub-experts of 1792
    (2 shared + top-2 of 6), 4096 tokens with Zipf-skewed outer routing."""
    cfg = synth.CONFIGS[4]
    hier, experts, w_router, offsets = _make(binding, cfg)
    x = synth.make_token_source(cfg).eval_batch(0)
    out = hier.forward(x)
    rng = np.random.Generator(np.random.PCG64(404))
    # outputs of 512 random tokens plus the last row tile of every one of the 64 groups' segments
    # (group id = outer expert * 8 + {0: its shared sub-experts, 1 + j: routed sub-expert j})
    gid = np.concatenate([out["outer"][:, :, None] * 8, out["outer"][:, :, None] * 8 + 1 + out["sub"]], axis=2)
    sample = tail_tokens(gid.reshape(x.shape[0], -1), 64, rows=32, extra=rng.choice(x.shape[0], size=512, replace=False))
    rep = _check(cfg, experts, w_router, offsets, x, out, hier.dense_forward(x), sample)
    print("\n[parity] hier cfg4 T=%d: %s" % (x.shape[0], rep), flush=True)
    hier.close()


def test_hier_cfg4_full_on_the_hierarchy_the_library_builds(binding):
    """The configuration the bench times: the Mixtral-8x7B-shaped layer restructured by cmoe_hier_build (profiling
    on the device, every outer expert on the calibration tokens routed to it), 4096 tokens.  The analytically
    built routers give skewed, ragged sub-expert segments, unlike an arbitrary partition.  Routing of every
    token, outputs of 512 random tokens plus the last row tile of every group's segment."""
    cfg = synth.CONFIGS[4]
    w_router, offsets = synth.make_outer_router(cfg)
    ws = [synth.make_outer_expert_weights(cfg, e) for e in range(cfg.n_outer)]
    src = synth.make_token_source(cfg)
    hier = binding.Hierarchy.build(cfg, cfg.outer_top_k, [w[0] for w in ws], [w[1] for w in ws], [w[2] for w in ws],
                                   w_router, offsets, src.calibration(), on_gpu=True)
    experts = []
    for e in range(cfg.n_outer):
        part = hier.expert_partition(e)
        experts.append({"w_gate": ws[e][0], "w_up": ws[e][1], "w_down": ws[e][2], "neuron_order": part["neuron_order"],
                        "rep_neuron": part["rep_neuron"]})
    x = src.eval_batch(0)
    out = hier.forward(x)
    rng = np.random.Generator(np.random.PCG64(405))
    gid = np.concatenate([out["outer"][:, :, None] * 8, out["outer"][:, :, None] * 8 + 1 + out["sub"]], axis=2)
    sample = tail_tokens(gid.reshape(x.shape[0], -1), 64, rows=32, extra=rng.choice(x.shape[0], size=512, replace=False))
    rep = _check(cfg, experts, w_router, offsets, x, out, hier.dense_forward(x), sample)
    sub_load = np.bincount((out["outer"][:, :, None] * cfg.n_routed + out["sub"]).ravel(), minlength=cfg.n_outer * cfg.n_routed)
    print("\n[parity] hier cfg4 (library build) T=%d: %s sub-expert rows min/max %d/%d" % (x.shape[0], rep, sub_load.min(), sub_load.max()),
          flush=True)
    hier.close()

