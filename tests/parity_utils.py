"""Shared checks for the GPU parity tests: compare one forward of the HIP library with the CPU oracle.

Rules (from the task's parity bar):
  * expert indices bit-exact, except tokens whose oracle top-k score gap is below 1e-5 (absolute, on the
    selection key); those tokens are counted and reported, and their GPU choice must still be a valid
    one (every chosen key within 1e-5 of the oracle's k-th key);
  * outputs: per-token norm-wise error  max|y - y_ref| / max|y_ref|  <= tol  (1e-2 bf16, 1e-5 fp32).
    For an excused token the oracle is re-evaluated with the GPU's (equally valid) selection.
"""
import numpy as np

from oracle import cmoe_oracle as O

GAP_EPS = 1e-5
TOL = {"bf16": 1e-2, "fp32": 1e-5}


def tokenwise_rel_err(y, y_ref):
    den = np.abs(y_ref).max(axis=1)
    den = np.where(den > 0, den, 1.0)
    return np.abs(y - y_ref).max(axis=1) / den


def tail_tokens(topk, n_groups, rows=128, extra=None):
    """Tokens that sit in the last `rows` rows of every expert's segment (segments are token-ascending, so
    these are the last tokens that selected the expert) and of the batch itself (the always-on group), i.e.
    the ragged last row tile of every group, merged with `extra`."""
    topk = np.asarray(topk)
    T = topk.shape[0]
    keep = set(range(max(0, T - rows), T))
    flat = topk.reshape(T, -1)
    for g in range(n_groups):
        toks = np.nonzero((flat == g).any(axis=1))[0]
        keep.update(toks[-rows:].tolist())
    if extra is not None:
        keep.update(int(t) for t in extra)
    return np.array(sorted(keep), dtype=np.int64)


def fragile_sparsity_tokens(cfg, weights, part, x, sel, tau, weight_informed, rel=5e-6):
    """Tokens for which the keep/drop decision of neuron-level sparsity is not robust: some neuron of a selected
    routed expert has |h| so close to a bfloat16 rounding boundary next to the threshold that fp32 and fp64
    evaluation may round it to different sides.  (Like near-ties of the router, these are counted and excused.)"""
    wg, wu, wd = weights
    order = np.asarray(part["neuron_order"], dtype=np.int64)
    m, n_s = cfg.m, cfg.n_shared
    bad = np.zeros(x.shape[0], dtype=bool)
    for j in range(cfg.n_routed):
        rows = np.nonzero((sel == j).any(axis=1))[0]
        if rows.size == 0:
            continue
        idx = order[(n_s + j) * m:(n_s + j + 1) * m]
        h = O.hidden_states(x[rows], wg[:, idx], wu[:, idx])
        lo = O.neuron_keep_mask(h * (1 - rel), wd[idx], tau, weight_informed, True)
        hi = O.neuron_keep_mask(h * (1 + rel), wd[idx], tau, weight_informed, True)
        bad[rows] |= (lo != hi).any(axis=1)
    return bad


def check_flat(cfg, weights, part, x, out, u=None, b=None, sample=None, score_tol=None, abs_score=False,
               exact_ties_strict=False, neuron=None):
    """out: dict from binding.Layer.forward.  sample: token indices whose outputs are compared
    (None = all).  exact_ties_strict: a token whose k-th and (k+1)-th keys are *equal* (two experts with
    the same representative neuron) is not excused: the lower expert id has to win.  neuron: (tau,
    weight_informed) of the neuron-level sparsity inside the routed experts; the oracle decides on the
    bfloat16 value of h as the kernels do, and tokens whose decision is not robust to fp32 rounding are
    excused and counted.  Returns a small report dict."""
    wg, wu, wd = weights
    T = x.shape[0]
    order, reps = part["neuron_order"], part["rep_neuron"]
    # routing of every token (cheap: only the router columns)
    s = O.router_scores(x, wg, wu, reps)
    skey = np.abs(s) if abs_score else s
    if u is None and b is None:
        key = skey
    else:
        key = O.softmax_rows(skey) + (0.0 if b is None else np.asarray(b, dtype=np.float64)[None, :])
    sel, gap = O.select_top_k(key, cfg.top_k)
    excused = gap < GAP_EPS
    if exact_ties_strict:
        excused &= gap != 0.0
    strict = ~excused
    assert np.array_equal(out["topk"][strict], sel[strict]), \
        "expert indices differ on %d tokens with gap >= 1e-5" % int((out["topk"][strict] != sel[strict]).any(axis=1).sum())
    # excused tokens: the GPU's choice must be distinct experts whose keys reach the oracle's k-th key - eps
    for t in np.nonzero(excused)[0]:
        g = out["topk"][t]
        assert len(set(g.tolist())) == cfg.top_k and g.min() >= 0 and g.max() < cfg.n_routed
        kth = key[t, sel[t, -1]]
        assert (key[t, g] >= kth - GAP_EPS).all()
    # scores (fp32 on the device)
    if score_tol is None:
        score_tol = 2e-5 if cfg.dtype == "bf16" else 1e-5
    s_err = np.abs(out["scores"] - s).max() if T else 0.0
    assert s_err <= score_tol * max(1.0, np.abs(s).max()), "router score error %g" % s_err
    # counts
    want_counts = np.bincount(out["topk"].ravel(), minlength=cfg.n_routed)
    assert np.array_equal(out["counts"], want_counts), "per-expert counts do not match the returned indices"
    assert out["counts"].sum() == T * cfg.top_k
    # outputs
    idx = np.arange(T) if sample is None else np.asarray(sample)
    kw, fragile = {}, 0
    if neuron is not None:
        kw = {"neuron_tau": float(neuron[0]), "neuron_weight_informed": bool(neuron[1]), "neuron_decide_in_bf16": cfg.dtype == "bf16"}
        bad = fragile_sparsity_tokens(cfg, weights, part, x[idx], out["topk"][idx], float(neuron[0]), bool(neuron[1]))
        fragile = int(bad.sum())
        idx = idx[~bad]
    ref = O.moe_forward(x[idx], wg, wu, wd, order, reps, cfg.n_experts, cfg.n_shared, cfg.top_k, u=u, b=b,
                        abs_score=abs_score, sel_override=out["topk"][idx], **kw)
    err = tokenwise_rel_err(out["y"][idx], ref["y"])
    tol = TOL[cfg.dtype]
    assert err.max() <= tol, "max per-token relative error %g > %g (token %d)" % (err.max(), tol, idx[int(err.argmax())])
    return {"near_ties": int(excused.sum()), "exact_ties": int((gap == 0.0).sum()), "checked_tokens": int(len(idx)),
            "max_rel_err": float(err.max()), "score_err": float(s_err),
            **({"kept": float(ref["kept"]), "fragile_tokens": fragile} if neuron is not None else {}),
            "min_gap": float(gap.min()) if T else np.inf, "union": int((want_counts > 0).sum())}


def check_dense(cfg, weights, x, y, sample=None):
    wg, wu, wd = weights
    idx = np.arange(x.shape[0]) if sample is None else np.asarray(sample)
    ref = O.dense_ffn(x[idx], wg, wu, wd)
    err = tokenwise_rel_err(y[idx], ref)
    assert err.max() <= TOL[cfg.dtype], "dense: max per-token relative error %g" % err.max()
    return float(err.max())
