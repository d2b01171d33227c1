"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.

Small cases are compared element by element on every token; the full-size configurations compare the
routing of every token and the outputs of a random sample of tokens (the oracle evaluates those one
group at a time), plus size-independent properties (counts, determinism)."""
import numpy as np
import pytest

from oracle import cmoe_oracle as O
from paper_2502_04416_amd import synth
from parity_utils import check_dense, check_flat, tail_tokens, tokenwise_rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2502_04416_amd import binding as b
    b.load()
    return b


def _layer(binding, cfg, weights, part, **kw):
    return binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"], **kw)


def _say(name, rep):
    print("\n[parity] %s: %s" % (name, rep), flush=True)


# ---------------------------------------------------------------------------------- config 0 (fp32)

@pytest.fixture(scope="module")
def cfg0():
    cfg = synth.CONFIGS[0]
    weights = synth.make_weights(cfg)
    src = synth.make_token_source(cfg)
    part = O.build(weights[0], weights[1], src.calibration(), cfg.n_experts, cfg.n_shared, cfg.k_act)
    return cfg, weights, src, part


def test_cfg0_fp32_end_to_end(binding, cfg0):
    cfg, weights, src, part = cfg0
    x = src.eval_batch(0)
    layer = _layer(binding, cfg, weights, part)
    out = layer.forward(x)
    rep = check_flat(cfg, weights, part, x, out)
    _say("cfg0 T=64", rep)
    rep_d = check_dense(cfg, weights, x, layer.dense_forward(x))
    _say("cfg0 dense", rep_d)
    # run-to-run determinism: bit-identical outputs
    out2 = layer.forward(x)
    assert np.array_equal(out["y"], out2["y"]) and np.array_equal(out["topk"], out2["topk"])
    layer.close()


@pytest.mark.parametrize("T", [1, 3, 65, 200])
def test_cfg0_ragged_batches(binding, cfg0, T):
    cfg, weights, src, part = cfg0
    x = src.eval_batch(0, n=T)
    layer = _layer(binding, cfg, weights, part)
    _say("cfg0 T=%d" % T, check_flat(cfg, weights, part, x, layer.forward(x)))
    layer.close()


def test_cfg0_gate_params(binding, cfg0):
    """Eq. 9 with non-zero u and b: softmax scores, biased selection, gate-weighted combine."""
    cfg, weights, src, part = cfg0
    x = src.eval_batch(0)
    u, b = synth.make_gate_params(cfg)
    layer = _layer(binding, cfg, weights, part)
    layer.set_gate_params(u, b)
    _say("cfg0 gate", check_flat(cfg, weights, part, x, layer.forward(x), u=u, b=b))
    layer.set_gate_params(None, None)
    _say("cfg0 gate reset", check_flat(cfg, weights, part, x, layer.forward(x)))
    layer.close()


def test_cfg0_all_experts_active_equals_dense(binding, cfg0):
    """N_k = N_r: the MoE output equals the dense FFN (Eq. 5 with no deactivated expert)."""
    cfg, weights, src, part = cfg0
    full = synth.scaled(cfg, top_k=cfg.n_routed)
    x = src.eval_batch(0)
    layer = _layer(binding, full, weights, part)
    out = layer.forward(x)
    dense_ref = O.dense_ffn(x, *weights)
    assert tokenwise_rel_err(out["y"], dense_ref).max() <= 1e-5
    assert tokenwise_rel_err(layer.dense_forward(x), dense_ref).max() <= 1e-5
    assert (out["counts"] == x.shape[0]).all()
    layer.close()


def test_cfg0_abs_score_mode(binding, cfg0):
    cfg, weights, src, part = cfg0
    x = src.eval_batch(0)
    layer = _layer(binding, cfg, weights, part, score_mode=1)
    _say("cfg0 |s|", check_flat(cfg, weights, part, x, layer.forward(x), abs_score=True))
    layer.close()


def test_identical_tokens_all_go_to_one_expert(binding, cfg0):
    """Degenerate routing: every token identical, so one routed expert receives the whole batch and the
    others none."""
    cfg, weights, src, part = cfg0
    x = np.repeat(src.eval_batch(0, n=1), 130, axis=0)
    layer = _layer(binding, cfg, weights, part)
    out = layer.forward(x)
    rep = check_flat(cfg, weights, part, x, out)
    assert rep["union"] == 1 and out["counts"].max() == 130
    layer.close()


def test_no_shared_expert(binding):
    cfg = synth.scaled(synth.CONFIGS[0], n_shared=0, top_k=2)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=77)
    layer = _layer(binding, cfg, weights, part)
    _say("N_s=0", check_flat(cfg, weights, part, x, layer.forward(x)))
    layer.close()


@pytest.mark.parametrize("base,T", [(0, 77), (1, 5), (1, 40), (1, 300)])
def test_one_slot_per_token(binding, base, T):
    """No shared expert and top-1 routing: every token has exactly one slot, but the slots are still a
    permutation of the tokens and carry the gate weight of Eq. 9, so the output has to go through the
    combine step (only the dense baseline may write y from the down contraction)."""
    if base == 0:
        cfg = synth.scaled(synth.CONFIGS[0], n_shared=0, top_k=1)
    else:
        cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_shared=0, top_k=1, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    u, b = synth.make_gate_params(cfg)
    layer = _layer(binding, cfg, weights, part)
    _say("top-1, N_s=0, %s T=%d" % (cfg.dtype, T), check_flat(cfg, weights, part, x, layer.forward(x)))
    layer.set_gate_params(u, b)
    _say("top-1, N_s=0, %s T=%d gate" % (cfg.dtype, T), check_flat(cfg, weights, part, x, layer.forward(x), u=u, b=b))
    layer.close()


def test_empty_batch_and_errors(binding, cfg0):
    import torch
    cfg, weights, src, part = cfg0
    layer = _layer(binding, cfg, weights, part)
    x = torch.zeros((0, cfg.d_model), device="cuda")
    y = torch.zeros((0, cfg.d_model), device="cuda")
    layer.forward_device(x, y)                     # T = 0 is a no-op
    ws = layer._ensure_ws(8)
    x8 = torch.zeros((8, cfg.d_model), device="cuda")
    y8 = torch.zeros((8, cfg.d_model), device="cuda")
    with pytest.raises(binding.CmoeError, match="workspace too small"):
        binding.cmoe_forward(layer.h, x8.data_ptr(), 8, y8.data_ptr(), None, None, None, ws.data_ptr(), 16)
    with pytest.raises(binding.CmoeError, match="null"):
        binding.cmoe_forward(layer.h, None, 8, y8.data_ptr(), None, None, None, ws.data_ptr(), ws.numel())
    layer.close()


# ---------------------------------------------------------------------------------- reduced bf16 cases

SMALL_BF16 = [
    # (name, d, d_ff, N, N_s, N_k, T)   widths that miss the 32-neuron tile, ragged T, several row tiles
    ("m172", 512, 2752, 16, 1, 3, 777),
    ("m44", 1024, 1408, 32, 2, 6, 1500),
    ("m448", 512, 3584, 8, 2, 2, 300),
    ("decode1", 512, 2752, 16, 1, 3, 1),
    ("decode16", 512, 2752, 16, 1, 3, 16),
]


@pytest.mark.parametrize("name,d,d_ff,N,N_s,N_k,T", SMALL_BF16)
def test_small_bf16(binding, name, d, d_ff, N, N_s, N_k, T):
    cfg = synth.scaled(synth.CONFIGS[1], d_model=d, d_ff=d_ff, n_experts=N, n_shared=N_s, top_k=N_k, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    layer = _layer(binding, cfg, weights, part)
    out = layer.forward(x)
    _say("small %s" % name, check_flat(cfg, weights, part, x, out))
    _say("small %s dense" % name, check_dense(cfg, weights, x, layer.dense_forward(x)))
    out2 = layer.forward(x)
    assert np.array_equal(out["y"], out2["y"])
    layer.close()


@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 31, 32, 33, 48, 64, 65])
def test_small_bf16_decode_sizes(binding, T):
    """Every batch size around the decode/tiled switch of the expert kernels (32), the 16-token MFMA tile
    and the one-tile limit of the two-launch routing front end (64); each runs twice and must give
    identical bits."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    u, b = synth.make_gate_params(cfg)
    layer = _layer(binding, cfg, weights, part)
    out1 = layer.forward(x)
    check_flat(cfg, weights, part, x, out1)
    out2 = layer.forward(x)
    assert np.array_equal(out1["y"], out2["y"]) and np.array_equal(out1["topk"], out2["topk"])
    layer.set_gate_params(u, b)
    _say("small decode T=%d gate" % T, check_flat(cfg, weights, part, x, layer.forward(x), u=u, b=b))
    check_dense(cfg, weights, x, layer.dense_forward(x))
    layer.close()


@pytest.mark.parametrize("dtype,T", [("bf16", 300), ("bf16", 9), ("fp32", 70)])
def test_maximum_expert_counts(binding, dtype, T):
    """The limits of the interface: 64 routed experts (one lane per expert in the wave-level top-k) and
    top-16 selection, with a shared expert, on a prefill-sized and a decode-sized batch."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=256, d_ff=65 * 32, n_experts=65, n_shared=1, top_k=16, dtype=dtype,
                       n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    layer = _layer(binding, cfg, weights, part)
    _say("N_r=64 top-16 %s T=%d" % (dtype, T), check_flat(cfg, weights, part, x, layer.forward(x)))
    u, b = synth.make_gate_params(cfg)
    layer.set_gate_params(u, b)
    _say("N_r=64 top-16 gate %s T=%d" % (dtype, T), check_flat(cfg, weights, part, x, layer.forward(x), u=u, b=b))
    layer.close()


def test_limits_are_rejected(binding):
    cfg = synth.scaled(synth.CONFIGS[0], d_model=64, d_ff=66 * 8, n_experts=66, n_shared=1, top_k=2)
    with pytest.raises(binding.CmoeError, match="routed experts"):
        binding.cmoe_build_from_partition(binding.make_config(cfg), *synth.make_weights(cfg),
                                          synth.trivial_partition(cfg)["neuron_order"],
                                          synth.trivial_partition(cfg)["rep_neuron"])
    cfg = synth.scaled(synth.CONFIGS[0], d_model=64, d_ff=20 * 8, n_experts=20, n_shared=1, top_k=17)
    with pytest.raises(binding.CmoeError, match="top_k"):
        binding.cmoe_build_from_partition(binding.make_config(cfg), *synth.make_weights(cfg),
                                          synth.trivial_partition(cfg)["neuron_order"],
                                          synth.trivial_partition(cfg)["rep_neuron"])


def test_small_bf16_gate_params(binding):
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=333)
    u, b = synth.make_gate_params(cfg)
    layer = _layer(binding, cfg, weights, part)
    layer.set_gate_params(u, b)
    _say("small gate", check_flat(cfg, weights, part, x, layer.forward(x), u=u, b=b))
    layer.close()


@pytest.mark.parametrize("T", [40, 130, 500])
def test_k_split_batches(binding, T):
    """Batches of a few hundred tokens on a layer deep enough (d = 2048) that the contractions split K
    over several workgroups and a finishing kernel adds the parts."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=2048, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    layer = _layer(binding, cfg, weights, part)
    out = layer.forward(x)
    _say("k-split T=%d" % T, check_flat(cfg, weights, part, x, out))
    _say("k-split T=%d dense" % T, check_dense(cfg, weights, x, layer.dense_forward(x)))
    assert np.array_equal(out["y"], layer.forward(x)["y"])
    layer.close()


@pytest.mark.parametrize("T", [1, 17, 32, 100])
def test_small_batches_without_decode_kernels(binding, T):
    """A model width the weight-streaming decode kernels are not built for (d = 1536: six K steps per
    slice): batches of a few tokens then run the tiled contraction kernels, whose few tiles split K, so the
    workspace must hold the partial sums at every batch size."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=1536, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    layer = _layer(binding, cfg, weights, part)
    out = layer.forward(x)
    _say("no-decode T=%d" % T, check_flat(cfg, weights, part, x, out))
    _say("no-decode T=%d dense" % T, check_dense(cfg, weights, x, layer.dense_forward(x)))
    assert np.array_equal(out["y"], layer.forward(x)["y"])
    layer.close()


@pytest.fixture
def tuning(binding):
    """Set tuning switches of the library for one test; the defaults come back afterwards."""
    touched = {}

    def set_(name, value, default):
        touched[name] = default
        binding.cmoe_set_tuning(name, value)
    yield set_
    for name, default in touched.items():
        binding.cmoe_set_tuning(name, default)


@pytest.mark.parametrize("which", ["CMOE_GEMM1_CFG", "CMOE_GEMM2_CFG"])
@pytest.mark.parametrize("shape", [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14])
def test_every_tile_shape(binding, tuning, which, shape):
    """Each tile shape of the bf16 contraction kernels forced on the gate/up or the down contraction of a
    layer whose segments end inside tiles: d = 328 (a ragged last K tile at either tile depth), experts of
    100 neurons, 333 tokens."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=328, d_ff=1200, n_experts=12, n_shared=2, top_k=3, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=333)
    layer = _layer(binding, cfg, weights, part)
    tuning("CMOE_SPLITK", 0, 1)                     # (a K split adds the parts in another order)
    tuning("CMOE_WS_DOWN", 0, 0)                    # (the forced shape must be the one that runs)
    ref = layer.forward(x)
    tuning(which, shape, -1)
    out = layer.forward(x)
    _say("%s=%d" % (which, shape), check_flat(cfg, weights, part, x, out))
    _say("%s=%d dense" % (which, shape), check_dense(cfg, weights, x, layer.dense_forward(x)))
    assert np.array_equal(out["topk"], ref["topk"])
    # every shape multiplies K in the same order with the same instruction, so without a K split the tile
    # shape does not change a single bit of the output
    assert np.array_equal(out["y"], ref["y"])
    layer.close()


@pytest.mark.parametrize("m,n_s,T", [(344, 1, 700), (344, 2, 129), (448, 1, 1000), (688, 1, 333), (448, 3, 515), (344, 0, 64)])
def test_weight_stationary_down_contraction(binding, tuning, m, n_s, T):
    """The weight-stationary down kernel forced on reduced layers whose expert widths it has instantiations for
    (344 -> 352, 448, 688 -> 704 neurons), with row chunks that end inside a 64-row piece, empty and tiny
    segments, a shared group of the same or of twice the width (also handled) or three times (left to the
    tiled kernel over the same work list), against the oracle and bit for bit against the tiled kernel."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=12 * m, n_experts=12, n_shared=n_s, top_k=3, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    layer = _layer(binding, cfg, weights, part)
    tuning("CMOE_SPLITK", 0, 1)
    tuning("CMOE_WS_DOWN", 0, 0)
    ref = layer.forward(x)
    tuning("CMOE_WS_DOWN", 2, 0)
    out = layer.forward(x)
    _say("ws down m=%d N_s=%d T=%d" % (m, n_s, T), check_flat(cfg, weights, part, x, out))
    # both kernels multiply K in steps of 16 in ascending order with the same instruction: identical bits
    assert np.array_equal(out["y"], ref["y"])
    assert np.array_equal(out["y"], layer.forward(x)["y"])
    layer.close()


@pytest.mark.parametrize("d,m,n_s", [(512, 64, 1), (1024, 48, 0), (2048, 32, 1)])
def test_one_token_front_end_variants(binding, tuning, d, m, n_s):
    """One token on a flat layer: the routed gate/up units in a launch of their own (0), inside the selection
    launch (1, the default), and with the scoring inside that launch too, every workgroup for itself from the
    router's copy in operand order (2).  Same arithmetic in the same order in all three: identical bits."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=d, d_ff=16 * m, n_experts=16, n_shared=n_s, top_k=3, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=1)
    layer = _layer(binding, cfg, weights, part)
    outs = []
    for v in (1, 0, 2):
        tuning("CMOE_FRONT_ALL", v, 1)
        outs.append(layer.forward(x))
    _say("one-token front end d=%d m=%d N_s=%d" % (d, m, n_s), check_flat(cfg, weights, part, x, outs[0]))
    for o in outs[1:]:
        assert np.array_equal(o["y"], outs[0]["y"])
        assert np.array_equal(o["topk"], outs[0]["topk"])
        assert np.array_equal(o["scores"], outs[0]["scores"])
    layer.close()


@pytest.mark.parametrize("T,n_s", [(2, 1), (7, 1), (16, 1), (5, 0)])
def test_small_batch_front_end_with_every_unit(binding, tuning, T, n_s):
    """Two to sixteen tokens: every routed gate/up unit inside the selection launch (each workgroup selects the
    batch by itself and derives its expert's tokens and rows of H; off by default) against the oracle and bit
    for bit against the default path with its separate gate/up launch."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=1024, d_ff=16 * 48, n_experts=16, n_shared=n_s, top_k=3, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    layer = _layer(binding, cfg, weights, part)
    ref = layer.forward(x)
    tuning("CMOE_FRONT_TILE", 1, 0)
    out = layer.forward(x)
    _say("small-batch front end T=%d N_s=%d" % (T, n_s), check_flat(cfg, weights, part, x, out))
    for k in ("y", "topk", "scores", "counts"):
        assert np.array_equal(out[k], ref[k])
    layer.close()


def _random_shapes(n, seed):
    """Seeded layer shapes and batch sizes inside the documented limits: model widths with and without the
    decode kernels (d / 256 in {2, 4} or not) and with a ragged last K tile (d = 200), expert counts up to 64,
    expert widths that miss the 32-neuron padding, batch sizes on both sides of every kernel switch."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        d = int(rng.choice([200, 256, 320, 512, 768, 1024]))
        N = int(rng.choice([4, 8, 12, 16, 24, 32, 64]))
        m = int(rng.choice([24, 40, 64, 100, 172]))
        N_s = int(rng.integers(0, min(N - 1, 4) + 1))
        N_k = int(rng.integers(1, min(N - N_s, 8) + 1))
        T = int(rng.choice([1, 3, 16, 17, 31, 33, 64, 65, 100, 257, 600]))
        out.append((i, d, N, m, N_s, N_k, T, bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("i,d,N,m,N_s,N_k,T,gate", _random_shapes(16, 20250211))
def test_random_bf16_shapes(binding, i, d, N, m, N_s, N_k, T, gate):
    cfg = synth.scaled(synth.CONFIGS[1], d_model=d, d_ff=N * m, n_experts=N, n_shared=N_s, top_k=N_k, n_centres=16)
    weights = synth.make_weights(cfg, seed=900 + i)
    part = synth.trivial_partition(cfg, seed=i)
    x = synth.make_token_source(cfg).eval_batch(i, n=T)
    layer = _layer(binding, cfg, weights, part)
    u = b = None
    if gate:
        u, b = synth.make_gate_params(cfg, seed=7000 + i)
        layer.set_gate_params(u, b)
    out = layer.forward(x)
    _say("random %d: d=%d N=%d m=%d S%dA%d T=%d gate=%s" % (i, d, N, m, N_s, N_k, T, gate),
         check_flat(cfg, weights, part, x, out, u=u, b=b))
    check_dense(cfg, weights, x, layer.dense_forward(x))
    assert np.array_equal(out["y"], layer.forward(x)["y"])
    layer.close()


@pytest.mark.parametrize("T", [1, 40, 300])
def test_wide_model(binding, T):
    """d = 8192 (twice the width of the study's layers): 128 K tiles per gate/up tile, a router scorer with
    1024 of K per slice, and no weight-streaming decode kernels (their K split covers d up to 4096), so one
    token runs the tile kernels too."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=8192, d_ff=8 * 352, n_experts=8, n_shared=1, top_k=2, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    layer = _layer(binding, cfg, weights, part)
    out = layer.forward(x)
    _say("d=8192 T=%d" % T, check_flat(cfg, weights, part, x, out))
    check_dense(cfg, weights, x, layer.dense_forward(x))
    layer.close()


def _random_fp32_shapes(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        d = int(rng.choice([64, 100, 256, 333]))
        N = int(rng.choice([4, 8, 16]))
        m = int(rng.choice([8, 24, 50]))
        N_s = int(rng.integers(0, 3))
        N_k = int(rng.integers(1, min(N - N_s, 4) + 1))
        T = int(rng.choice([1, 5, 64, 65, 200]))
        out.append((i, d, N, m, N_s, N_k, T, bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("i,d,N,m,N_s,N_k,T,gate", _random_fp32_shapes(8, 20250213))
def test_random_fp32_shapes(binding, i, d, N, m, N_s, N_k, T, gate):
    """The plain-FMA path on seeded shapes, including model widths that are not a multiple of any tile."""
    cfg = synth.scaled(synth.CONFIGS[0], d_model=d, d_ff=N * m, n_experts=N, n_shared=N_s, top_k=N_k, n_centres=8)
    weights = synth.make_weights(cfg, seed=950 + i)
    part = synth.trivial_partition(cfg, seed=i)
    x = synth.make_token_source(cfg).eval_batch(i, n=T)
    layer = _layer(binding, cfg, weights, part)
    u = b = None
    if gate:
        u, b = synth.make_gate_params(cfg, seed=7100 + i)
        layer.set_gate_params(u, b)
    out = layer.forward(x)
    _say("random fp32 %d: d=%d N=%d m=%d S%dA%d T=%d gate=%s" % (i, d, N, m, N_s, N_k, T, gate),
         check_flat(cfg, weights, part, x, out, u=u, b=b))
    check_dense(cfg, weights, x, layer.dense_forward(x))
    layer.close()


@pytest.mark.parametrize("T", [1, 16, 40, 300])
def test_forward_is_capturable_in_a_graph(binding, T):
    """A forward enqueues kernels only (no allocation, no synchronisation, no memset), so it can be recorded
    into a HIP graph; every replay, with eager forwards and synchronisations in between, reproduces the
    eager result bit for bit."""
    import torch
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    layer = _layer(binding, cfg, weights, part)
    src = synth.make_token_source(cfg)
    x = torch.from_numpy(src.eval_batch(0, n=T)).to("cuda", torch.bfloat16)
    x2 = torch.from_numpy(src.eval_batch(1, n=T)).to("cuda", torch.bfloat16)
    y = torch.empty_like(x)
    y2 = torch.empty_like(x)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up outside the capture (first-launch set-up)
        layer.forward_device(x, y, None, None, None)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    ref = y.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer.forward_device(x, y, None, None, None)
    for _ in range(4):
        y.zero_()
        layer.forward_device(x2, y2, None, None, None)   # eager work on the same layer and workspace in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, ref)
    out = layer.forward(x.float().cpu().numpy())
    assert np.array_equal(out["y"], ref.float().cpu().numpy())
    del graph
    layer.close()


def test_bias_update_loop_balances_the_load(binding):
    """Sec. 4.3: forward -> per-expert counts -> cmoe_update_bias, repeated on one batch.  The library's
    biases follow the oracle's step applied to the same counts, the most loaded expert's share falls,
    and the forward with the final biases still matches the oracle."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=777)
    layer = _layer(binding, cfg, weights, part)
    layer.set_gate_params(None, np.zeros(cfg.n_routed, dtype=np.float32))
    ref_b = np.zeros(cfg.n_routed)
    shares = []
    for _ in range(120):
        counts = layer.forward(x)["counts"]
        assert counts.sum() == 777 * cfg.top_k
        shares.append(counts.max() / counts.sum())
        layer.update_bias(counts, 2e-3)
        ref_b = O.bias_update(ref_b, counts, 2e-3)
    u, b = layer.gate_params()
    assert np.abs(b.astype(np.float64) - ref_b).max() < 1e-5
    _say("bias loop", {"share_first": shares[0], "share_last": shares[-1], "uniform": 1.0 / cfg.n_routed})
    assert shares[-1] < 0.65 * shares[0]
    _say("bias loop parity", check_flat(cfg, weights, part, x, layer.forward(x), u=None, b=b))
    layer.close()


# ---------------------------------------------------------------------------------- full-size configs

ALL_TOKENS_UP_TO = 8192     # the oracle evaluates a batch of this size in seconds


def _full(binding, ci, batches, n_sample=48, sizes=None, part=None, **scale):
    """Full-size layer `ci` on its evaluation batches, or (sizes) on the first `n` tokens of batch 0;
    `scale` replaces fields of the configuration (e.g. another expert split of the same dense layer).
    The routing of every token is checked; outputs are compared for every token up to ALL_TOKENS_UP_TO
    tokens, above that for a random sample plus the tokens of the ragged last row tile of every expert
    segment (a defect confined to one tile of one group would sit there or in a full tile, which the random
    tokens cover)."""
    cfg = synth.CONFIGS[ci] if not scale else synth.scaled(synth.CONFIGS[ci], **scale)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg) if part is None else part
    src = synth.make_token_source(cfg)
    layer = _layer(binding, cfg, weights, part)
    rng = np.random.Generator(np.random.PCG64(99 + ci))
    for bi in (batches if sizes is None else sizes):
        x = src.eval_batch(bi) if sizes is None else src.eval_batch(0, n=bi)
        T = x.shape[0]
        out = layer.forward(x)
        if T <= ALL_TOKENS_UP_TO:
            sample = None
        else:
            sample = tail_tokens(out["topk"], cfg.n_routed, rows=256, extra=rng.choice(T, size=n_sample, replace=False))
        _say("cfg%d T=%d" % (ci, T), check_flat(cfg, weights, part, x, out, sample=sample))
        dsample = None if T <= 2048 else np.sort(rng.choice(T, size=256, replace=False))
        _say("cfg%d T=%d dense" % (ci, T), check_dense(cfg, weights, x, layer.dense_forward(x), sample=dsample))
    layer.close()


def test_cfg1_full(binding):
    _full(binding, 1, [0, 1, 2])


def test_cfg1_on_the_partition_the_library_constructs(binding):
    """The forward on the partition cmoe_build produces from the calibration set (Sec. 4.1-4.2, Eq. 7), not an
    arbitrary one: the analytically built router on clustered tokens gives skewed, ragged expert segments
    (7 to 1700 tokens per expert at T = 2048), which is the workload the bench times.  The oracle runs on the
    same partition through cmoe_export_partition; every token of every evaluation batch is compared."""
    cfg = synth.CONFIGS[1]
    weights = synth.make_weights(cfg)
    src = synth.make_token_source(cfg)
    layer = binding.Layer.build(cfg, *weights, src.calibration())
    part = layer.export_partition()
    for bi in range(len(cfg.eval_batches)):
        x = src.eval_batch(bi)
        out = layer.forward(x)
        rep = check_flat(cfg, weights, part, x, out)
        rep["counts_min_max"] = (int(out["counts"].min()), int(out["counts"].max()))
        _say("cfg1 library partition T=%d" % x.shape[0], rep)
        assert np.array_equal(out["y"], layer.forward(x)["y"])
    x = src.eval_batch(2)
    assert layer.forward(x)["counts"].max() > 3 * layer.forward(x)["counts"].mean()      # the skew is there
    layer.close()


@pytest.mark.parametrize("ci", [2, 3])
def test_cfg2_cfg3_on_the_partition_the_library_constructs(binding, ci):
    """Configs 2 and 3 as the bench runs them: partition from cmoe_build_gpu on the calibration set, every
    evaluation batch (4096 and 8192 tokens; 1, 32 and 4096 tokens), every token compared."""
    cfg = synth.CONFIGS[ci]
    weights = synth.make_weights(cfg)
    src = synth.make_token_source(cfg)
    layer = binding.Layer.build(cfg, *weights, src.calibration(), on_gpu=True)
    part = layer.export_partition()
    for bi in range(len(cfg.eval_batches)):
        x = src.eval_batch(bi)
        out = layer.forward(x)
        rep = check_flat(cfg, weights, part, x, out)
        rep["counts_min_max"] = (int(out["counts"].min()), int(out["counts"].max()))
        _say("cfg%d library partition T=%d" % (ci, x.shape[0]), rep)
    layer.close()


def test_cfg1_mid_batches(binding):
    """Batch sizes between the decode path and the large-tile regime: the contraction kernels run their
    128x128 and 256x128 tile shapes at the layer's real depth."""
    _full(binding, 1, None, n_sample=32, sizes=[33, 64, 65, 300, 1000, 3072])


def test_cfg1_very_large_batch(binding):
    """32768 tokens (131072 slots, 1 GB of per-slot outputs): many rounds of every tile shape, 64-bit offsets
    into the hidden and slot buffers; routing of every token, and outputs of a random sample plus the last
    row tile of every expert segment, against the oracle."""
    _full(binding, 1, None, n_sample=256, sizes=[32768])


@pytest.mark.parametrize("n,n_s,n_k", [(8, 1, 5), (16, 3, 9), (16, 6, 6)])
def test_paper_expert_configurations(binding, n, n_s, n_k):
    """SxAyEz splits of the paper's configuration study (75 % of the neurons active) on the full-size layer."""
    _full(binding, 1, None, n_sample=24, sizes=[700], n_experts=n, n_shared=n_s, top_k=n_k)


def test_cfg2_full(binding):
    _full(binding, 2, [0, 1], n_sample=32)


def test_cfg3_full(binding):
    _full(binding, 3, [0, 1, 2], n_sample=32)


@pytest.mark.parametrize("dtype,d,T", [("bf16", 512, 300), ("bf16", 512, 9), ("bf16", 512, 1), ("bf16", 512, 40),
                                       ("fp32", 256, 70), ("bf16", 328, 100)])
@pytest.mark.parametrize("gate", [False, True])
def test_exact_score_ties_go_to_the_lower_expert_id(binding, dtype, d, T, gate):
    """Two pairs of routed experts share a representative neuron, so their scores (Eq. 8) are equal on every
    token, bit for bit.  The interface promises descending key with ties to the lowest expert id; the oracle's
    stable sort does the same, so here a token whose boundary keys are *equal* is not excused: the indices
    must match.  Sizes cover the one-token path, the team selection of the decode front end, the tile
    router and the fp32 / odd-width scorer; with the gate of Eq. 9 the tied pair gets equal biases."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=d, d_ff=12 * 64, n_experts=12, n_shared=2, top_k=3, dtype=dtype,
                       n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    reps = part["rep_neuron"].copy()
    reps[5] = reps[1]                         # experts 1 and 5, 2 and 3 tie on every token
    reps[3] = reps[2]
    part = {"neuron_order": part["neuron_order"], "rep_neuron": reps}
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    layer = _layer(binding, cfg, weights, part)
    u = b = None
    if gate:
        u, b = synth.make_gate_params(cfg)
        b[5], b[3] = b[1], b[2]
        layer.set_gate_params(u, b)
    out = layer.forward(x)
    rep = check_flat(cfg, weights, part, x, out, u=u, b=b, exact_ties_strict=True)
    _say("exact ties %s d=%d T=%d gate=%s" % (dtype, d, T, gate), rep)
    sel = out["topk"]
    for hi, lo in ((5, 1), (3, 2)):
        has_hi, has_lo = (sel == hi).any(axis=1), (sel == lo).any(axis=1)
        assert not (has_hi & ~has_lo).any()                    # the higher id never gets in without the lower one
        both = has_hi & has_lo
        pos_lo = np.argmax(sel == lo, axis=1)
        pos_hi = np.argmax(sel == hi, axis=1)
        assert (pos_lo[both] + 1 == pos_hi[both]).all()        # equal keys: listed next to each other, lower id first
    if T >= 40:
        assert rep["exact_ties"] > 0                           # the pair did sit on the boundary for some tokens
    layer.close()


def test_layer_without_its_dense_baseline(binding):
    """cmoe_set_baseline(0): half the device memory, the same MoE forward, and the dense call says why it cannot run."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=200)
    full = _layer(binding, cfg, weights, part)
    lean = _layer(binding, cfg, weights, part, baseline=False)
    assert binding.cmoe_packed_bytes(lean.h) < 0.6 * binding.cmoe_packed_bytes(full.h)
    a, b_ = full.forward(x), lean.forward(x)
    assert np.array_equal(a["y"], b_["y"]) and np.array_equal(a["topk"], b_["topk"])
    check_flat(cfg, weights, part, x, b_)
    with pytest.raises(binding.CmoeError, match="baseline"):
        lean.dense_forward(x)
    full.close()
    lean.close()


def test_set_gate_params_between_forwards_in_flight(binding):
    """Gate parameters changed while forwards are queued on a non-blocking stream: the call waits for the
    device, so every forward enqueued before it used the old values and every one after it the new ones."""
    import torch
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    layer = _layer(binding, cfg, weights, part)
    xh = synth.make_token_source(cfg).eval_batch(0, n=300)
    u, b = synth.make_gate_params(cfg)
    ref0 = layer.forward(xh)["y"]
    layer.set_gate_params(u, b)
    ref1 = layer.forward(xh)["y"]
    layer.set_gate_params(None, None)
    assert not np.array_equal(ref0, ref1)
    x = torch.from_numpy(xh).to("cuda", torch.bfloat16)
    ys = [torch.empty_like(x) for _ in range(6)]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for i in range(3):
            layer.forward_device(x, ys[i])
        layer.set_gate_params(u, b)
        for i in range(3, 6):
            layer.forward_device(x, ys[i])
    torch.cuda.synchronize()
    for i in range(6):
        assert np.array_equal(ys[i].float().cpu().numpy().astype(np.float64), ref0 if i < 3 else ref1)
    layer.close()


def test_mfma_probe_reports_a_plausible_rate(binding):
    """The measurement aid runs, and all-zero operands are never slower than random ones."""
    binding.cmoe_probe_mfma(True, 16384)            # brings an idle device up to its sustained clock first
    tf0, mhz0 = binding.cmoe_probe_mfma(False, 2048)
    tf1, mhz1 = binding.cmoe_probe_mfma(True, 2048)
    _say("mfma probe", {"zero_TFLOPs": tf0, "zero_MHz": mhz0, "random_TFLOPs": tf1, "random_MHz": mhz1})
    assert 100.0 < tf1 <= tf0 * 1.05 < 2700.0
    with pytest.raises(binding.CmoeError):
        binding.cmoe_probe_mfma(True, 0)


def test_hbm_probe_reports_a_plausible_rate(binding):
    """The streaming-read probe reports a rate between what a single HBM stack delivers and the published
    peak of the part, and rejects sizes it cannot run."""
    g = binding.cmoe_probe_hbm(1 << 30, 3)
    _say("hbm probe", {"GBs": g})
    assert 1000.0 < g < 8000.0
    with pytest.raises(binding.CmoeError):
        binding.cmoe_probe_hbm(1024, 3)
    with pytest.raises(binding.CmoeError):
        binding.cmoe_probe_hbm(1 << 30, 0)
