"""GPU parity of neuron-level activation sparsity inside the routed experts (Sec. 5, 'Orthogonality with
Activation Sparsity'): hidden activations of the selected routed experts below a threshold are dropped before
the down projection; the shared experts are left alone.  One and two tokens run the kernel that reads only the
surviving neurons' rows of W_down; larger batches zero the dropped activations and run the usual kernels."""
import numpy as np
import pytest

from oracle import cmoe_oracle as O
from paper_2502_04416_amd import synth
from parity_utils import check_flat

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2502_04416_amd import binding as b
    b.load()
    return b


def _threshold(cfg, weights, x, weight_informed, share):
    """A threshold that drops about `share` of the activations: that quantile of the criterion over all neurons
    of a sample of tokens, as a float32 (the interface takes a float)."""
    wg, wu, wd = weights
    h = np.abs(O.hidden_states(x[:64], wg, wu))
    if weight_informed:
        h = h * np.sqrt((wd.astype(np.float64) ** 2).sum(axis=1))[None, :]
    return float(np.float32(np.quantile(h, share)))


@pytest.mark.parametrize("T", [1, 2, 3, 16, 40, 300])
@pytest.mark.parametrize("mode", [1, 2])
def test_neuron_sparsity_small(binding, T, mode):
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    src = synth.make_token_source(cfg)
    x = src.eval_batch(0, n=T)
    tau = _threshold(cfg, weights, src.calibration(n=64), mode == 2, 0.5)
    layer = binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"], neuron_sparsity=(mode, tau))
    out = layer.forward(x)
    rep = check_flat(cfg, weights, part, x, out, neuron=(tau, mode == 2))
    print("\n[parity] neuron sparsity mode %d T=%d tau=%.4g: %s" % (mode, T, tau, rep), flush=True)
    assert 0.2 < rep["kept"] < 0.8
    assert np.array_equal(out["y"], layer.forward(x)["y"])                  # deterministic
    # the threshold matters: the plain forward differs, and switching the feature off restores it bit for bit
    plain = binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"])
    want = plain.forward(x)
    assert not np.array_equal(want["y"], out["y"])
    layer.set_neuron_sparsity(0, 0.0)
    off = layer.forward(x)
    assert np.array_equal(off["y"], want["y"]) and np.array_equal(off["topk"], want["topk"])
    # gate parameters of Eq. 9 and the threshold together
    u, b = synth.make_gate_params(cfg)
    layer.set_gate_params(u, b)
    layer.set_neuron_sparsity(mode, tau)
    rep = check_flat(cfg, weights, part, x, layer.forward(x), u=u, b=b, neuron=(tau, mode == 2))
    print("[parity] neuron sparsity mode %d T=%d with gate: %s" % (mode, T, rep), flush=True)
    plain.close()
    layer.close()


@pytest.mark.parametrize("T", [1, 2, 33])
def test_neuron_sparsity_extreme_thresholds(binding, T):
    """tau = 0 keeps everything (the plain layer within rounding); a threshold above every activation leaves the
    shared experts only."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    x = synth.make_token_source(cfg).eval_batch(0, n=T)
    layer = binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"], neuron_sparsity=(1, 0.0))
    rep = check_flat(cfg, weights, part, x, layer.forward(x), neuron=(0.0, False))
    assert rep["kept"] == 1.0
    check_flat(cfg, weights, part, x, layer.forward(x))                     # ... which is the plain oracle too
    layer.set_neuron_sparsity(1, 1e30)
    out = layer.forward(x)
    rep = check_flat(cfg, weights, part, x, out, neuron=(1e30, False))
    assert rep["kept"] == 0.0
    shared = O.expert_output(x, *weights, part["neuron_order"][: cfg.n_shared * cfg.m])
    assert (np.abs(out["y"] - shared).max(axis=1) <= 1e-2 * np.abs(shared).max(axis=1)).all()
    layer.close()


def test_neuron_sparsity_full_size_config_1(binding):
    """The LLaMA-2-7B-shaped layer on the partition the library constructs, half of the routed activations
    dropped by magnitude: one token, two tokens (surviving rows only), 16 and 2048 tokens (masked activations)."""
    cfg = synth.CONFIGS[1]
    weights = synth.make_weights(cfg)
    src = synth.make_token_source(cfg)
    tau = _threshold(cfg, weights, src.calibration(n=64), False, 0.5)
    layer = binding.Layer.build(cfg, *weights, src.calibration(), upload=False, on_gpu=True)
    layer.set_neuron_sparsity(1, tau)
    layer.upload()
    part = layer.export_partition()
    for T in (1, 2, 16, 2048):
        x = src.eval_batch(2, n=T)
        rep = check_flat(cfg, weights, part, x, layer.forward(x), neuron=(tau, False))
        print("\n[parity] neuron sparsity cfg1 T=%d tau=%.4g: %s" % (T, tau, rep), flush=True)
    layer.close()


def test_neuron_sparsity_argument_errors(binding):
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    layer = binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"])
    with pytest.raises(binding.CmoeError, match="before cmoe_upload"):
        layer.set_neuron_sparsity(1, 0.1)
    layer.set_neuron_sparsity(0, 0.0)                                       # switching off is always allowed
    layer.close()
    lazy = binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"], upload=False)
    before = binding.cmoe_packed_bytes(lazy.h)
    with pytest.raises(binding.CmoeError, match="mode"):
        lazy.set_neuron_sparsity(3, 0.1)
    with pytest.raises(binding.CmoeError, match="tau"):
        lazy.set_neuron_sparsity(1, -1.0)
    with pytest.raises(binding.CmoeError, match="tau"):
        lazy.set_neuron_sparsity(1, float("nan"))
    lazy.set_neuron_sparsity(2, 0.1)
    assert binding.cmoe_packed_bytes(lazy.h) - before >= 2 * cfg.n_routed * cfg.m * cfg.d_model
    with pytest.raises(binding.CmoeError, match="sparsity"):
        binding.Hierarchy([lazy], 1, np.zeros((cfg.d_model, 1), dtype=np.float32), None)
    lazy.close()
    f32 = synth.scaled(synth.CONFIGS[0], d_model=64, d_ff=256, n_experts=8, n_shared=1, top_k=2)
    w = synth.make_weights(f32)
    p = synth.trivial_partition(f32)
    l32 = binding.Layer.from_partition(f32, *w, p["neuron_order"], p["rep_neuron"], upload=False)
    with pytest.raises(binding.CmoeError, match="bf16"):
        l32.set_neuron_sparsity(1, 0.1)
    l32.close()
