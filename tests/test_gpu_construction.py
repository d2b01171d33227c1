"""GPU-side activation profiling (App. A.2 steps 1-2 on the device) against the CPU oracle, and
cmoe_build_gpu against cmoe_build.

The device accumulates bf16 products in fp32 where the oracle works in fp64, so a token whose K_a-th and
(K_a+1)-th largest |h| are closer than that rounding may legitimately get a different index set; such
tokens are counted, must be rare, and their sets must still be valid (every chosen magnitude at least the
(K_a+1)-th largest, up to the same tolerance)."""
import numpy as np
import pytest

from oracle import cmoe_oracle as O
from paper_2502_04416_amd import synth

pytestmark = pytest.mark.gpu

REL_GAP = 2e-5      # fp32 accumulation over d <= 4096 exact bf16 products: observed error <= 3e-6 relative


@pytest.fixture(scope="module")
def binding():
    from paper_2502_04416_amd import binding as b
    b.load()
    return b


def _check_active(active, h_abs, k_act):
    """active [n, k_act] from the library, h_abs [n, d_ff] the oracle's magnitudes.  Returns #excused tokens."""
    excused = 0
    for t in range(h_abs.shape[0]):
        order = np.argsort(-h_abs[t], kind="stable")
        ref = set(order[:k_act].tolist())
        got = active[t].tolist()
        assert len(set(got)) == k_act and min(got) >= 0 and max(got) < h_abs.shape[1]
        if set(got) == ref:
            continue
        kth, nxt = h_abs[t, order[k_act - 1]], h_abs[t, order[k_act]]
        assert kth - nxt <= REL_GAP * kth, "token %d: index sets differ although the gap is %g relative" % (t, (kth - nxt) / kth)
        assert (h_abs[t, got] >= nxt * (1.0 - REL_GAP)).all()
        excused += 1
    return excused


def test_profile_small_bf16(binding):
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16, n_calib=333)
    wg, wu, _ = synth.make_weights(cfg)
    x = synth.make_token_source(cfg).calibration()
    active = binding.cmoe_profile_activations(binding.make_config(cfg), wg, wu, x, on_gpu=True)
    h_abs = np.abs(O.hidden_states(x, wg, wu))
    excused = _check_active(active, h_abs, cfg.k_act)
    print("\n[parity] gpu profile small: %d of %d tokens excused" % (excused, x.shape[0]), flush=True)
    assert excused <= 2
    # descending order of magnitude inside a row
    for t in range(0, x.shape[0], 37):
        v = h_abs[t, active[t]]
        assert (np.diff(v) <= REL_GAP * v[:-1]).all()


def test_profile_cfg1_full_size_sample(binding):
    """The LLaMA-2-7B-shaped layer: 2048 calibration tokens on the device, 256 of them checked."""
    cfg = synth.CONFIGS[1]
    wg, wu, _ = synth.make_weights(cfg)
    x = synth.make_token_source(cfg).calibration()
    active = binding.cmoe_profile_activations(binding.make_config(cfg), wg, wu, x, on_gpu=True)
    idx = np.arange(0, x.shape[0], 8)
    h_abs = np.abs(O.hidden_states(x[idx], wg, wu))
    excused = _check_active(active[idx], h_abs, cfg.k_act)
    print("\n[parity] gpu profile cfg1: %d of %d sampled tokens excused" % (excused, idx.size), flush=True)
    assert excused <= 3


def test_build_gpu_matches_build_on_the_host(binding):
    """Same construction from the device's profile: rates, shared set and optimal cost agree with the host
    build whenever no token was excused; otherwise the rates differ by at most the excused tokens."""
    cfg = synth.scaled(synth.CONFIGS[1], d_model=512, d_ff=2752, n_centres=16, n_calib=400)
    w = synth.make_weights(cfg)
    x = synth.make_token_source(cfg).calibration()
    c = binding.make_config(cfg)
    a_gpu = binding.cmoe_profile_activations(c, w[0], w[1], x, on_gpu=True)
    a_cpu = binding.cmoe_profile_activations(c, w[0], w[1], x, on_gpu=False)
    differing = sum(set(a_gpu[t].tolist()) != set(a_cpu[t].tolist()) for t in range(x.shape[0]))
    h_gpu = binding.cmoe_build_gpu(c, *w, x)
    h_cpu = binding.cmoe_build(c, *w, x)
    e_gpu = binding.cmoe_export_partition(h_gpu, cfg.d_ff, cfg.n_routed)
    e_cpu = binding.cmoe_export_partition(h_cpu, cfg.d_ff, cfg.n_routed)
    print("\n[parity] build_gpu: %d tokens with a different set, cost %.6f vs %.6f" % (differing, e_gpu["cost"], e_cpu["cost"]),
          flush=True)
    assert np.abs(e_gpu["mu"] - e_cpu["mu"]).max() <= differing / x.shape[0] + 1e-7
    if differing == 0:
        assert np.array_equal(e_gpu["mu"], e_cpu["mu"])
        assert np.array_equal(e_gpu["neuron_order"], e_cpu["neuron_order"])
        assert np.array_equal(e_gpu["rep_neuron"], e_cpu["rep_neuron"])
        assert e_gpu["cost"] == e_cpu["cost"]
    # whatever the profile, the result is a valid partition
    assert sorted(e_gpu["neuron_order"].tolist()) == list(range(cfg.d_ff))
    m = cfg.m
    for j, r in enumerate(e_gpu["rep_neuron"]):
        assert r in e_gpu["neuron_order"][(cfg.n_shared + j) * m:(cfg.n_shared + j + 1) * m]
    binding.cmoe_destroy(h_gpu)
    binding.cmoe_destroy(h_cpu)


def test_build_gpu_rejects_what_it_cannot_do(binding):
    cfg = synth.CONFIGS[0]                                   # fp32 layer
    w = synth.make_weights(cfg)
    x = synth.make_token_source(cfg).calibration()
    with pytest.raises(binding.CmoeError, match="bf16"):
        binding.cmoe_build_gpu(binding.make_config(cfg), *w, x)
