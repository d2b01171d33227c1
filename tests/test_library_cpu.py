"""Host-side checks of libcmoe that need no GPU: the library loads, exports every symbol the public
header declares, and its argument checks turn bad input into error codes (never a crash)."""
import os
import re

import numpy as np
import pytest

from paper_2502_04416_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "cmoe.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(cmoe_[a-z_]+)\s*\(", header))
    assert len(declared) >= 32
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert "gfx950" in binding.cmoe_version()


def _tiny():
    cfg = synth.scaled(synth.CONFIGS[0], d_model=16, d_ff=32, n_experts=4, n_shared=1, top_k=1)
    return cfg, synth.make_weights(cfg), synth.trivial_partition(cfg)


def test_build_from_partition_roundtrip(lib):
    cfg, w, p = _tiny()
    h = binding.cmoe_build_from_partition(binding.make_config(cfg), *w, p["neuron_order"], p["rep_neuron"])
    e = binding.cmoe_export_partition(h, cfg.d_ff, cfg.n_routed)
    assert np.array_equal(e["neuron_order"], p["neuron_order"]) and np.array_equal(e["rep_neuron"], p["rep_neuron"])
    assert binding.cmoe_packed_bytes(h) > 3 * cfg.d_model * cfg.d_ff * 4
    assert binding.cmoe_workspace_bytes(h, 128) > binding.cmoe_workspace_bytes(h, 1) > 0
    binding.cmoe_destroy(h)


@pytest.mark.parametrize("field,value,msg", [
    ("n_experts", 5, "multiple"),            # d_ff % N != 0
    ("n_shared", 4, "n_shared"),             # N_s >= N
    ("top_k", 4, "top_k"),                   # N_k > N_r
    ("top_k", 0, "top_k"),
    ("dtype", "bad", "dtype"),
])
def test_bad_config_is_rejected(lib, field, value, msg):
    cfg, w, p = _tiny()
    c = binding.make_config(cfg)
    if field == "dtype":
        c.dtype = 7
    else:
        setattr(c, field, value)
    with pytest.raises(binding.CmoeError, match=msg):
        binding.cmoe_build_from_partition(c, *w, p["neuron_order"], p["rep_neuron"])


def test_bad_partition_is_rejected(lib):
    cfg, w, p = _tiny()
    order = p["neuron_order"].copy()
    order[0] = order[1]
    with pytest.raises(binding.CmoeError, match="permutation"):
        binding.cmoe_build_from_partition(binding.make_config(cfg), *w, order, p["rep_neuron"])
    reps = p["rep_neuron"].copy()
    reps[0] = cfg.d_ff
    with pytest.raises(binding.CmoeError, match="rep_neuron"):
        binding.cmoe_build_from_partition(binding.make_config(cfg), *w, p["neuron_order"], reps)


def test_forward_before_upload_is_an_error(lib):
    cfg, w, p = _tiny()
    h = binding.cmoe_build_from_partition(binding.make_config(cfg), *w, p["neuron_order"], p["rep_neuron"])
    with pytest.raises(binding.CmoeError, match="upload"):
        binding.cmoe_forward(h, 1, 1, 1, None, None, None, 1, 1)
    binding.cmoe_destroy(h)


def test_null_handles(lib):
    assert binding.cmoe_packed_bytes(None) == 0
    assert binding.cmoe_workspace_bytes(None, 4) == 0
    with pytest.raises(binding.CmoeError):
        binding.cmoe_set_gate_params(None, None, None)
    binding.cmoe_destroy(None)


def test_generator_rounding_matches_torch():
    """The input generator's bf16 rounding against torch's conversion (a library routine)."""
    import torch
    x = (np.random.default_rng(0).standard_normal(100000) * 3).astype(np.float32)
    assert np.array_equal(synth.round_to_bf16(x), torch.from_numpy(x).bfloat16().float().numpy())


def test_update_bias_matches_the_oracle_on_the_host(lib):
    """cmoe_update_bias is host arithmetic (Sec. 4.3): same result as the oracle's step, fp32 vs fp64."""
    from oracle import cmoe_oracle as O
    cfg = synth.scaled(synth.CONFIGS[0], d_model=16, d_ff=48, n_experts=6, n_shared=1, top_k=2)
    w, p = synth.make_weights(cfg), synth.trivial_partition(cfg)
    h = binding.cmoe_build_from_partition(binding.make_config(cfg), *w, p["neuron_order"], p["rep_neuron"])
    u0 = np.linspace(-0.5, 0.5, cfg.n_routed).astype(np.float32)
    b0 = np.linspace(0.3, -0.3, cfg.n_routed).astype(np.float32)
    binding.cmoe_set_gate_params(h, u0, b0)
    ref = b0.astype(np.float64)
    rng = np.random.Generator(np.random.PCG64(3))
    for _ in range(5):
        counts = rng.integers(0, 50, size=cfg.n_routed)
        binding.cmoe_update_bias(h, counts, 1e-3)
        ref = O.bias_update(ref, counts, 1e-3)
    u, b = binding.cmoe_get_gate_params(h, cfg.n_routed)
    assert np.array_equal(u, u0)
    assert np.abs(b.astype(np.float64) - ref).max() < 1e-6
    binding.cmoe_update_bias(h, np.zeros(cfg.n_routed, dtype=np.int32), 1e-3)        # no routed token: unchanged
    assert np.array_equal(binding.cmoe_get_gate_params(h, cfg.n_routed)[1], b)
    with pytest.raises(binding.CmoeError):
        binding.cmoe_update_bias(h, -np.ones(cfg.n_routed, dtype=np.int32), 1e-3)
    binding.cmoe_destroy(h)


def test_baseline_copy_is_optional(lib):
    """Without the dense baseline the packed weights are about half the size, and the switch is one-way."""
    cfg, w, p = _tiny()
    h = binding.cmoe_build_from_partition(binding.make_config(cfg), *w, p["neuron_order"], p["rep_neuron"])
    both = binding.cmoe_packed_bytes(h)
    binding.cmoe_set_baseline(h, False)
    moe_only = binding.cmoe_packed_bytes(h)
    assert moe_only < both and both - moe_only >= 3 * cfg.d_model * cfg.d_ff * 4
    with pytest.raises(binding.CmoeError, match="released"):
        binding.cmoe_set_baseline(h, True)
    binding.cmoe_destroy(h)


def test_tuning_switches(lib):
    binding.cmoe_set_tuning("CMOE_SPLITK", 0)
    binding.cmoe_set_tuning("CMOE_SPLITK", 1)
    binding.cmoe_set_tuning("CMOE_GEMM1_CFG", -1)
    with pytest.raises(binding.CmoeError, match="unknown"):
        binding.cmoe_set_tuning("CMOE_NO_SUCH_SWITCH", 1)


def test_non_finite_calibration_tokens_are_rejected(lib):
    cfg = synth.scaled(synth.CONFIGS[0], d_model=16, d_ff=32, n_experts=4, n_shared=1, top_k=1, k_act=3)
    w = synth.make_weights(cfg)
    x = synth.make_token_source(cfg).calibration(n=40).copy()
    x[17, 3] = np.nan
    with pytest.raises(binding.CmoeError, match="token 17"):
        binding.cmoe_build(binding.make_config(cfg), *w, x)
    with pytest.raises(binding.CmoeError, match="token 17"):
        binding.cmoe_profile_activations(binding.make_config(cfg), w[0], w[1], x, on_gpu=False)
    x[17, 3] = np.inf
    with pytest.raises(binding.CmoeError, match="token 17"):
        binding.cmoe_build(binding.make_config(cfg), *w, x)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: the bench says so and exits instead of launching ranks."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
