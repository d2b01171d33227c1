"""The forward entry point that allocates nothing (cmoe_forward_static): its workspace is a static device
array inside the library.  Called through the C ABI and compared with cmoe_forward on the same inputs:
expert indices, scores and counts bit for bit, outputs within the bf16 tolerance (the K split of a batch of
a few hundred tokens may differ, see the header) and bit for bit at decode sizes; two calls in a row, the
second with a smaller batch, so that nothing may depend on what the first left in the array."""
import numpy as np
import pytest

from paper_2502_04416_amd import synth
from parity_utils import check_flat, tokenwise_rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2502_04416_amd import binding as b
    b.load()
    return b


def _both(binding, layer, cfg, x_host, stream_ptr):
    import torch
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    x = torch.from_numpy(x_host).to("cuda", tdt)
    T = x.shape[0]
    outs = []
    for static in (False, True):
        y = torch.full_like(x, float("nan"))
        topk = torch.full((T, cfg.top_k), -1, dtype=torch.int32, device="cuda")
        scores = torch.zeros((T, cfg.n_routed), dtype=torch.float32, device="cuda")
        counts = torch.zeros((cfg.n_routed,), dtype=torch.int32, device="cuda")
        if static:
            binding.cmoe_forward_static(layer.h, x.data_ptr(), T, y.data_ptr(), topk.data_ptr(), scores.data_ptr(),
                                        counts.data_ptr(), stream_ptr)
        else:
            layer.forward_device(x, y, topk, scores, counts)
        torch.cuda.synchronize()
        outs.append({"y": y.float().cpu().numpy().astype(np.float64), "topk": topk.cpu().numpy().astype(np.int64),
                     "scores": scores.cpu().numpy().astype(np.float64), "counts": counts.cpu().numpy()})
    return outs


@pytest.mark.parametrize("dtype,d,sizes,bitwise", [
    ("bf16", 512, (16, 5), True),          # weight-streaming decode kernels
    ("bf16", 2048, (300, 40), False),      # tiled contractions; batches of this size split K
    ("fp32", 256, (200, 64), True),        # plain-FMA path
])
def test_static_forward_matches_the_workspace_forward(binding, dtype, d, sizes, bitwise):
    import torch
    cfg = synth.scaled(synth.CONFIGS[1], d_model=d, d_ff=2752, dtype=dtype, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    layer = binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"])
    assert binding.cmoe_forward_static_max_tokens(layer.h) >= max(sizes)
    src = synth.make_token_source(cfg)
    stream = int(torch.cuda.current_stream().cuda_stream)
    for i, T in enumerate(sizes):                        # two calls in a row, the second one smaller
        x = src.eval_batch(i, n=T)
        ref, got = _both(binding, layer, cfg, x, stream)
        assert np.array_equal(got["topk"], ref["topk"])
        assert np.array_equal(got["scores"], ref["scores"])
        assert np.array_equal(got["counts"], ref["counts"])
        assert np.isfinite(got["y"]).all()
        if bitwise:
            assert np.array_equal(got["y"], ref["y"])
        else:
            assert tokenwise_rel_err(got["y"], ref["y"]).max() <= 1e-2
        rep = check_flat(cfg, weights, part, x, got)       # ... and against the oracle
        print("\n[parity] static forward %s d=%d T=%d: %s" % (dtype, d, T, rep), flush=True)
    layer.close()


def test_static_forward_rejects_what_does_not_fit(binding):
    import torch
    cfg = synth.scaled(synth.CONFIGS[1], d_model=2048, d_ff=2752, n_centres=16)
    weights = synth.make_weights(cfg)
    part = synth.trivial_partition(cfg)
    layer = binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"])
    t_max = binding.cmoe_forward_static_max_tokens(layer.h)
    assert 100 < t_max < 100000 and binding.cmoe_static_scratch_bytes() == 32 << 20
    T = t_max + 1
    x = torch.zeros((T, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros_like(x)
    with pytest.raises(binding.CmoeError, match="static scratch"):
        binding.cmoe_forward_static(layer.h, x.data_ptr(), T, y.data_ptr(), None, None, None, 0)
    with pytest.raises(binding.CmoeError, match="null"):
        binding.cmoe_forward_static(layer.h, None, 4, y.data_ptr(), None, None, None, 0)
    binding.cmoe_forward_static(layer.h, x.data_ptr(), 0, y.data_ptr(), None, None, None, 0)      # T = 0: no-op
    # the largest batch that fits does run
    xs = torch.from_numpy(synth.make_token_source(cfg).eval_batch(0, n=t_max)).to("cuda", torch.bfloat16)
    ys = torch.full_like(xs, float("nan"))
    binding.cmoe_forward_static(layer.h, xs.data_ptr(), t_max, ys.data_ptr(), None, None, None,
                                int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    assert torch.isfinite(ys.float()).all()
    layer.close()
