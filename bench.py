#!/usr/bin/env python3
"""Bench of the MoE-FFN forward (router -> top-k -> permute -> shared + routed SwiGLU experts -> combine)
on one MI355X, through the C ABI of libcmoe.

    python bench.py [--gpus 1] [--steps K] [--warmup W]            # every configuration, one JSON line
    python bench.py --config 1 [--batch 2048]                      # one flat configuration in detail
    python bench.py --config 1 --sweep | --batch-sweep             # expert-configuration / batch-size studies

A step is one pass of the whole hot path over one batch of synthetic tokens already resident in HBM.
Without --config the headline (`value`, `ms_per_step`, `roofline`, `cpu_baseline`) is the largest
single-GPU workload, config 4: the Mixtral-8x7B-shaped layer of 8 experts whose experts were each
restructured into 8 sub-experts (2 shared + top-2 of 6), 4096 tokens, constructed by cmoe_hier_build from
the calibration set.  The `configs` array of the same line carries, for each of configs 1-4 and each of
their evaluation batches (decode batches included), the forward time, the baseline's time (dense FFN of
the same kernels; for config 4 the un-restructured MoE layer), the speedup, and the dominant kernel's
duration and roofline fraction.

The dominant kernel's duration is measured live by difference between two loops of forwards, each between
two HIP events on the launch stream: for compute-bound batches the loop with the gate/up launch issued twice
(tuning switch CMOE_REPEAT_STAGE) minus the plain loop, for decode batches the plain loop minus the loop
without that launch (CMOE_SKIP_STAGE).  What the loop gains or loses is that launch's cost inside the stream,
launch gap included, which is what a kernel trace reports for back-to-back launches of one stream; no
event-pair overhead enters (4-5 us on this runtime, half of a decode kernel).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TF = 2500.0     # dense bf16 MFMA
FP32_VALU_PEAK_TF = 157.3
# HBM bytes (fetched + written) of one gate/up launch from the two rocprofv3 --pmc runs summarised under
# profiles/ (FETCH_SIZE x 2.000 and WRITE_SIZE x 1.000 against a copy of known size), keyed by (config, T);
# a property of the tiling and the workload, not re-measured per run
MEASURED_GATE_UP_TRAFFIC_BYTES = {(1, 2048): 310.6e6, (4, 4096): 2642.2e6}
METRIC = "MoE-FFN layer tokens/s (+ speedup vs dense FFN; % HBM BW decode, % MFMA prefill)"


RAMP_MS = 40.0


def timed(fn, steps, warmup):
    """Milliseconds per call of `fn` over exactly `steps` calls bracketed by synchronize, after `warmup` untimed
    calls.  Before the warm-up the same call runs for RAMP_MS of wall time: a device that has been idle (a
    fresh process, host-side construction, a CPU timing leg) starts at a low clock and takes tens of
    milliseconds of load to reach the clock it then holds; ten warm-up steps of 0.25 ms are over before that
    (measured on config 1, T = 2048: 0.250 ms per step after 10 warm-up steps, 0.219-0.223 ms after 100 or more,
    and 0.220 ms by per-forward events either way)."""
    import torch
    t_ramp = time.perf_counter()
    while (time.perf_counter() - t_ramp) * 1e3 < RAMP_MS:
        for _ in range(8):
            fn()
        torch.cuda.synchronize()
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=None,
                    help="one configuration in detail (1-3 flat, 4 hierarchical); default: all of them in one line")
    ap.add_argument("--batch", type=int, default=None, help="token count (default: the config's largest eval batch)")
    ap.add_argument("--construct", choices=["library", "gpu", "arbitrary"], default="library",
                    help="partition from cmoe_build on the calibration set (host), from cmoe_build_gpu (activation "
                         "profiling on the device), or a seeded arbitrary one")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-batch measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-dense", action="store_true",
                    help="skip the dense-FFN baseline (so that a kernel trace holds MoE launches only)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (reference reading for HBM byte counters)")
    ap.add_argument("--layer-copies", type=int, default=8, help="device copies of the layer cycled at decode")
    ap.add_argument("--sweep", action="store_true",
                    help="the paper's expert configurations SxAyEz at 75 %% active and the sparsity ladder with 16 "
                         "experts, on the config's dense layer (speedup vs dense at two batch sizes)")
    ap.add_argument("--sparsity", action="store_true",
                    help="neuron-level activation sparsity inside the routed experts (Sec. 5): forward time at 1, 2, 16 and "
                         "2048 tokens with the feature off and with thresholds that drop 25 / 50 / 75 %% of the routed "
                         "activations, on the config's layer")
    ap.add_argument("--balance", action="store_true",
                    help="load-balancing study (Sec. 4.3): the +-gamma bias step of Eq. 9 run on a stream of batches, and "
                         "what the routing skew costs the expert kernels before and after")
    ap.add_argument("--balance-steps", type=int, default=200, help="bias steps of the load-balancing study")
    ap.add_argument("--gamma", type=float, default=1e-3, help="step size of the bias update (the paper's 1e-3)")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="the layer against its baseline over batch sizes from 1 token up (arbitrary partition; several "
                         "device copies of the layer and token sets are cycled so that weights come from HBM)")
    return ap.parse_args()


BATCH_SWEEP = [1, 4, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096]


def shared_in_front(cfg, T):
    """Does the library run the shared expert's gate/up units inside the selection/placement launch (so that
    the gate/up launch streams the routed experts only)?  Mirrors the library's rule: bf16 flat layer with
    shared experts, at most 16 tokens, a model width the decode kernels are built for."""
    return (cfg.dtype == "bf16" and cfg.n_shared > 0 and not cfg.n_outer and 1 <= T <= 16
            and cfg.d_model % 256 == 0 and cfg.d_model // 256 in (2, 4, 8, 16)
            and os.environ.get("CMOE_FRONT_SHARED", "1")[:1] != "0")


def bench_batches(args, cfg, np, torch, binding, synth):
    """Forward time of the restructured layer and of its baseline (dense FFN, or the un-restructured MoE layer
    for the hierarchical config) as a function of the batch size."""
    dev = torch.device("cuda:0")
    t_setup = time.time()
    src = synth.make_token_source(cfg)
    n_sets = 8 if cfg.n_outer else 4
    if cfg.n_outer:
        w_router, offsets = synth.make_outer_router(cfg)
        subs = []
        for e in range(cfg.n_outer):
            wg, wu, wd = synth.make_outer_expert_weights(cfg, e)
            part = synth.trivial_partition(cfg, seed=e)
            subs.append(binding.Layer.from_partition(cfg, wg, wu, wd, part["neuron_order"], part["rep_neuron"], upload=False))
        layers = [binding.Hierarchy(subs, cfg.outer_top_k, w_router, offsets)]       # 2.8 GB: beyond the Infinity Cache
    else:
        weights = synth.make_weights(cfg)
        part = synth.trivial_partition(cfg)
        layers = [binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"]) for _ in range(n_sets)]

    rows = []
    for T in ([args.batch] if args.batch else BATCH_SWEEP):
        xs = [torch.from_numpy(src.draw(100 + i, T)).to(dev, torch.bfloat16) for i in range(n_sets)]
        y = torch.empty_like(xs[0])
        st = {"i": 0}

        def moe():
            i = st["i"] % n_sets
            st["i"] += 1
            if cfg.n_outer:
                layers[0].forward_device(xs[i], y)
            else:
                layers[i].forward_device(xs[i], y, None, None, None)

        def base():
            i = st["i"] % n_sets
            st["i"] += 1
            (layers[0] if cfg.n_outer else layers[i]).dense_forward_device(xs[i], y)

        a = timed(moe, args.steps, args.warmup)
        b = timed(base, args.steps, args.warmup)
        layers[0].forward_timed(xs[0], y, False)
        stage = layers[0].forward_timed(xs[0], y, False)
        rows.append({"T": T, "ms_per_step": a, "baseline_ms_per_step": b, "speedup_vs_baseline": b / a,
                     "tokens_per_s": T / (a * 1e-3),
                     "stage_ms_with_event_overhead": dict(zip(("router", "permute", "gate_up", "down", "combine"), map(float, stage)))})
    head = rows[-1]
    print(json.dumps({
        "metric": METRIC,
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "clock_ramp_ms": RAMP_MS,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "batch sizes on cfg%d %s; headline fields are T=%d" % (cfg.cfg, cfg.name, head["T"]),
                   "partition": "arbitrary", "baseline": "un-restructured MoE layer" if cfg.n_outer else "dense FFN"},
        "batch_sweep": rows, "setup_s": time.time() - t_setup}))


def bench_hier(args, cfg, np, torch, binding, synth):
    """The hierarchical case (Sec. 4.4): an MoE layer with a linear top-k router whose experts were each
    restructured; the baseline is the same layer with every selected expert evaluated densely."""
    dev = torch.device("cuda:0")
    t_setup = time.time()
    w_router, offsets = synth.make_outer_router(cfg)
    layers = []
    for e in range(cfg.n_outer):
        wg, wu, wd = synth.make_outer_expert_weights(cfg, e)
        part = synth.trivial_partition(cfg, seed=e)
        layers.append(binding.Layer.from_partition(cfg, wg, wu, wd, part["neuron_order"], part["rep_neuron"], upload=False))
    hier = binding.Hierarchy(layers, cfg.outer_top_k, w_router, offsets)
    T = args.batch if args.batch else max(cfg.eval_batches)
    x = torch.from_numpy(synth.make_token_source(cfg).eval_batch(0, n=T)).to(dev, torch.bfloat16)
    y = torch.empty_like(x)

    ms_moe = timed(lambda: hier.forward_device(x, y), args.steps, args.warmup)
    ms_dense = timed(lambda: hier.dense_forward_device(x, y), args.steps, args.warmup)
    n_prof = max(5, min(args.steps, 20))
    st = np.zeros(5)
    sd = np.zeros(5)
    for _ in range(3):
        hier.forward_timed(x, y, False)
        hier.forward_timed(x, y, True)
    for _ in range(n_prof):
        st += hier.forward_timed(x, y, False)
        sd += hier.forward_timed(x, y, True)
    st /= n_prof
    sd /= n_prof
    ev = float(sd[0]) if sd[0] < 0.02 else 0.0044           # the dense form has no sub-expert scoring on some paths
    d, m = cfg.d_model, cfg.m
    act = cfg.outer_top_k * (cfg.n_shared + cfg.top_k)       # active sub-experts per token
    gu_ms = max(float(st[2]) - 0.0044, 1e-6)
    tf1, mhz1 = binding.cmoe_probe_mfma(True, 16384)
    roofline = {"kernel": "grouped_gemm_bf16_dma<gate_up>", "bound": "mfma",
                "achieved": 4.0 * d * m * act * T / (gu_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TF, "unit": "TFLOP/s",
                "traffic": None, "avg_launch_ms": gu_ms}
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    roofline["frac_of_sustained_mfma"] = roofline["achieved"] / tf1
    out = {
        "metric": METRIC,
        "value": T / (ms_moe * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "clock_ramp_ms": RAMP_MS,
        "ms_per_step": ms_moe, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "cfg%d %s: %d outer experts (top-%d) of d=%d d_ff=%d, each %d sub-experts of %d neurons, "
                               "%d shared + top-%d of %d routed, T=%d tokens"
                   % (cfg.cfg, cfg.name, cfg.n_outer, cfg.outer_top_k, d, cfg.d_ff, cfg.n_experts, m, cfg.n_shared,
                      cfg.top_k, cfg.n_routed, T), "partition": "arbitrary"},
        "dense_ms_per_step": ms_dense, "speedup_vs_dense": ms_dense / ms_moe,
        "active_fraction": act * m / float(cfg.outer_top_k * cfg.d_ff),
        "stage_ms": dict(zip(binding.STAGES, [float(v) for v in st])),
        "dense_stage_ms": dict(zip(binding.STAGES, [float(v) for v in sd])),
        "roofline": roofline, "mfma_probe": {"random_operands_TFLOPs": tf1, "random_operands_MHz": mhz1},
        "setup_s": time.time() - t_setup,
    }
    print(json.dumps(out))


# SxAyEz shapes of the paper's configuration study (all 75 % of the neurons active) and its sparsity ladder
# with 16 experts (fraction of inactive neurons 0.75 ... 0.125; the split into shared and routed experts
# is not given there: a quarter of the active experts, at least one, are shared here)
SWEEP_SHAPES = [("S1A5E8", 8, 1, 5), ("S3A3E8", 8, 3, 3), ("S2A4E8", 8, 2, 4), ("S4A8E16", 16, 4, 8),
                ("S6A6E16", 16, 6, 6), ("S3A9E16", 16, 3, 9),
                ("S1A3E16", 16, 1, 3), ("S2A4E16", 16, 2, 4), ("S2A6E16", 16, 2, 6), ("S3A7E16", 16, 3, 7),
                ("S4A10E16", 16, 4, 10)]


def bench_sweep(args, base, np, torch, binding, synth):
    """Speedup of the restructured layer over the dense one as a function of the expert configuration
    (Sec. 5, expert-configuration and sparsity studies), arbitrary partitions of the config's dense layer."""
    dev = torch.device("cuda:0")
    t_setup = time.time()
    weights = synth.make_weights(base)
    src = synth.make_token_source(base)
    batches = [args.batch] if args.batch else [2048, 8192]
    xs = {T: torch.from_numpy(src.eval_batch(0, n=T)).to(dev, torch.bfloat16) for T in batches}

    rows = []
    dense_ms = {}
    for name, n, n_s, n_k in SWEEP_SHAPES:
        cfg = synth.scaled(base, n_experts=n, n_shared=n_s, top_k=n_k)
        part = synth.trivial_partition(cfg)
        layer = binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"])
        for T in batches:
            y = torch.empty_like(xs[T])
            if T not in dense_ms:
                dense_ms[T] = timed(lambda: layer.dense_forward_device(xs[T], y), args.steps, args.warmup)
            ms = timed(lambda: layer.forward_device(xs[T], y), args.steps, args.warmup)
            rows.append({"shape": name, "T": T, "active_fraction": (n_s + n_k) / n, "ms_per_step": ms,
                         "tokens_per_s": T / (ms * 1e-3), "dense_ms_per_step": dense_ms[T],
                         "speedup_vs_dense": dense_ms[T] / ms})
        layer.close()
    head = rows[0]
    out = {
        "metric": METRIC,
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "clock_ramp_ms": RAMP_MS,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": base.dtype, "data": "synthetic",
        "config": {"workload": "sweep of expert configurations on cfg%d %s (d=%d d_ff=%d); headline fields are %s at T=%d"
                   % (base.cfg, base.name, base.d_model, base.d_ff, head["shape"], head["T"]), "partition": "arbitrary"},
        "sweep": rows, "setup_s": time.time() - t_setup,
    }
    print(json.dumps(out))


def event_loop_ms(fn, steps, warmup=8):
    """Milliseconds per call of `fn`: `steps` calls between two HIP events on the current (launch) stream,
    after the clock ramp and `warmup` calls."""
    import torch
    t_ramp = time.perf_counter()
    while (time.perf_counter() - t_ramp) * 1e3 < RAMP_MS:
        for _ in range(8):
            fn()
        torch.cuda.synchronize()
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def stage_costs_ms(binding, fn, steps, prefill, timed_fns):
    """Forward time and the cost of the gate/up launch inside the stream, by difference, both loops measured
    here back to back.  Compute-bound batches: the loop with that launch issued twice minus the plain loop
    (same clocks and power as the plain forward; agrees with a kernel trace within 2 %; leaving the launch out
    instead lets the clock rise for the other kernels and overstates it by 15 %).  Decode batches: the plain
    loop minus the loop without that launch (a second launch would find its weights in the cache; agrees with
    a trace within 3-6 %).  The per-stage table comes from events inside the library and contains the 4-5 us an
    event pair costs on this runtime in every entry."""
    import numpy as np
    full = event_loop_ms(fn, steps)
    out = {"forward": full}
    try:
        if prefill:
            binding.cmoe_set_tuning("CMOE_REPEAT_STAGE", 3)
            out["gate_up"] = max(event_loop_ms(fn, steps) - full, 1e-6)
        else:
            binding.cmoe_set_tuning("CMOE_SKIP_STAGE", 3)
            out["gate_up"] = max(full - event_loop_ms(fn, steps), 0.0)
            if out["gate_up"] < 0.1 * full:
                # one token on a flat layer: there is no gate/up launch, the selection launch runs every gate/up
                # unit.  Without the down launch the forward is scoring + that launch; the scoring launch's cost
                # is what a second one adds to the plain loop (a loop of scoring launches alone would run at the
                # host's launch rate, 8 us, and say nothing about the 5-6 us kernel).
                binding.cmoe_set_tuning("CMOE_SKIP_STAGE", 4)
                no_down = event_loop_ms(fn, steps)
                binding.cmoe_set_tuning("CMOE_SKIP_STAGE", 0)
                binding.cmoe_set_tuning("CMOE_REPEAT_STAGE", 6)
                out["score"] = max(event_loop_ms(fn, steps) - full, 0.0)
                out["gate_up"] = max(no_down - out["score"], 1e-6)
                out["fused_front"] = True
    finally:
        binding.cmoe_set_tuning("CMOE_SKIP_STAGE", 0)
        binding.cmoe_set_tuning("CMOE_REPEAT_STAGE", 0)
    acc, n = np.zeros(5), 0
    for f in timed_fns:
        f()
    for _ in range(3 if prefill else 2):
        for f in timed_fns:
            acc += f()
            n += 1
    out["events_raw"] = dict(zip(("router", "permute", "gate_up", "down", "combine"), (float(v) for v in acc / max(n, 1))))
    return out


def entry(cfg, T, ms, base_ms, costs, act_per_token, union=None, shared_front=False, baseline="dense FFN"):
    """One row of the `configs` array.  act_per_token: active experts per token ((N_s + N_k), times the outer
    top-k for the hierarchy); union: routed experts (plus shared ones) whose weights the batch touches (decode)."""
    d, m, es = cfg.d_model, cfg.m, 2
    row = {"cfg": cfg.cfg, "name": cfg.name, "T": T, "ms_per_step": ms, "tokens_per_s": T / (ms * 1e-3),
           "baseline": baseline, "baseline_ms_per_step": base_ms, "speedup_vs_baseline": base_ms / ms,
           "stage_ms_events_raw": costs["events_raw"]}
    gu = max(costs["gate_up"], 1e-6)
    if T >= 256:
        flops_gu = 4.0 * d * m * act_per_token * T
        n_router = cfg.n_routed * (cfg.n_outer or 1)
        flops_all = T * (6.0 * d * m * act_per_token + 4.0 * d * n_router + (2.0 * d * cfg.n_outer if cfg.n_outer else 0.0))
        row.update({"dominant_kernel": "grouped_gemm_bf16_dma<gate_up>", "bound": "mfma", "kernel_ms": gu,
                    "achieved": flops_gu / (gu * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TF, "unit": "TFLOP/s",
                    "frac": flops_gu / (gu * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF,
                    "down_frac_from_raw_events": 0.5 * flops_gu / (max(costs["events_raw"]["down"], 1e-6) * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF,
                    "whole_path_frac": flops_all / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF})
    else:
        n_shared_groups = cfg.n_shared * (cfg.outer_top_k if cfg.n_outer else 1)
        fused = bool(costs.get("fused_front"))
        bytes_gu = es * 2.0 * d * m * (union - (n_shared_groups if (shared_front and not fused) else 0))
        n_router = cfg.n_routed * (cfg.n_outer or 1)
        bytes_all = es * (3.0 * d * m * union + 2.0 * d * n_router)
        row.update({"dominant_kernel": ("route_place_all_kernel (selection + every gate/up unit)" if fused else
                                        "decode_gate_up_kernel" if T <= 16 else "grouped_gemm_bf16_dma<gate_up> (64x128 tiles)"),
                    "bound": "hbm", "kernel_ms": gu, "expert_groups_touched": union,
                    "shared_experts_in_front_launch": bool(shared_front), "all_gate_up_units_in_front_launch": fused,
                    "achieved": bytes_gu / (gu * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": bytes_gu / (gu * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "whole_path_frac": bytes_all / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS})
    return row


def bench_all(args, np, torch, binding, synth):
    """Every configuration in one line: headline = config 4 (hierarchical, 4096 tokens)."""
    dev = torch.device("cuda:0")
    t_setup = time.time()
    rows = []
    sub_steps = max(20, min(args.steps, 60))
    if args.copy_probe:
        # a copy of known size: 2^30 bytes read + 2^30 bytes written; scales FETCH_SIZE / WRITE_SIZE readings
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        a.copy_(b)
        torch.cuda.synchronize()
        del a, b

    def cycle(fns):
        st = {"i": 0}

        def step():
            fns[st["i"] % len(fns)]()
            st["i"] += 1
        return step

    # ---- flat layers: configs 1, 2 (same dense layer, two expert splits), 3 ----
    for ci in (1, 2, 3):
        cfg = synth.CONFIGS[ci]
        weights = synth.make_weights(cfg)
        src = synth.make_token_source(cfg)
        layer = binding.Layer.build(cfg, *weights, src.calibration(), on_gpu=True)
        part = layer.export_partition()
        copies = [layer]
        if any(T <= 64 for T in cfg.eval_batches):
            for _ in range(args.layer_copies - 1):
                copies.append(binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"]))
        for bi, T in enumerate(cfg.eval_batches):
            decode = T <= 64
            use = copies if decode else copies[:1]
            xs = [torch.from_numpy(src.eval_batch(bi) if i == 0 else src.draw(9000 + 100 * T + i, T)).to(dev, torch.bfloat16)
                  for i in range(len(use))]
            y = torch.empty_like(xs[0])
            cnt = torch.zeros((cfg.n_routed,), dtype=torch.int32, device=dev)
            moe = cycle([(lambda L=L, x=x: L.forward_device(x, y, None, None, None)) for L, x in zip(use, xs)])
            dense = cycle([(lambda L=L, x=x: L.dense_forward_device(x, y)) for L, x in zip(use, xs)])
            steps = max(sub_steps, 96) if decode else sub_steps
            costs = stage_costs_ms(binding, moe, steps, not decode,
                                   [(lambda L=L, x=x: L.forward_timed(x, y, False)) for L, x in zip(use, xs)])
            base_ms = event_loop_ms(dense, steps)
            union = None
            if decode:
                touched = 0.0
                for L, x in zip(use, xs):
                    L.forward_device(x, y, None, None, cnt)
                    torch.cuda.synchronize()
                    touched += float((cnt.cpu().numpy() > 0).sum())
                union = cfg.n_shared + touched / len(use)
            rows.append(entry(cfg, T, costs["forward"], base_ms, costs, cfg.n_shared + cfg.top_k, union,
                              shared_front=shared_in_front(cfg, T)))
        for L in copies:
            L.close()
        del copies, layer, weights
        torch.cuda.empty_cache()

    # ---- config 4, the headline: constructed by the library from the un-restructured layer ----
    cfg = synth.CONFIGS[4]
    w_router, offsets = synth.make_outer_router(cfg)
    ws = [synth.make_outer_expert_weights(cfg, e) for e in range(cfg.n_outer)]
    src = synth.make_token_source(cfg)
    t0 = time.time()
    hier = binding.Hierarchy.build(cfg, cfg.outer_top_k, [w[0] for w in ws], [w[1] for w in ws], [w[2] for w in ws],
                                   w_router, offsets, src.calibration(), on_gpu=True)
    construct_s = time.time() - t0
    T = max(cfg.eval_batches)
    x_host = src.eval_batch(0, n=T)
    x = torch.from_numpy(x_host).to(dev, torch.bfloat16)
    y = torch.empty_like(x)
    ms_moe = timed(lambda: hier.forward_device(x, y), args.steps, args.warmup)          # the contract's K steps
    ms_base = timed(lambda: hier.dense_forward_device(x, y), args.steps, args.warmup)
    costs = stage_costs_ms(binding, lambda: hier.forward_device(x, y), sub_steps, True, [lambda: hier.forward_timed(x, y, False)])
    act = cfg.outer_top_k * (cfg.n_shared + cfg.top_k)
    head = entry(cfg, T, ms_moe, ms_base, costs, act, baseline="un-restructured MoE layer (top-2 of 8 dense experts)")
    rows.append(head)
    outer = torch.empty((T, cfg.outer_top_k), dtype=torch.int32, device=dev)
    hier.forward_device(x, y, outer, None)
    torch.cuda.synchronize()
    outer_load = np.bincount(outer.cpu().numpy().ravel(), minlength=cfg.n_outer).tolist()
    tf0, mhz0 = binding.cmoe_probe_mfma(False, 16384)
    tf1, mhz1 = binding.cmoe_probe_mfma(True, 16384)
    roofline = {"kernel": head["dominant_kernel"], "bound": "mfma", "achieved": head["achieved"], "peak": MFMA_BF16_PEAK_TF,
                "unit": "TFLOP/s", "frac": head["frac"], "traffic": MEASURED_GATE_UP_TRAFFIC_BYTES.get((4, T)),
                "avg_launch_ms": head["kernel_ms"], "frac_of_sustained_mfma": head["achieved"] / tf1,
                "how": "loop of forwards with this launch issued twice minus the plain loop, HIP events on the launch stream"}
    out = {
        "metric": METRIC, "value": T / (ms_moe * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "clock_ramp_ms": RAMP_MS, "ms_per_step": ms_moe, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "cfg%d %s: %d outer experts (top-%d, Zipf(1.1) logit offsets) of d=%d d_ff=%d, each restructured "
                               "into %d sub-experts of %d neurons (%d shared + top-%d of %d routed), T=%d tokens"
                   % (cfg.cfg, cfg.name, cfg.n_outer, cfg.outer_top_k, cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.m,
                      cfg.n_shared, cfg.top_k, cfg.n_routed, T),
                   "partition": "cmoe_hier_build (profiling on the device), %d calibration tokens" % cfg.n_calib,
                   "k_act": cfg.k_act, "sigma_o": synth.SIGMA_O},
        "baseline_ms_per_step": ms_base, "speedup_vs_baseline": ms_base / ms_moe, "outer_expert_load": outer_load,
        "active_fraction": act * cfg.m / float(cfg.outer_top_k * cfg.d_ff),
        "roofline": roofline, "construct_s": construct_s,
        "mfma_probe": {"zero_operands_TFLOPs": tf0, "zero_operands_MHz": mhz0, "random_operands_TFLOPs": tf1,
                       "random_operands_MHz": mhz1},
        "configs": rows,
    }
    try:
        out["hbm_probe_GBs"] = binding.cmoe_probe_hbm(2 << 30, 5)
    except binding.CmoeError:
        out["hbm_probe_GBs"] = None
    if not args.no_cpu:
        from oracle import cmoe_oracle as O
        n_cpu = min(T, 4096)                       # the whole batch: about 12 s of oracle time on the box's 16 threads
        experts = []
        for e in range(cfg.n_outer):
            part = hier.expert_partition(e)
            experts.append({"w_gate": ws[e][0], "w_up": ws[e][1], "w_down": ws[e][2],
                            "neuron_order": part["neuron_order"], "rep_neuron": part["rep_neuron"]})
        t0 = time.perf_counter()
        O.hier_forward(x_host[:n_cpu], w_router, offsets, cfg.outer_top_k, experts, cfg.n_experts, cfg.n_shared, cfg.top_k)
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = {"value": n_cpu / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": "the first %d tokens of the same batch (all of it), fp64 numpy oracle (hier_forward), %.1f s" % (n_cpu, dt)}
    hier.close()
    out["setup_s"] = time.time() - t_setup
    print(json.dumps(out))


def bench_sparsity(args, cfg, np, torch, binding, synth):
    """Effect of neuron-level activation sparsity inside the routed experts on the forward time."""
    from oracle import cmoe_oracle as O          # only to place the thresholds (quantiles of |h| on calibration tokens)
    dev = torch.device("cuda:0")
    t_setup = time.time()
    weights = synth.make_weights(cfg)
    src = synth.make_token_source(cfg)
    base = binding.Layer.build(cfg, *weights, src.calibration(), upload=False, on_gpu=True)
    part = base.export_partition()
    base.close()
    h = np.abs(O.hidden_states(src.calibration(n=64), weights[0], weights[1]))
    copies = []
    for _ in range(args.layer_copies):
        L = binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"], upload=False, baseline=False)
        L.set_neuron_sparsity(1, 0.0)
        L.set_neuron_sparsity(0, 0.0)
        L.upload()
        copies.append(L)
    rows = []
    for T in ([args.batch] if args.batch else [1, 2, 16, 2048]):
        use = copies if T <= 64 else copies[:1]
        xs = [torch.from_numpy(src.draw(9000 + 100 * T + i, T)).to(dev, torch.bfloat16) for i in range(len(use))]
        y = torch.empty_like(xs[0])
        st = {"i": 0}

        def step():
            i = st["i"] % len(use)
            st["i"] += 1
            use[i].forward_device(xs[i], y, None, None, None)
        steps = max(args.steps, 200) if T <= 64 else args.steps
        row = {"T": T, "off_ms": event_loop_ms(step, steps)}
        for share in (0.25, 0.5, 0.75):
            tau = float(np.float32(np.quantile(h, share)))
            for L in use:
                L.set_neuron_sparsity(1, tau)
            row["drop_%d_ms" % int(share * 100)] = event_loop_ms(step, steps)
            row["tau_%d" % int(share * 100)] = tau
        for L in use:
            L.set_neuron_sparsity(0, 0.0)
        rows.append(row)
    head = rows[0]
    print(json.dumps({
        "metric": METRIC, "value": head["T"] / (head["off_ms"] * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "clock_ramp_ms": RAMP_MS, "ms_per_step": head["off_ms"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "neuron-level sparsity study on cfg%d %s; headline fields are T=%d with the feature off"
                   % (cfg.cfg, cfg.name, head["T"]), "partition": "library"},
        "neuron_sparsity": rows, "setup_s": time.time() - t_setup}))


def bench_balance(args, cfg, np, torch, binding, synth):
    """What routing skew costs, and what the bias step of Sec. 4.3 (Eq. 9) buys: forward and gate/up time of
    held-out batches with b = 0 and after `--balance-steps` bias steps on a stream of other batches."""
    dev = torch.device("cuda:0")
    t_setup = time.time()
    weights = synth.make_weights(cfg)
    src = synth.make_token_source(cfg)
    layer = binding.Layer.build(cfg, *weights, src.calibration(), on_gpu=True)
    T = args.batch or max(cfg.eval_batches)
    held = [torch.from_numpy(src.draw(7000 + i, T)).to(dev, torch.bfloat16) for i in range(4)]
    y = torch.empty_like(held[0])
    topk = torch.empty((T, cfg.top_k), dtype=torch.int32, device=dev)
    counts = torch.zeros(cfg.n_routed, dtype=torch.int32, device=dev)
    bm = 256                                      # rows of the gate/up tile at this batch size

    def measure():
        st = {"i": 0}

        def step():
            layer.forward_device(held[st["i"] % len(held)], y, None, None, None)
            st["i"] += 1
        costs = stage_costs_ms(binding, step, args.steps, True, [])
        shares, tiles, rows = [], [], []
        for x in held:
            layer.forward_device(x, y, topk, None, counts)
            torch.cuda.synchronize()
            c = counts.cpu().numpy().astype(np.int64)
            shares.append(float(c.max()) / float(c.sum()))
            tiles.append(int(np.sum((c + bm - 1) // bm)))
            rows.append(int(c.sum()))
        return {"forward_ms": costs["forward"], "gate_up_ms": costs["gate_up"], "busiest_expert_share": float(np.mean(shares)),
                "routed_row_tiles": float(np.mean(tiles)), "routed_rows_over_tile_rows": float(np.mean(rows)) / (bm * float(np.mean(tiles)))}
    layer.set_gate_params(None, np.zeros(cfg.n_routed, dtype=np.float32))
    before = measure()
    gamma, n_steps = args.gamma, args.balance_steps
    pool = [torch.from_numpy(src.draw(8000 + i, T)).to(dev, torch.bfloat16) for i in range(16)]   # the stream: 16 batches in turn
    for i in range(n_steps):
        layer.forward_device(pool[i % len(pool)], y, topk, None, counts)
        torch.cuda.synchronize()
        layer.update_bias(counts.cpu().numpy(), gamma)
        if (i + 1) % 100 == 0:
            print("bench.py: %d bias steps" % (i + 1), file=sys.stderr, flush=True)
    after = measure()
    _, b = layer.gate_params()
    print(json.dumps({
        "metric": METRIC, "value": T / (after["forward_ms"] * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "clock_ramp_ms": RAMP_MS, "ms_per_step": after["forward_ms"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "load-balancing study on cfg%d %s, T=%d; headline fields are the forward after %d bias steps of "
                   "gamma=%g on a stream of other batches" % (cfg.cfg, cfg.name, T, n_steps, gamma), "partition": "library"},
        "balance": {"before": before, "after": after, "uniform_share": 1.0 / cfg.n_routed, "bias_min": float(b.min()),
                    "bias_max": float(b.max())}, "setup_s": time.time() - t_setup}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported (the design notes say how the path would shard)." % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2502_04416_amd import binding, synth
    binding.load()
    if not torch.cuda.is_available():
        print("bench.py: no HIP device visible", file=sys.stderr)
        sys.exit(2)
    if args.sparsity:
        bench_sparsity(args, synth.CONFIGS[1 if args.config is None else args.config], np, torch, binding, synth)
        return
    if args.balance:
        bench_balance(args, synth.CONFIGS[1 if args.config is None else args.config], np, torch, binding, synth)
        return
    if args.config is None and not (args.sweep or args.batch_sweep):
        bench_all(args, np, torch, binding, synth)
        return
    cfg = synth.CONFIGS[1 if args.config is None else args.config]
    if args.batch_sweep:
        bench_batches(args, cfg, np, torch, binding, synth)
        return
    if cfg.n_outer:
        bench_hier(args, cfg, np, torch, binding, synth)
        return
    if args.sweep:
        bench_sweep(args, cfg, np, torch, binding, synth)
        return
    T = args.batch if args.batch else max(cfg.eval_batches)
    dev = torch.device("cuda:0")
    t_setup = time.time()
    weights = synth.make_weights(cfg)
    src = synth.make_token_source(cfg)
    construct_s = None
    if args.construct in ("library", "gpu"):
        t0 = time.time()
        try:
            layer = binding.Layer.build(cfg, *weights, src.calibration(), on_gpu=(args.construct == "gpu"))
            construct_s = time.time() - t0
        except binding.CmoeError as e:
            print("bench.py: cmoe_build unavailable (%s); using an arbitrary partition" % e, file=sys.stderr)
            args.construct = "arbitrary"
    if args.construct == "arbitrary":
        part = synth.trivial_partition(cfg)
        layer = binding.Layer.from_partition(cfg, *weights, part["neuron_order"], part["rep_neuron"])
    part = layer.export_partition()
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    es = 2 if cfg.dtype == "bf16" else 4
    bi = cfg.eval_batches.index(T) if T in cfg.eval_batches else 0
    x_host = src.eval_batch(bi, n=T)
    x = torch.from_numpy(x_host).to(dev, tdt)
    y = torch.empty_like(x)
    topk = torch.empty((T, cfg.top_k), dtype=torch.int32, device=dev)
    counts = torch.empty((cfg.n_routed,), dtype=torch.int32, device=dev)

    if args.copy_probe:
        # a copy of known size: 2^30 bytes read + 2^30 bytes written; scales FETCH_SIZE / WRITE_SIZE readings
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        a.copy_(b)
        torch.cuda.synchronize()
        del a, b

    # ---- headline: K steps of the MoE forward, bracketed by synchronize ----
    ms_moe = timed(lambda: layer.forward_device(x, y, topk, None, counts), args.steps, args.warmup)
    ms_dense = float("nan") if args.no_dense else timed(lambda: layer.dense_forward_device(x, y), args.steps, args.warmup)
    layer.forward_device(x, y, topk, None, counts)
    torch.cuda.synchronize()
    cnt = counts.cpu().numpy()

    # ---- spread of single forwards: 100 of them, each between its own pair of events on the launch stream
    # (the library enqueues on torch's current stream; a pair of events around nothing reads 4-5 us here, which
    # these figures contain and the headline, timed by the host clock around all steps, does not) ----
    def spread(fn, n=100):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for e0, e1 in ev:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        us = np.sort(np.array([e0.elapsed_time(e1) * 1e3 for e0, e1 in ev]))
        return {"n": n, "median": float(us[n // 2]), "p10": float(us[n // 10]), "p90": float(us[(9 * n) // 10])}
    forward_us = spread(lambda: layer.forward_device(x, y, topk, None, counts))
    dense_forward_us = None if args.no_dense else spread(lambda: layer.dense_forward_device(x, y))

    # ---- per-stage times from HIP events recorded inside the library on the launch stream ----
    def stages(dense, n):
        acc = np.zeros(5)
        for _ in range(3):
            layer.forward_timed(x, y, dense)
        for _ in range(n):
            acc += layer.forward_timed(x, y, dense)
        return acc / n
    n_prof = max(5, min(args.steps, 30))
    st_moe = stages(False, n_prof)
    st_dense = np.full(5, np.nan) if args.no_dense else stages(True, n_prof)

    # Two events around nothing still read ~4-5 us apart on this runtime; calibrate it on a null stage
    # (the dense path records the router and combine stages without launching anything there).
    ev_overhead = float("nan") if args.no_dense else float(min(st_dense[0], st_dense[4]))

    def net(ms):
        return max(ms - (0.0 if ev_overhead != ev_overhead else ev_overhead), 1e-6)

    # same-run streaming-read reference: a plain reduction over 1 GiB
    big = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    for _ in range(2):
        big.sum()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        big.sum()
    e1.record()
    torch.cuda.synchronize()
    read_ref_gbs = (1 << 30) / (e0.elapsed_time(e1) / 5 * 1e-3) / 1e9
    del big

    d, m = cfg.d_model, cfg.m
    act = cfg.n_shared + cfg.top_k
    flops_gate_up = 4.0 * d * m * act * T                     # two contractions of 2*d*m flops per active neuron-row
    flops_total = T * (6.0 * d * m * act + 4.0 * d * cfg.n_routed)
    flops_dense = T * 6.0 * d * cfg.d_ff
    union = int((cnt > 0).sum())
    w_bytes_touched = es * (3.0 * d * m * (cfg.n_shared + union) + 2.0 * d * cfg.n_routed)
    prefill = T >= 256
    if prefill:
        gu_ms = net(float(st_moe[2]))
        roofline = {"kernel": "grouped_gemm_bf16_dma<gate_up>", "bound": "mfma",
                    "achieved": flops_gate_up / (gu_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TF, "unit": "TFLOP/s",
                    "traffic": None}
    else:
        gu_ms = net(float(st_moe[2]))
        b = es * 2.0 * d * m * (union + (0 if shared_in_front(cfg, T) else cfg.n_shared))
        roofline = {"kernel": "decode_gate_up_kernel", "bound": "hbm", "achieved": b / (gu_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "traffic": None}
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    roofline["avg_launch_ms"] = gu_ms
    if prefill and cfg.cfg == 1 and T == 2048 and args.construct in ("library", "gpu"):
        # HBM bytes of one launch of this kernel on this workload from the two rocprofv3 --pmc runs
        # (FETCH_SIZE x 2.000 scale, WRITE_SIZE x 1.000; profiles/cfg1_T2048_hbm_traffic.md)
        roofline["traffic"] = MEASURED_GATE_UP_TRAFFIC_BYTES.get((1, 2048))
    # what the matrix cores sustain on register operands alone, in this process, right now
    mfma_probe = None
    if cfg.dtype == "bf16":
        tf0, mhz0 = binding.cmoe_probe_mfma(False, 16384)
        tf1, mhz1 = binding.cmoe_probe_mfma(True, 16384)
        mfma_probe = {"zero_operands_TFLOPs": tf0, "zero_operands_MHz": mhz0, "random_operands_TFLOPs": tf1,
                      "random_operands_MHz": mhz1}
        if prefill:
            roofline["frac_of_sustained_mfma"] = roofline["achieved"] / tf1
    if cfg.dtype != "bf16":
        roofline.update({"bound": "alu", "peak": FP32_VALU_PEAK_TF, "frac": roofline["achieved"] / FP32_VALU_PEAK_TF})

    out = {
        "metric": METRIC,
        "value": T / (ms_moe * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "clock_ramp_ms": RAMP_MS,
        "ms_per_step": ms_moe, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "cfg%d %s: d=%d d_ff=%d, %d experts of %d neurons, %d shared + top-%d of %d routed, T=%d tokens"
                   % (cfg.cfg, cfg.name, d, cfg.d_ff, cfg.n_experts, m, cfg.n_shared, cfg.top_k, cfg.n_routed, T),
                   "partition": args.construct, "k_act": cfg.k_act, "sigma_o": synth.SIGMA_O},
        "dense_ms_per_step": ms_dense, "dense_tokens_per_s": T / (ms_dense * 1e-3),
        "speedup_vs_dense": ms_dense / ms_moe,
        "whole_path_tflops": flops_total / (ms_moe * 1e-3) / 1e12,
        "dense_tflops": flops_dense / (ms_dense * 1e-3) / 1e12,
        "forward_us_by_events": forward_us, "dense_forward_us_by_events": dense_forward_us,
        "stage_ms": dict(zip(binding.STAGES, [float(v) for v in st_moe])),
        "dense_stage_ms": dict(zip(binding.STAGES, [float(v) for v in st_dense])),
        "expert_counts": cnt.tolist(), "experts_touched": union,
        "weight_bytes_touched": w_bytes_touched,
        "roofline": roofline,
        "construct_s": construct_s,
        "event_pair_overhead_ms": ev_overhead,
        "streaming_read_reference_GBs": read_ref_gbs,
        "mfma_probe": mfma_probe,
    }
    # what a kernel that only reads achieves on this device with 1 KB of consecutive bytes per load
    # instruction (2 GiB, beyond the last-level cache): the practical ceiling of the decode streams
    try:
        out["hbm_probe_GBs"] = binding.cmoe_probe_hbm(2 << 30, 5)
    except binding.CmoeError as e:
        print("bench.py: cmoe_probe_hbm failed (%s)" % e, file=sys.stderr)
        out["hbm_probe_GBs"] = None

    # ---- decode batches: cycle over several device copies of the layer so weights come from HBM ----
    if not args.no_decode and cfg.dtype == "bf16":
        copies = [layer]
        order, reps = part["neuron_order"], part["rep_neuron"]
        for _ in range(max(0, args.layer_copies - 1)):
            copies.append(binding.Layer.from_partition(cfg, *weights, order, reps))
        dec = []
        for Td in [b for b in cfg.eval_batches if b <= 64] or [1]:
            xs = [torch.from_numpy(src.draw(9000 + 100 * Td + i, Td)).to(dev, tdt)
                  for i in range(len(copies))]
            yd = torch.empty_like(xs[0])
            cd = torch.empty((cfg.n_routed,), dtype=torch.int32, device=dev)
            state = {"i": 0}

            def step_moe():
                i = state["i"] % len(copies)
                state["i"] += 1
                copies[i].forward_device(xs[i], yd, None, None, cd)

            def step_dense():
                i = state["i"] % len(copies)
                state["i"] += 1
                copies[i].dense_forward_device(xs[i], yd)
            steps_d = max(args.steps, 64)
            ms_m = timed(step_moe, steps_d, 16)
            ms_dn = timed(step_dense, steps_d, 16)
            # stage times and touched bytes, averaged over the copies
            st = np.zeros(5)
            std_ = np.zeros(5)
            touched = 0.0
            for i, c in enumerate(copies):
                c.forward_timed(xs[i], yd, False)
            for rep_i in range(2):
                for i, c in enumerate(copies):
                    st += c.forward_timed(xs[i], yd, False)
                    std_ += c.forward_timed(xs[i], yd, True)
                    if rep_i == 0:
                        c.forward_device(xs[i], yd, None, None, cd)
                        torch.cuda.synchronize()
                        touched += float((cd.cpu().numpy() > 0).sum())
            st /= 2 * len(copies)
            std_ /= 2 * len(copies)
            u_avg = touched / len(copies)
            bytes_moe = es * (3.0 * d * m * (cfg.n_shared + u_avg) + 2.0 * d * cfg.n_routed)
            # bytes the gate/up launch itself streams (the shared group's units may run in the launch before it)
            bytes_gu = es * 2.0 * d * m * (u_avg + (0 if shared_in_front(cfg, Td) else cfg.n_shared))
            bytes_dense = es * 3.0 * d * cfg.d_ff
            dec.append({
                "T": Td, "ms_per_step": ms_m, "tokens_per_s": Td / (ms_m * 1e-3), "dense_ms_per_step": ms_dn,
                "speedup_vs_dense": ms_dn / ms_m, "experts_touched_avg": u_avg,
                "weight_bytes_touched": bytes_moe, "shared_group_in_front_launch": shared_in_front(cfg, Td),
                "hbm_frac_whole_path": bytes_moe / (ms_m * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "dense_hbm_frac": bytes_dense / (ms_dn * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "stage_ms": dict(zip(binding.STAGES, [float(v) for v in st])),
                "dense_stage_ms": dict(zip(binding.STAGES, [float(v) for v in std_])),
                "roofline": {"kernel": "decode_gate_up_kernel", "bound": "hbm",
                             "achieved": bytes_gu / (net(st[2]) * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": bytes_gu / (net(st[2]) * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                             "avg_launch_ms": net(st[2])},
                "dense_roofline": {"kernel": "decode_gate_up_kernel (dense)", "bound": "hbm",
                                   "achieved": es * 2.0 * d * cfg.d_ff / (net(std_[2]) * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                                   "unit": "GB/s", "frac": es * 2.0 * d * cfg.d_ff / (net(std_[2]) * 1e-3) / 1e9 / HBM_PEAK_GBS},
            })
        if out.get("hbm_probe_GBs"):
            for e in dec:
                e["roofline"]["frac_of_streaming_read"] = e["roofline"]["achieved"] / out["hbm_probe_GBs"]
                e["dense_roofline"]["frac_of_streaming_read"] = e["dense_roofline"]["achieved"] / out["hbm_probe_GBs"]
        out["decode"] = dec
        out["decode_layer_copies"] = len(copies)

    # ---- CPU oracle on the host cores (reported baseline) ----
    if not args.no_cpu:
        from oracle import cmoe_oracle as O
        n_cpu = min(T, 2048)
        xs_cpu = x_host[:n_cpu]
        t0 = time.perf_counter()
        O.moe_forward(xs_cpu, *weights, part["neuron_order"], part["rep_neuron"], cfg.n_experts, cfg.n_shared, cfg.top_k)
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = {"value": n_cpu / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": "%d tokens of the same batch, fp64 numpy oracle, %.1f s" % (n_cpu, dt)}
    out["setup_s"] = time.time() - t_setup
    print(json.dumps(out))


if __name__ == "__main__":
    main()
