"""ctypes binding of libcmoe.so (the C ABI declared in include/cmoe.h).

Argument marshalling only: every step of the forward pass runs in the library's HIP kernels.
PyTorch supplies device memory (torch.empty on cuda) and the current HIP stream, nothing else.
There is no CPU fallback: if the library is missing, or was not built, every call raises.

The module-level functions carry the C names (cmoe_build, cmoe_forward, ...) and take/return raw
handles; `Layer` and `Hierarchy` wrap them for the tests and the bench.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcmoe.so")
_lib = None

CMOE_F32, CMOE_BF16 = 0, 1


class CmoeError(RuntimeError):
    pass


class cmoe_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "d_model", "d_ff", "n_experts", "n_shared", "top_k", "k_act", "kmeans_iters", "dtype",
        "dist_mode", "score_mode")]


EXPORTS = [
    "cmoe_build", "cmoe_build_from_partition", "cmoe_export_partition", "cmoe_set_gate_params",
    "cmoe_packed_bytes", "cmoe_workspace_bytes", "cmoe_upload", "cmoe_forward", "cmoe_dense_forward",
    "cmoe_destroy", "cmoe_hier_create", "cmoe_hier_packed_bytes", "cmoe_hier_workspace_bytes",
    "cmoe_hier_upload", "cmoe_hier_forward", "cmoe_hier_dense_forward", "cmoe_hier_destroy",
    "cmoe_last_error", "cmoe_version", "cmoe_forward_timed", "cmoe_hier_forward_timed",
    "cmoe_balanced_assignment", "cmoe_probe_mfma", "cmoe_probe_hbm", "cmoe_get_gate_params", "cmoe_update_bias",
    "cmoe_build_gpu", "cmoe_profile_activations", "cmoe_set_baseline", "cmoe_hier_build", "cmoe_hier_expert",
    "cmoe_set_tuning", "cmoe_set_neuron_sparsity", "cmoe_forward_static", "cmoe_static_scratch_bytes", "cmoe_forward_static_max_tokens",
]


def load():
    """Load libcmoe.so (built by __graft_entry__.build()).  Raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise CmoeError("libcmoe.so is not built (%s missing): run `python __graft_entry__.py`; "
                        "there is no fallback path" % LIB_PATH)
    # torch first: its bundled HIP runtime must be the one already in the process when libcmoe.so
    # resolves libamdhip64, so that both share one runtime (device pointers and streams come from torch)
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32p, f32p, i64, sz = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_int64, C.c_size_t
    cfgp = C.POINTER(cmoe_config)
    lib.cmoe_build.argtypes = [cfgp, f32p, f32p, f32p, f32p, i64, C.POINTER(vp)]
    lib.cmoe_build_gpu.argtypes = [cfgp, f32p, f32p, f32p, f32p, i64, C.POINTER(vp)]
    lib.cmoe_profile_activations.argtypes = [cfgp, f32p, f32p, f32p, i64, C.c_int, i32p]
    lib.cmoe_build_from_partition.argtypes = [cfgp, f32p, f32p, f32p, i32p, i32p, C.POINTER(vp)]
    lib.cmoe_balanced_assignment.argtypes = [C.POINTER(C.c_double), C.c_int32, C.c_int32, C.c_int32, i32p,
                                             C.POINTER(C.c_double)]
    lib.cmoe_export_partition.argtypes = [vp, i32p, i32p, f32p, C.POINTER(C.c_double)]
    lib.cmoe_set_gate_params.argtypes = [vp, f32p, f32p]
    lib.cmoe_get_gate_params.argtypes = [vp, f32p, f32p]
    lib.cmoe_update_bias.argtypes = [vp, i32p, C.c_float]
    lib.cmoe_packed_bytes.argtypes = [vp]
    lib.cmoe_packed_bytes.restype = sz
    lib.cmoe_workspace_bytes.argtypes = [vp, i64]
    lib.cmoe_workspace_bytes.restype = sz
    lib.cmoe_upload.argtypes = [vp, vp, vp]
    lib.cmoe_forward.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.cmoe_dense_forward.argtypes = [vp, vp, i64, vp, vp, sz, vp]
    lib.cmoe_forward_timed.argtypes = [vp, C.c_int, vp, i64, vp, vp, sz, vp, f32p]
    lib.cmoe_hier_forward_timed.argtypes = [vp, C.c_int, vp, i64, vp, vp, sz, vp, f32p]
    lib.cmoe_destroy.argtypes = [vp]
    lib.cmoe_destroy.restype = None
    lib.cmoe_hier_create.argtypes = [C.POINTER(vp), C.c_int32, C.c_int32, f32p, f32p, C.POINTER(vp)]
    lib.cmoe_hier_packed_bytes.argtypes = [vp]
    lib.cmoe_hier_packed_bytes.restype = sz
    lib.cmoe_hier_workspace_bytes.argtypes = [vp, i64]
    lib.cmoe_hier_workspace_bytes.restype = sz
    lib.cmoe_hier_upload.argtypes = [vp, vp, vp]
    lib.cmoe_hier_forward.argtypes = [vp, vp, i64, vp, vp, vp, vp, sz, vp]
    lib.cmoe_hier_dense_forward.argtypes = [vp, vp, i64, vp, vp, sz, vp]
    lib.cmoe_hier_destroy.argtypes = [vp]
    lib.cmoe_hier_destroy.restype = None
    lib.cmoe_probe_mfma.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.cmoe_probe_hbm.argtypes = [C.c_size_t, C.c_int, C.POINTER(C.c_double)]
    lib.cmoe_set_baseline.argtypes = [vp, C.c_int]
    fpp = C.POINTER(f32p)
    lib.cmoe_hier_build.argtypes = [cfgp, C.c_int32, C.c_int32, fpp, fpp, fpp, f32p, f32p, f32p, i64, C.c_int32, C.c_int,
                                    C.c_int, C.POINTER(vp)]
    lib.cmoe_hier_expert.argtypes = [vp, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.cmoe_hier_expert.restype = vp
    lib.cmoe_set_tuning.argtypes = [C.c_char_p, C.c_int]
    lib.cmoe_set_neuron_sparsity.argtypes = [vp, C.c_int, C.c_float]
    lib.cmoe_forward_static.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp]
    lib.cmoe_static_scratch_bytes.argtypes = []
    lib.cmoe_static_scratch_bytes.restype = sz
    lib.cmoe_forward_static_max_tokens.argtypes = [vp]
    lib.cmoe_forward_static_max_tokens.restype = i64
    lib.cmoe_last_error.restype = C.c_char_p
    lib.cmoe_version.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        raise CmoeError("%s failed (%d): %s" % (what, rc, load().cmoe_last_error().decode()))


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _fp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_float))


def _ip(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_int32))


def make_config(cfg, kmeans_iters: int = 1, dist_mode: int = 0, score_mode: int = 0) -> cmoe_config:
    """cmoe_config from a synth.LayerConfig-like object (d_model, d_ff, n_experts, n_shared, top_k, k_act, dtype)."""
    return cmoe_config(cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.n_shared, cfg.top_k, cfg.k_act, kmeans_iters,
                       CMOE_BF16 if cfg.dtype == "bf16" else CMOE_F32, dist_mode, score_mode)


# ---- C names ------------------------------------------------------------------------------------

def cmoe_build(cfg: cmoe_config, w_gate, w_up, w_down, calib_x) -> int:
    wg, wu, wd, cx = _f32(w_gate), _f32(w_up), _f32(w_down), _f32(calib_x)
    h = C.c_void_p()
    _check(load().cmoe_build(C.byref(cfg), _fp(wg), _fp(wu), _fp(wd), _fp(cx), cx.shape[0], C.byref(h)), "cmoe_build")
    return h.value


def cmoe_build_gpu(cfg: cmoe_config, w_gate, w_up, w_down, calib_x) -> int:
    wg, wu, wd, cx = _f32(w_gate), _f32(w_up), _f32(w_down), _f32(calib_x)
    h = C.c_void_p()
    _check(load().cmoe_build_gpu(C.byref(cfg), _fp(wg), _fp(wu), _fp(wd), _fp(cx), cx.shape[0], C.byref(h)),
           "cmoe_build_gpu")
    return h.value


def cmoe_profile_activations(cfg: cmoe_config, w_gate, w_up, calib_x, on_gpu: bool) -> np.ndarray:
    """active [q, k_act]: per calibration token the k_act neurons of largest |h| (App. A.2 steps 1-2)."""
    wg, wu, cx = _f32(w_gate), _f32(w_up), _f32(calib_x)
    out = np.empty((cx.shape[0], cfg.k_act), dtype=np.int32)
    _check(load().cmoe_profile_activations(C.byref(cfg), _fp(wg), _fp(wu), _fp(cx), cx.shape[0], int(on_gpu), _ip(out)),
           "cmoe_profile_activations")
    return out


def cmoe_build_from_partition(cfg: cmoe_config, w_gate, w_up, w_down, neuron_order, rep_neuron) -> int:
    wg, wu, wd = _f32(w_gate), _f32(w_up), _f32(w_down)
    no, rn = _i32(neuron_order), _i32(rep_neuron)
    h = C.c_void_p()
    _check(load().cmoe_build_from_partition(C.byref(cfg), _fp(wg), _fp(wu), _fp(wd), _ip(no), _ip(rn), C.byref(h)),
           "cmoe_build_from_partition")
    return h.value


def cmoe_balanced_assignment(dist: np.ndarray, m: int):
    """(label [n], cost) of the exact balanced assignment of App. A.3 for dist [n, n_r], n = n_r * m."""
    dd = np.ascontiguousarray(dist, dtype=np.float64)
    n, n_r = dd.shape
    label = np.empty(n, dtype=np.int32)
    cost = C.c_double()
    _check(load().cmoe_balanced_assignment(dd.ctypes.data_as(C.POINTER(C.c_double)), n, n_r, m, _ip(label),
                                           C.byref(cost)), "cmoe_balanced_assignment")
    return label, cost.value


def cmoe_probe_mfma(random_operands: bool, iters: int):
    """(TFLOP/s, shader MHz) the matrix cores sustain on register operands alone (measurement aid)."""
    tf, mhz = C.c_double(), C.c_double()
    _check(load().cmoe_probe_mfma(int(random_operands), int(iters), C.byref(tf), C.byref(mhz)), "cmoe_probe_mfma")
    return tf.value, mhz.value


def cmoe_probe_hbm(n_bytes: int, reps: int = 5) -> float:
    """GB/s of a plain streaming read of n_bytes of device memory (measurement aid)."""
    g = C.c_double()
    _check(load().cmoe_probe_hbm(int(n_bytes), int(reps), C.byref(g)), "cmoe_probe_hbm")
    return g.value


def cmoe_export_partition(layer: int, d_ff: int, n_routed: int) -> Dict[str, np.ndarray]:
    order = np.empty(d_ff, dtype=np.int32)
    reps = np.empty(n_routed, dtype=np.int32)
    mu = np.empty(d_ff, dtype=np.float32)
    cost = C.c_double()
    _check(load().cmoe_export_partition(layer, _ip(order), _ip(reps), _fp(mu), C.byref(cost)), "cmoe_export_partition")
    return {"neuron_order": order, "rep_neuron": reps, "mu": mu, "cost": cost.value}


def cmoe_set_gate_params(layer: int, u, b) -> None:
    uu = None if u is None else _f32(u)
    bb = None if b is None else _f32(b)
    _check(load().cmoe_set_gate_params(layer, _fp(uu), _fp(bb)), "cmoe_set_gate_params")


def cmoe_get_gate_params(layer: int, n_routed: int):
    u = np.empty(n_routed, dtype=np.float32)
    b = np.empty(n_routed, dtype=np.float32)
    _check(load().cmoe_get_gate_params(layer, _fp(u), _fp(b)), "cmoe_get_gate_params")
    return u, b


def cmoe_update_bias(layer: int, counts, gamma: float = 1e-3) -> None:
    c = np.ascontiguousarray(counts, dtype=np.int32)
    _check(load().cmoe_update_bias(layer, _ip(c), float(gamma)), "cmoe_update_bias")


def cmoe_packed_bytes(layer: int) -> int:
    return load().cmoe_packed_bytes(layer)


def cmoe_workspace_bytes(layer: int, max_tokens: int) -> int:
    return load().cmoe_workspace_bytes(layer, max_tokens)


def cmoe_upload(layer: int, dev_weights_ptr: int, stream: int = 0) -> None:
    _check(load().cmoe_upload(layer, dev_weights_ptr, stream), "cmoe_upload")


def cmoe_forward(layer: int, x_ptr: int, T: int, y_ptr: int, topk_ptr, scores_ptr, counts_ptr, ws_ptr: int,
                 ws_bytes: int, stream: int = 0) -> None:
    _check(load().cmoe_forward(layer, x_ptr, T, y_ptr, topk_ptr, scores_ptr, counts_ptr, ws_ptr, ws_bytes, stream),
           "cmoe_forward")


def cmoe_forward_static(layer: int, x_ptr: int, T: int, y_ptr: int, topk_ptr, scores_ptr, counts_ptr, stream: int = 0) -> None:
    _check(load().cmoe_forward_static(layer, x_ptr, T, y_ptr, topk_ptr, scores_ptr, counts_ptr, stream), "cmoe_forward_static")


def cmoe_static_scratch_bytes() -> int:
    return load().cmoe_static_scratch_bytes()


def cmoe_forward_static_max_tokens(layer: int) -> int:
    return load().cmoe_forward_static_max_tokens(layer)


def cmoe_dense_forward(layer: int, x_ptr: int, T: int, y_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(load().cmoe_dense_forward(layer, x_ptr, T, y_ptr, ws_ptr, ws_bytes, stream), "cmoe_dense_forward")


STAGES = ("router", "permute", "gate_up", "down", "combine")


def cmoe_forward_timed(layer: int, dense: int, x_ptr: int, T: int, y_ptr: int, ws_ptr: int, ws_bytes: int,
                       stream: int = 0) -> np.ndarray:
    ms = np.zeros(5, dtype=np.float32)
    _check(load().cmoe_forward_timed(layer, dense, x_ptr, T, y_ptr, ws_ptr, ws_bytes, stream, _fp(ms)), "cmoe_forward_timed")
    return ms


def cmoe_hier_forward_timed(h: int, dense: int, x_ptr: int, T: int, y_ptr: int, ws_ptr: int, ws_bytes: int,
                            stream: int = 0) -> np.ndarray:
    ms = np.zeros(5, dtype=np.float32)
    _check(load().cmoe_hier_forward_timed(h, dense, x_ptr, T, y_ptr, ws_ptr, ws_bytes, stream, _fp(ms)),
           "cmoe_hier_forward_timed")
    return ms


def cmoe_destroy(layer: int) -> None:
    load().cmoe_destroy(layer)


def cmoe_hier_create(layers: Sequence[int], outer_top_k: int, w_router, logit_offset) -> int:
    arr = (C.c_void_p * len(layers))(*layers)
    wr = _f32(w_router)
    off = None if logit_offset is None else _f32(logit_offset)
    h = C.c_void_p()
    _check(load().cmoe_hier_create(arr, len(layers), outer_top_k, _fp(wr), _fp(off), C.byref(h)), "cmoe_hier_create")
    return h.value


def cmoe_hier_build(cfg: cmoe_config, outer_top_k: int, w_gate: Sequence, w_up: Sequence, w_down: Sequence, w_router,
                    logit_offset, calib_x, min_tokens: int = 64, on_gpu: bool = False, with_baseline: bool = True) -> int:
    n = len(w_gate)
    wg, wu, wd = [_f32(a) for a in w_gate], [_f32(a) for a in w_up], [_f32(a) for a in w_down]
    fpp = C.POINTER(C.c_float) * n
    wr, cx = _f32(w_router), _f32(calib_x)
    off = None if logit_offset is None else _f32(logit_offset)
    h = C.c_void_p()
    _check(load().cmoe_hier_build(C.byref(cfg), n, outer_top_k, fpp(*[_fp(a) for a in wg]), fpp(*[_fp(a) for a in wu]),
                                  fpp(*[_fp(a) for a in wd]), _fp(wr), _fp(off), _fp(cx), cx.shape[0], int(min_tokens),
                                  int(on_gpu), int(with_baseline), C.byref(h)), "cmoe_hier_build")
    return h.value


def cmoe_hier_expert(h: int, e: int):
    """(borrowed layer handle, calibration tokens routed to the expert, calibration tokens it was built on)."""
    routed, used = C.c_int64(), C.c_int64()
    layer = load().cmoe_hier_expert(h, e, C.byref(routed), C.byref(used))
    if not layer:
        raise CmoeError("cmoe_hier_expert failed: %s" % load().cmoe_last_error().decode())
    return layer, routed.value, used.value


def cmoe_set_baseline(layer: int, enabled: bool) -> None:
    _check(load().cmoe_set_baseline(layer, int(enabled)), "cmoe_set_baseline")


def cmoe_set_neuron_sparsity(layer: int, mode: int, tau: float) -> None:
    _check(load().cmoe_set_neuron_sparsity(layer, int(mode), float(tau)), "cmoe_set_neuron_sparsity")


def cmoe_set_tuning(name: str, value: int) -> None:
    _check(load().cmoe_set_tuning(name.encode(), int(value)), "cmoe_set_tuning")


def cmoe_hier_packed_bytes(h: int) -> int:
    return load().cmoe_hier_packed_bytes(h)


def cmoe_hier_workspace_bytes(h: int, max_tokens: int) -> int:
    return load().cmoe_hier_workspace_bytes(h, max_tokens)


def cmoe_hier_upload(h: int, dev_ptr: int, stream: int = 0) -> None:
    _check(load().cmoe_hier_upload(h, dev_ptr, stream), "cmoe_hier_upload")


def cmoe_hier_forward(h: int, x_ptr: int, T: int, y_ptr: int, outer_ptr, sub_ptr, ws_ptr: int, ws_bytes: int,
                      stream: int = 0) -> None:
    _check(load().cmoe_hier_forward(h, x_ptr, T, y_ptr, outer_ptr, sub_ptr, ws_ptr, ws_bytes, stream), "cmoe_hier_forward")


def cmoe_hier_dense_forward(h: int, x_ptr: int, T: int, y_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(load().cmoe_hier_dense_forward(h, x_ptr, T, y_ptr, ws_ptr, ws_bytes, stream), "cmoe_hier_dense_forward")


def cmoe_hier_destroy(h: int) -> None:
    load().cmoe_hier_destroy(h)


def cmoe_version() -> str:
    return load().cmoe_version().decode()


# ---- conveniences for tests and the bench ----------------------------------------------------------

def _torch():
    import torch
    if not torch.cuda.is_available():
        raise CmoeError("no HIP device: the forward pass runs only on the GPU (there is no CPU path)")
    return torch


def _stream_ptr(torch) -> int:
    return int(torch.cuda.current_stream().cuda_stream)


class _DeviceMixin:
    """Device buffers (allocated through torch) shared by Layer and Hierarchy."""

    def _alloc(self, nbytes: int):
        torch = _torch()
        return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")

    def _to_device(self, x):
        torch = _torch()
        if isinstance(x, np.ndarray):
            x = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
        x = x.to(device="cuda", dtype=torch.bfloat16 if self.bf16 else torch.float32).contiguous()
        return x

    def _ensure_ws(self, T: int):
        if T > self._ws_tokens:
            self._ws = None
            self._ws = self._alloc(self._ws_bytes(T))
            self._ws_tokens = T
        return self._ws


class Layer(_DeviceMixin):
    """One restructured FFN on the GPU."""

    def __init__(self, handle: int, cfg):
        self.h = handle
        self.cfg = cfg
        self.bf16 = cfg.dtype == "bf16"
        self._weights = None
        self._ws = None
        self._ws_tokens = -1

    @classmethod
    def from_partition(cls, cfg, w_gate, w_up, w_down, neuron_order, rep_neuron, score_mode: int = 0, upload=True,
                       baseline=True, neuron_sparsity=None):
        """neuron_sparsity: (mode, tau) handed to cmoe_set_neuron_sparsity before the upload."""
        h = cmoe_build_from_partition(make_config(cfg, score_mode=score_mode), w_gate, w_up, w_down, neuron_order, rep_neuron)
        self = cls(h, cfg)
        if not baseline:
            cmoe_set_baseline(h, False)
        if neuron_sparsity is not None:
            cmoe_set_neuron_sparsity(h, *neuron_sparsity)
        if upload:
            self.upload()
        return self

    @classmethod
    def build(cls, cfg, w_gate, w_up, w_down, calib_x, kmeans_iters=1, dist_mode=0, upload=True, on_gpu=False):
        make = cmoe_build_gpu if on_gpu else cmoe_build
        h = make(make_config(cfg, kmeans_iters, dist_mode), w_gate, w_up, w_down, calib_x)
        self = cls(h, cfg)
        if upload:
            self.upload()
        return self

    def upload(self):
        torch = _torch()
        self._weights = self._alloc(cmoe_packed_bytes(self.h))
        cmoe_upload(self.h, self._weights.data_ptr(), _stream_ptr(torch))

    def _ws_bytes(self, T):
        return cmoe_workspace_bytes(self.h, T)

    def export_partition(self):
        return cmoe_export_partition(self.h, self.cfg.d_ff, self.cfg.n_routed)

    def set_gate_params(self, u, b):
        cmoe_set_gate_params(self.h, u, b)

    def set_neuron_sparsity(self, mode: int, tau: float):
        cmoe_set_neuron_sparsity(self.h, mode, tau)

    def gate_params(self):
        """(u, b) as currently stored in the layer."""
        return cmoe_get_gate_params(self.h, self.cfg.n_routed)

    def update_bias(self, counts, gamma: float = 1e-3):
        """One load-balancing step of Sec. 4.3 from the per-expert token counts of a forward."""
        cmoe_update_bias(self.h, counts, gamma)

    def forward_device(self, x_dev, y_dev, topk=None, scores=None, counts=None):
        """x_dev, y_dev: torch cuda tensors [T, d] in the layer dtype; enqueues only."""
        torch = _torch()
        T = x_dev.shape[0]
        ws = self._ensure_ws(T)
        cmoe_forward(self.h, x_dev.data_ptr(), T, y_dev.data_ptr(),
                     None if topk is None else topk.data_ptr(), None if scores is None else scores.data_ptr(),
                     None if counts is None else counts.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(torch))

    def dense_forward_device(self, x_dev, y_dev):
        torch = _torch()
        T = x_dev.shape[0]
        ws = self._ensure_ws(T)
        cmoe_dense_forward(self.h, x_dev.data_ptr(), T, y_dev.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(torch))

    def forward_timed(self, x_dev, y_dev, dense: bool = False) -> np.ndarray:
        """Per-stage milliseconds of one forward (see binding.STAGES); synchronises."""
        torch = _torch()
        T = x_dev.shape[0]
        ws = self._ensure_ws(T)
        return cmoe_forward_timed(self.h, int(dense), x_dev.data_ptr(), T, y_dev.data_ptr(), ws.data_ptr(), ws.numel(),
                                  _stream_ptr(torch))

    def forward(self, x) -> Dict[str, np.ndarray]:
        torch = _torch()
        xd = self._to_device(x)
        T = xd.shape[0]
        c = self.cfg
        y = torch.empty_like(xd)
        topk = torch.full((max(T, 1), c.top_k), -1, dtype=torch.int32, device="cuda")
        scores = torch.zeros((max(T, 1), c.n_routed), dtype=torch.float32, device="cuda")
        counts = torch.zeros((c.n_routed,), dtype=torch.int32, device="cuda")
        self.forward_device(xd, y, topk, scores, counts)
        torch.cuda.synchronize()
        return {"y": y.float().cpu().numpy().astype(np.float64), "topk": topk.cpu().numpy()[:T].astype(np.int64),
                "scores": scores.cpu().numpy()[:T].astype(np.float64), "counts": counts.cpu().numpy()}

    def dense_forward(self, x) -> np.ndarray:
        torch = _torch()
        xd = self._to_device(x)
        y = torch.empty_like(xd)
        self.dense_forward_device(xd, y)
        torch.cuda.synchronize()
        return y.float().cpu().numpy().astype(np.float64)

    def close(self):
        if self.h:
            cmoe_destroy(self.h)
            self.h = None
        self._weights = None
        self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Hierarchy(_DeviceMixin):
    """An MoE layer whose experts were each restructured (Sec. 4.4)."""

    def __init__(self, layers: Sequence[Layer], outer_top_k: int, w_router, logit_offset, handle=None, cfg=None):
        self.layers = list(layers)
        self.cfg = layers[0].cfg if cfg is None else cfg
        self.bf16 = self.cfg.dtype == "bf16"
        self.outer_top_k = outer_top_k
        self.h = handle if handle is not None else cmoe_hier_create([l.h for l in layers], outer_top_k, w_router, logit_offset)
        torch = _torch()
        self._weights = self._alloc(cmoe_hier_packed_bytes(self.h))
        cmoe_hier_upload(self.h, self._weights.data_ptr(), _stream_ptr(torch))
        self._ws = None
        self._ws_tokens = -1

    @classmethod
    def build(cls, cfg, outer_top_k: int, w_gate, w_up, w_down, w_router, logit_offset, calib_x, kmeans_iters=1,
              dist_mode=0, score_mode=0, min_tokens=64, on_gpu=False, with_baseline=True):
        """cmoe_hier_build: the library routes the calibration tokens and restructures every outer expert."""
        h = cmoe_hier_build(make_config(cfg, kmeans_iters, dist_mode, score_mode), outer_top_k, w_gate, w_up, w_down,
                            w_router, logit_offset, calib_x, min_tokens, on_gpu, with_baseline)
        return cls([], outer_top_k, None, None, handle=h, cfg=cfg)

    def expert_partition(self, e: int):
        """Partition of outer expert e plus the calibration-token counts of cmoe_hier_build."""
        layer, routed, used = cmoe_hier_expert(self.h, e)
        part = cmoe_export_partition(layer, self.cfg.d_ff, self.cfg.n_routed)
        part["calib_routed"], part["calib_used"] = routed, used
        return part

    def _ws_bytes(self, T):
        return cmoe_hier_workspace_bytes(self.h, T)

    def forward_device(self, x_dev, y_dev, outer=None, sub=None):
        torch = _torch()
        T = x_dev.shape[0]
        ws = self._ensure_ws(T)
        cmoe_hier_forward(self.h, x_dev.data_ptr(), T, y_dev.data_ptr(), None if outer is None else outer.data_ptr(),
                          None if sub is None else sub.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(torch))

    def dense_forward_device(self, x_dev, y_dev):
        torch = _torch()
        T = x_dev.shape[0]
        ws = self._ensure_ws(T)
        cmoe_hier_dense_forward(self.h, x_dev.data_ptr(), T, y_dev.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(torch))

    def forward_timed(self, x_dev, y_dev, dense: bool = False) -> np.ndarray:
        torch = _torch()
        T = x_dev.shape[0]
        ws = self._ensure_ws(T)
        return cmoe_hier_forward_timed(self.h, int(dense), x_dev.data_ptr(), T, y_dev.data_ptr(), ws.data_ptr(),
                                       ws.numel(), _stream_ptr(torch))

    def forward(self, x) -> Dict[str, np.ndarray]:
        torch = _torch()
        xd = self._to_device(x)
        T = xd.shape[0]
        y = torch.empty_like(xd)
        outer = torch.full((T, self.outer_top_k), -1, dtype=torch.int32, device="cuda")
        sub = torch.full((T, self.outer_top_k, self.cfg.top_k), -1, dtype=torch.int32, device="cuda")
        self.forward_device(xd, y, outer, sub)
        torch.cuda.synchronize()
        return {"y": y.float().cpu().numpy().astype(np.float64), "outer": outer.cpu().numpy().astype(np.int64),
                "sub": sub.cpu().numpy().astype(np.int64)}

    def dense_forward(self, x) -> np.ndarray:
        torch = _torch()
        xd = self._to_device(x)
        y = torch.empty_like(xd)
        self.dense_forward_device(xd, y)
        torch.cuda.synchronize()
        return y.float().cpu().numpy().astype(np.float64)

    def close(self):
        if self.h:
            cmoe_hier_destroy(self.h)
            self.h = None
        for l in self.layers:
            l.close()
        self._weights = None
        self._ws = None
