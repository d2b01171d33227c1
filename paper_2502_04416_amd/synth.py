"""Seeded synthetic inputs for the restructured-FFN (FFN-as-MoE) layer.

This module only *draws numbers*: layer shapes, weight matrices, clustered
token batches and the outer router of the hierarchical case.  It holds none of
the method's arithmetic (no SwiGLU, no routing, no clustering) so that both the
CPU oracle's tests and the HIP path's tests can be fed from it without sharing
any computation.  It imports numpy only.

The layers are stand-ins with the *shapes* of LLaMA-2-7B / LLaMA-3-8B /
Mixtral-8x7B FFN blocks; no trained weights or text are involved.

Recipe
------
weights   W_gate, W_up ~ N(0, 1/d) ; W_down ~ N(0, 1/d_ff)   (second argument = variance)
tokens    x_t = c_{k(t)} + o + eps_t ;  k(t) uniform over C centres, c_k ~ N(0, I),
          one offset o ~ N(0, sigma_o^2 I) per config (sigma_o = 2) shared by the
          calibration set and every eval batch, eps ~ N(0, 0.5 I)
          (config 3: Student-t, nu = 4, rescaled to variance 0.5).
seeds     weights 1000+cfg, centres/offset 2000+cfg, calibration 3000+cfg,
          eval batch 4000 + 100*cfg + batch_index.
rounding  for the bf16 configs every array is rounded once to a bf16-representable
          fp32 value (round-to-nearest-even on the bit pattern), so whatever
          rounding a consumer applies afterwards is the identity.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

SIGMA_O = 2.0
NOISE_VAR = 0.5


@dataclass(frozen=True)
class LayerConfig:
    """Shape of one restructuring problem (the paper's N, N_s, N_k, m = d_ff / N)."""

    cfg: int
    name: str
    d_model: int
    d_ff: int
    n_experts: int          # N
    n_shared: int           # N_s
    top_k: int              # N_k
    dtype: str              # "fp32" or "bf16"
    n_centres: int          # C
    n_calib: int            # q
    eval_batches: Tuple[int, ...]
    k_act: int = 10         # K_a
    noise: str = "gauss"    # "gauss" or "student4"
    # hierarchical case only
    n_outer: int = 0
    outer_top_k: int = 0

    @property
    def m(self) -> int:
        return self.d_ff // self.n_experts

    @property
    def n_routed(self) -> int:
        return self.n_experts - self.n_shared


CONFIGS: List[LayerConfig] = [
    LayerConfig(0, "tiny-fp32", 256, 1024, 8, 1, 1, "fp32", 16, 512, (64,)),
    LayerConfig(1, "llama2-7b-E16", 4096, 11008, 16, 1, 3, "bf16", 64, 2048, (1, 16, 2048)),
    LayerConfig(2, "llama2-7b-E32", 4096, 11008, 32, 2, 6, "bf16", 64, 2048, (4096, 8192)),
    LayerConfig(3, "llama3-8b-E32", 4096, 14336, 32, 4, 4, "bf16", 128, 2048, (1, 32, 4096),
                noise="student4"),
    LayerConfig(4, "mixtral-8x7b-hier", 4096, 14336, 8, 2, 2, "bf16", 64, 2048, (4096,),
                n_outer=8, outer_top_k=2),
]


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of `cfg` with some fields replaced (used for reduced-size test cases)."""
    d = {f: getattr(cfg, f) for f in cfg.__dataclass_fields__}
    d.update(kw)
    return LayerConfig(**d)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array -> nearest bf16-representable fp32 array (ties to even); finite inputs only."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    out = (bits >> np.uint32(16)) & np.uint32(1)
    out += np.uint32(0x7FFF)
    out += bits
    out &= np.uint32(0xFFFF0000)
    return out.view(np.float32).reshape(a.shape)


def _finish(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


def _normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    out = rng.standard_normal(shape, dtype=np.float32)
    out *= np.float32(std)
    return out


def make_weights(cfg: LayerConfig, seed: Optional[int] = None):
    """Dense SwiGLU weights (W_gate [d, d_ff], W_up [d, d_ff], W_down [d_ff, d]), fp32 arrays."""
    rng = np.random.Generator(np.random.PCG64(1000 + cfg.cfg if seed is None else seed))
    d, f = cfg.d_model, cfg.d_ff
    w_gate = _finish(_normal(rng, (d, f), (1.0 / d) ** 0.5), cfg.dtype)
    w_up = _finish(_normal(rng, (d, f), (1.0 / d) ** 0.5), cfg.dtype)
    w_down = _finish(_normal(rng, (f, d), (1.0 / f) ** 0.5), cfg.dtype)
    return w_gate, w_up, w_down


@dataclass
class TokenSource:
    """Cluster centres and the shared offset of one config; draws calibration/eval batches."""

    cfg: LayerConfig
    centres: np.ndarray = field(repr=False)
    offset: np.ndarray = field(repr=False)

    def _draw(self, seed: int, n: int) -> np.ndarray:
        rng = np.random.Generator(np.random.PCG64(seed))
        d = self.cfg.d_model
        k = rng.integers(0, self.centres.shape[0], size=n)
        if self.cfg.noise == "student4":
            # t_4 has variance 2; scale so the noise variance is NOISE_VAR
            eps = rng.standard_t(4.0, size=(n, d)).astype(np.float32) * np.float32((NOISE_VAR / 2.0) ** 0.5)
        else:
            eps = _normal(rng, (n, d), NOISE_VAR ** 0.5)
        x = self.centres[k] + self.offset[None, :] + eps
        return _finish(x, self.cfg.dtype)

    def draw(self, seed: int, n: int) -> np.ndarray:
        """n tokens from this source with an explicit seed (extra batches for timing loops)."""
        return self._draw(seed, n)

    def calibration(self, n: Optional[int] = None) -> np.ndarray:
        return self._draw(3000 + self.cfg.cfg, self.cfg.n_calib if n is None else n)

    def eval_batch(self, batch_index: int, n: Optional[int] = None) -> np.ndarray:
        n = self.cfg.eval_batches[batch_index] if n is None else n
        return self._draw(4000 + 100 * self.cfg.cfg + batch_index, n)


def make_token_source(cfg: LayerConfig, seed: Optional[int] = None) -> TokenSource:
    rng = np.random.Generator(np.random.PCG64(2000 + cfg.cfg if seed is None else seed))
    centres = _normal(rng, (cfg.n_centres, cfg.d_model), 1.0)
    offset = _normal(rng, (cfg.d_model,), SIGMA_O)
    return TokenSource(cfg, centres, offset)


def make_outer_router(cfg: LayerConfig, seed: Optional[int] = None):
    """Outer router of the hierarchical case: W_router [d, n_outer] ~ N(0, 1/d) and the
    Zipf(1.1) logit offsets -1.1 * ln(rank), rank = 1..n_outer."""
    assert cfg.n_outer > 0
    rng = np.random.Generator(np.random.PCG64(5000 + cfg.cfg if seed is None else seed))
    w_router = _finish(_normal(rng, (cfg.d_model, cfg.n_outer), (1.0 / cfg.d_model) ** 0.5), cfg.dtype)
    offsets = (-1.1 * np.log(np.arange(1, cfg.n_outer + 1, dtype=np.float64))).astype(np.float32)
    return w_router, offsets


def make_outer_expert_weights(cfg: LayerConfig, e: int):
    """Dense weights of outer expert `e` in the hierarchical case (independent seeds per expert)."""
    return make_weights(cfg, seed=1000 + cfg.cfg + 97 * (e + 1))


def make_gate_params(cfg: LayerConfig, seed: int = 7000) -> Tuple[np.ndarray, np.ndarray]:
    """A non-trivial (u, b): u ~ U(-0.5, 0.5), b ~ N(0, 1e-3 as std) per routed expert, fp32."""
    rng = np.random.Generator(np.random.PCG64(seed + cfg.cfg))
    u = rng.uniform(-0.5, 0.5, size=cfg.n_routed).astype(np.float32)
    b = (rng.standard_normal(cfg.n_routed) * 1e-3).astype(np.float32)
    return u, b


def trivial_partition(cfg: LayerConfig, seed: int = 0) -> Dict[str, np.ndarray]:
    """A seeded *arbitrary* partition (random neuron order, first neuron of each routed
    expert as its representative).  Not the paper's construction: it only exercises a
    forward pass with a known neuron-to-expert layout."""
    rng = np.random.Generator(np.random.PCG64(6000 + cfg.cfg + seed))
    order = rng.permutation(cfg.d_ff).astype(np.int32)
    m = cfg.m
    reps = np.array([order[(cfg.n_shared + j) * m] for j in range(cfg.n_routed)], dtype=np.int32)
    return {"neuron_order": order, "rep_neuron": reps}
