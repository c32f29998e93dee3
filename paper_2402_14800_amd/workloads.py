"""Seeded synthetic inputs for the MoE-layer workloads.

This module only draws random tensors of the stated shapes and distributions
and rounds them once to their storage dtype.  It holds none of the method's
arithmetic and imports neither the GPU binding nor the CPU oracle, so both can
be fed from it.

Recipe.  seed = 20240214 + 1000 * config index.  One independent sub-stream per
tensor, in the fixed order x, Wgate, W1, W3, W2, bias.  Values are drawn in fp32
(fp64 draws cast to fp32 for the numpy backend) and rounded once to the storage
dtype; the rounded arrays are the inputs for every consumer.
  * backend "numpy": numpy PCG64 streams spawned from SeedSequence(seed); the
    result lives on the host (and may then be copied to a device).  Row-major
    fill, so a smaller T is a prefix of a larger one.
  * backend "torch": torch.Generator on the target device seeded with seed + i
    for tensor i; used for the layers that are too large to draw on the host.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np
import torch

BASE_SEED = 20240214


@dataclass(frozen=True)
class LayerConfig:
    name: str
    index: int            # position in the benchmark's config list (sets the seed)
    dtype: str            # "f32" or "bf16": storage type of x, weights, Y, out
    E: int                # experts
    k: int                # experts per token
    H: int                # hidden size
    F: int                # SwiGLU ffn size
    T: int                # tokens
    rs: Tuple[int, ...]   # kept-expert counts to enumerate
    rms_norm: bool = False        # x rows scaled to unit RMS before rounding
    gate_bias_var: float = 0.0    # variance of a per-expert bias added to the logits

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 * self.index

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def with_tokens(self, T: int) -> "LayerConfig":
        return replace(self, T=T)


CONFIGS = {
    "C1": LayerConfig("C1-tiny-f32", 0, "f32", E=4, k=2, H=64, F=128, T=512, rs=(2,)),
    "C2": LayerConfig("C2-mid-bf16", 1, "bf16", E=8, k=2, H=1024, F=3584, T=16384, rs=(6, 4)),
    "C3": LayerConfig("C3-mixtral-bf16", 2, "bf16", E=8, k=2, H=4096, F=14336, T=262144,
                      rs=(6, 4), rms_norm=True),
    "C4": LayerConfig("C4-stress-bf16", 3, "bf16", E=16, k=4, H=2048, F=5632, T=65536,
                      rs=(8, 12), gate_bias_var=0.5),
    "C5": LayerConfig("C5-skip-bf16", 4, "bf16", E=8, k=2, H=4096, F=14336, T=32768,
                      rs=(), rms_norm=True),
}

_TENSOR_ORDER = ("x", "Wgate", "W1", "W3", "W2", "bias")


def _shapes(cfg: LayerConfig):
    return {
        "x": ((cfg.T, cfg.H), 1.0),
        "Wgate": ((cfg.E, cfg.H), cfg.H ** -0.5),
        "W1": ((cfg.E, cfg.F, cfg.H), cfg.H ** -0.5),
        "W3": ((cfg.E, cfg.F, cfg.H), cfg.H ** -0.5),
        "W2": ((cfg.E, cfg.H, cfg.F), cfg.F ** -0.5),
        "bias": ((cfg.E,), cfg.gate_bias_var ** 0.5),
    }


def _unit_rms_rows(x: torch.Tensor) -> torch.Tensor:
    return x / x.pow(2).mean(dim=1, keepdim=True).sqrt()


def make_layer(cfg: LayerConfig, device="cpu", backend: Optional[str] = None):
    """Draw the layer's tensors.  Returns a dict with x, Wgate, W1, W3, W2 in the
    storage dtype, `bias` (fp32 [E], or None when the config has none) and `backend`."""
    device = torch.device(device)
    if backend is None:
        backend = "numpy" if device.type == "cpu" else "torch"
    shapes = _shapes(cfg)
    out = {"backend": backend}
    if backend == "numpy":
        streams = np.random.SeedSequence(cfg.seed).spawn(len(_TENSOR_ORDER))
    for i, name in enumerate(_TENSOR_ORDER):
        shape, std = shapes[name]
        if name == "bias" and cfg.gate_bias_var == 0.0:
            out[name] = None
            continue
        if backend == "numpy":
            rng = np.random.Generator(np.random.PCG64(streams[i]))
            t = torch.from_numpy(rng.standard_normal(shape).astype(np.float32)).to(device)
        elif backend == "torch":
            gen = torch.Generator(device=device)
            gen.manual_seed(cfg.seed + i)
            t = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
        else:
            raise ValueError(f"unknown backend {backend!r}")
        if name == "x" and cfg.rms_norm:
            t = _unit_rms_rows(t)
        elif std != 1.0:
            t = t * std
        out[name] = t if name == "bias" else t.to(cfg.torch_dtype)
    return out


def make_enumeration_inputs(E: int, T: int, H: int, dtype: str = "bf16", seed: int = 0,
                            bias_var: float = 0.0, scale: float = 1.0, device="cpu"):
    """Stand-alone inputs for the enumeration pass: logits [T,E] fp32 ~ N(0,1) (+ a
    per-expert bias of the given variance) and Y [E,T,H] ~ N(0, scale^2) in the storage
    dtype, from numpy PCG64 streams (logits, bias, Y) spawned from `seed`."""
    s_logits, s_bias, s_y = np.random.SeedSequence(seed).spawn(3)
    logits = np.random.Generator(np.random.PCG64(s_logits)).standard_normal((T, E)).astype(np.float32)
    if bias_var > 0.0:
        b = np.random.Generator(np.random.PCG64(s_bias)).standard_normal((E,)) * bias_var ** 0.5
        logits = (logits + b.astype(np.float32)).astype(np.float32)
    y = np.random.Generator(np.random.PCG64(s_y)).standard_normal((E, T, H)).astype(np.float32) * scale
    tdtype = torch.float32 if dtype == "f32" else torch.bfloat16
    return (torch.from_numpy(logits).to(device),
            torch.from_numpy(y.astype(np.float32)).to(tdtype).to(device))


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact upcast of a stored tensor (fp32 or bf16, any device) to an fp64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy()
