"""Seeded synthetic tensors for a stage: weights, per-micro-batch stage inputs and
output gradients.  Every tensor is generated on its own stream
PCG64(SeedSequence([seed, tag, index, sub])) so any one can be rebuilt alone.

Distributions (second argument is the standard deviation): linear weights
N(0, 0.02); norm gains 1 + N(0, 0.02), norm biases N(0, 0.02); stage inputs
N(0, 1); output gradients N(0, 1e-3).  Values are drawn in float32; for bf16
workloads they are rounded to bf16 (round to nearest even) and that rounded
value is what both the oracle and the GPU consume.

No arithmetic of the method lives here.
"""
from __future__ import annotations

import numpy as np

from .configs import BF16, LLAMA, StageConfig

_TAG_WEIGHT, _TAG_X, _TAG_DY = 1, 2, 3
_WNAMES = ("g1", "b1", "wqkv", "wo", "g2", "b2", "wgu", "wd")


def _rng(seed, tag, index, sub=0):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tag, index, sub])))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def quantize(a: np.ndarray, dtype: int) -> np.ndarray:
    """Value as stored in the workload's dtype, returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return bf16_bits_to_f32(f32_to_bf16_bits(a)) if dtype == BF16 else a


def weight_shapes(cfg: StageConfig) -> dict:
    h, f = cfg.hidden, cfg.ffn
    shapes = {"g1": (h,), "wqkv": (cfg.qkv_width, h), "wo": (h, cfg.n_q_heads * cfg.head_dim),
              "g2": (h,), "wgu": (cfg.up_width, h), "wd": (h, f)}
    if cfg.family != LLAMA:
        shapes["b1"] = (h,)
        shapes["b2"] = (h,)
    return shapes


def layer_weights(cfg: StageConfig, layer: int) -> dict:
    """float32 arrays (already rounded to the workload dtype)."""
    out = {}
    for name, shape in weight_shapes(cfg).items():
        r = _rng(cfg.seed, _TAG_WEIGHT, layer, _WNAMES.index(name))
        w = r.standard_normal(shape, dtype=np.float32) * np.float32(0.02)
        if name in ("g1", "g2"):
            w = w + np.float32(1.0)
        out[name] = quantize(w, cfg.dtype)
    return out


def stage_weights(cfg: StageConfig) -> list:
    return [layer_weights(cfg, l) for l in range(cfg.n_layers)]


def stage_input(cfg: StageConfig, mb: int) -> np.ndarray:
    r = _rng(cfg.seed, _TAG_X, mb)
    x = r.standard_normal((cfg.seq * cfg.micro_batch, cfg.hidden), dtype=np.float32)
    return quantize(x, cfg.dtype)


def output_grad(cfg: StageConfig, mb: int) -> np.ndarray:
    r = _rng(cfg.seed, _TAG_DY, mb)
    g = r.standard_normal((cfg.seq * cfg.micro_batch, cfg.hidden), dtype=np.float32) * np.float32(1e-3)
    return quantize(g, cfg.dtype)


# ---- the same distributions drawn on the device (host generation of several GiB of weights is slow): seeded
# torch generators, so a tensor can be rebuilt alone; checks against the oracle read these tensors back

def device_weights(cfg: StageConfig) -> list:
    """Per layer dict name -> device tensor in the workload dtype: linear weights N(0, 0.02), gains 1 + N(0, 0.02),
    biases N(0, 0.02)."""
    import torch
    g = torch.Generator(device="cuda")
    dt = torch.bfloat16 if cfg.dtype == BF16 else torch.float32
    out = []
    for l in range(cfg.n_layers):
        w = {}
        for i, (name, shape) in enumerate(weight_shapes(cfg).items()):
            g.manual_seed(cfg.seed * 1000003 + l * 101 + i)
            t = torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * 0.02
            if name in ("g1", "g2"):
                t = t + 1.0
            w[name] = t.to(dt).contiguous()
        out.append(w)
    return out


def device_io(cfg: StageConfig, mb: int):
    """(stage input N(0, 1), output gradient N(0, 1e-3)) of micro-batch mb as device tensors in the workload dtype."""
    import torch
    g = torch.Generator(device="cuda")
    dt = torch.bfloat16 if cfg.dtype == BF16 else torch.float32
    shape = (cfg.seq * cfg.micro_batch, cfg.hidden)
    g.manual_seed(cfg.seed * 1000003 + 50000 + mb)
    x = torch.randn(shape, generator=g, device="cuda", dtype=torch.float32).to(dt)
    g.manual_seed(cfg.seed * 1000003 + 90000 + mb)
    dy = (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * 1e-3).to(dt)
    return x.contiguous(), dy.contiguous()
