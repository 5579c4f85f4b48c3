"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import torch

from oracle import stage_fp64 as O
from paper_2510_05186_amd import binding as B
from stage_inputs import tensors as T

TOL = {0: 1e-4, 1: 2e-2}      # max relative error: fp32 workload 1e-4, bf16 workloads 2e-2
TDT = {0: torch.float32, 1: torch.bfloat16}


def rel_err(got, ref):
    """Per-tensor infinity-norm relative error: max|got - ref| / max|ref|."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got))
    den = np.max(np.abs(ref))
    return float(np.max(np.abs(got - ref)) / den) if den > 0 else float(np.max(np.abs(got)))


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda", TDT[dtype]).contiguous()


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def q(a, dtype):
    """Round a float array to the storage dtype; returns float64 of the stored value."""
    return T.quantize(np.asarray(a, dtype=np.float32), dtype).astype(np.float64)


def stream():
    return torch.cuda.current_stream().cuda_stream


def oracle_shape(cfg):
    return O.StageShape(cfg.family, cfg.n_layers, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                        cfg.ffn, cfg.seq, cfg.norm_eps, cfg.rope_base)


def oracle_weights(ws):
    return [{k: v.astype(np.float64) for k, v in w.items()} for w in ws]


def ok(status):
    assert status == B.OK, (status, B.lib().optstage_last_error().decode())
