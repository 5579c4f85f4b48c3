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


def rms_err(got, ref):
    """Per-tensor RMS-relative error: ||got - ref||_2 / ||ref||_2.  Beside the infinity-norm figure it sees what that one
    cannot: an error spread thinly over the whole tensor, or a wrong region whose values are small against the
    tensor's maximum."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    den = np.sqrt(np.mean(ref * ref))
    num = np.sqrt(np.mean((got - ref) ** 2))
    return float(num / den) if den > 0 else float(num)


# RMS-relative bound beside TOL.  Every stored bf16 value carries a rounding error of up to 2^-9 of its magnitude,
# 2^-9 / sqrt(3) = 1.1e-3 RMS; a result that went through n roundings of comparable weight sits near sqrt(n) times
# that (4-5 layers of ten stored tensors each: about 8e-3).  fp32: 2^-24 / sqrt(3) per operation.
RMS_TOL = {0: 2e-5, 1: 1e-2}
OBSERVED = []       # (label, max-relative, RMS-relative) of every close() call, printed by the tests that want a record


def close(got, ref, dtype, label="", tol=None, rms_tol=None):
    """Asserts both error measures and records them."""
    e, r = rel_err(got, ref), rms_err(got, ref)
    OBSERVED.append((label, e, r))
    assert e < (TOL[dtype] if tol is None else tol), (label, "max-relative", e)
    assert r < (RMS_TOL[dtype] if rms_tol is None else rms_tol), (label, "rms-relative", r)
    return e, r


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
