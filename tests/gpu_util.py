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


def block_rms_err(got, ref, blocks=8):
    """Largest RMS-relative error over a blocks x blocks partition of the tensor (blocks pieces for a vector), each
    block measured against its OWN reference energy: a wrong region whose values are small against the rest of the
    tensor (early attention rows, one mis-scaled column group) stands out here and nowhere else."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if got.ndim == 1:
        got, ref = got[None, :], ref[None, :]
    got, ref = got.reshape(-1, got.shape[-1]), ref.reshape(-1, ref.shape[-1])
    worst = 0.0
    for rg, rr in zip(np.array_split(got, min(blocks, got.shape[0]), axis=0), np.array_split(ref, min(blocks, ref.shape[0]), axis=0)):
        for cg, cr in zip(np.array_split(rg, min(blocks, rg.shape[1]), axis=1), np.array_split(rr, min(blocks, rr.shape[1]), axis=1)):
            den = np.sqrt(np.mean(cr * cr))
            num = np.sqrt(np.mean((cg - cr) ** 2))
            worst = max(worst, float(num / den) if den > 0 else float(num))
    return worst


# Bounds on the two L2 measures, beside TOL on the infinity-norm one: the tolerance the workloads state, applied to
# the whole tensor's RMS-relative error and to every block's.  What rounding alone predicts: a stored bf16 value is
# off by up to 2^-9 of its magnitude, 2^-9 / sqrt(3) = 1.1e-3 RMS; a stage output has about 12 such roundings per
# layer behind it (ten stored tensors, the attention probabilities and their gradients inside the kernels), a
# gradient about 24, adding in quadrature: sqrt(24 * 5) * 1.1e-3 = 1.2e-2 for five layers.  fp32: 1e-4 as for TOL.
RMS_TOL = {0: 1e-4, 1: 2e-2}
OBSERVED = []       # (label, max-relative, RMS-relative, worst block RMS-relative) of every close() call


def close(got, ref, dtype, label="", tol=None, rms_tol=None):
    """Asserts the three error measures and records them."""
    e, r, bl = rel_err(got, ref), rms_err(got, ref), block_rms_err(got, ref)
    OBSERVED.append((label, e, r, bl))
    assert e < (TOL[dtype] if tol is None else tol), (label, "max-relative", e, r, bl)
    assert r < (RMS_TOL[dtype] if rms_tol is None else rms_tol), (label, "rms-relative", e, r, bl)
    assert bl < (RMS_TOL[dtype] if rms_tol is None else rms_tol), (label, "block rms-relative", e, r, bl)
    return e, r


def report(out=print):
    """Prints and clears the record of close() calls."""
    for label, e, r, bl in OBSERVED:
        out(f"  {label}: max-rel {e:.2e} rms-rel {r:.2e} worst-block rms-rel {bl:.2e}")
    del OBSERVED[:]


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
