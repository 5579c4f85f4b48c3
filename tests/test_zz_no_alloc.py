"""The norm backward entry point that allocates nothing (its partial sums live in an array inside the
library's device image) against the entry point that takes the same scratch from the caller: bit-identical
results on two calls in a row, the second on a smaller input, and both within tolerance of the oracle.
Also: a hidden size beyond the static array's maximum is refused and writes nothing."""
import numpy as np
import pytest
import torch

from oracle import stage_fp64 as O
from paper_2510_05186_amd import binding as B
from gpu_util import TOL, dev, host, ok, q, rel_err, rms_err, stream

pytestmark = pytest.mark.gpu
BF16, FP32 = 1, 0


def _case(dtype, family, rows, h, seed):
    rng = np.random.default_rng(seed)
    x = q(2.0 * rng.standard_normal((rows, h)) + 0.3, dtype)
    g = q(1 + 0.1 * rng.standard_normal(h), dtype)
    b = q(0.1 * rng.standard_normal(h), dtype)
    dn = q(rng.standard_normal((rows, h)), dtype)
    dres = q(rng.standard_normal((rows, h)), dtype)
    dg0 = rng.standard_normal(h).astype(np.float32)
    return x, g, b, dn, dres, dg0


def _run_both(dtype, family, rows, h, seed):
    lib = B.lib()
    x, g, b, dn, dres, dg0 = _case(dtype, family, rows, h, seed)
    X, G, Bt, DN, DR = (dev(a, dtype) for a in (x, g, b, dn, dres))
    nst = 1 if family == O.LLAMA else 2
    OUT = torch.empty_like(X)
    ST = torch.empty(rows * nst, dtype=torch.float32, device="cuda")
    ok(lib.optstage_op_norm_fwd(dtype, family, X.data_ptr(), G.data_ptr(), Bt.data_ptr(), OUT.data_ptr(), ST.data_ptr(), rows, h, 1e-5, stream()))
    res = []
    for static in (False, True):
        DX = torch.full_like(X, float("nan"))
        DG = torch.from_numpy(dg0.copy()).cuda()
        DB = torch.zeros(h, dtype=torch.float32, device="cuda")
        if static:
            print(f"norm_bwd_static dtype={dtype} family={family} rows={rows} hidden={h}", flush=True)
            ok(lib.optstage_op_norm_bwd_static(dtype, family, DN.data_ptr(), X.data_ptr(), ST.data_ptr(), G.data_ptr(), DR.data_ptr(),
                                               DX.data_ptr(), DG.data_ptr(), DB.data_ptr(), rows, h, stream()))
        else:
            part = torch.empty(2 * min(rows, 512) * h, dtype=torch.float32, device="cuda")
            ok(lib.optstage_op_norm_bwd(dtype, family, DN.data_ptr(), X.data_ptr(), ST.data_ptr(), G.data_ptr(), DR.data_ptr(),
                                        DX.data_ptr(), part.data_ptr(), DG.data_ptr(), DB.data_ptr(), rows, h, stream()))
        torch.cuda.synchronize()
        res.append((DX, DG, DB))
    (dx0, dg_0, db0), (dx1, dg_1, db1) = res
    assert torch.equal(dx0, dx1) and torch.equal(dg_0, dg_1) and torch.equal(db0, db1)
    if family == O.LLAMA:
        _, r = O.rmsnorm_fwd(x, g, 1e-5)
        dx, dgam = O.rmsnorm_bwd(dn, x, r, g)
    else:
        _, mu, r = O.layernorm_fwd(x, g, b, 1e-5)
        dx, dgam, dbeta = O.layernorm_bwd(dn, x, mu, r, g)
        assert rel_err(host(db1), dbeta) < 1e-5
    assert rel_err(host(dx1), dres + dx) < TOL[dtype]
    assert rms_err(host(dx1), dres + dx) < TOL[dtype] / 4
    assert rel_err(host(dg_1), dg0 + dgam) < 1e-5


@pytest.mark.parametrize("dtype,family,first,second", [
    (BF16, O.LLAMA, (2500, 4096), (300, 1024)),      # row-per-workgroup kernel, then the row-per-wave kernel on fewer rows
    (BF16, O.GPT, (2100, 2048), (64, 1024)),         # LayerNorm: gain and bias partials, then fewer workgroups than 256
    (FP32, O.GPT, (700, 1000), (37, 256)),
])
def test_static_scratch_entry_point_equals_the_workspace_one(dtype, family, first, second):
    _run_both(dtype, family, first[0], first[1], 1)
    _run_both(dtype, family, second[0], second[1], 2)      # smaller input on the array the first call left behind


def test_static_scratch_entry_point_rejects_sizes_beyond_its_array():
    lib = B.lib()
    rows, h = 8, 16384
    X = torch.zeros(rows, h, dtype=torch.bfloat16, device="cuda")
    DX = torch.zeros_like(X)
    F = torch.zeros(h, dtype=torch.float32, device="cuda")
    st = lib.optstage_op_norm_bwd_static(BF16, O.LLAMA, X.data_ptr(), X.data_ptr(), F.data_ptr(), X.data_ptr(), 0, DX.data_ptr(),
                                         F.data_ptr(), 0, rows, h, stream())
    assert st == B.E_ARG and b"8192" in lib.optstage_last_error()
    torch.cuda.synchronize()
    assert float(DX.float().abs().sum()) == 0.0 and float(F.abs().sum()) == 0.0
