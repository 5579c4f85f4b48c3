"""Kernel-by-kernel parity of the HIP path against the fp64 oracle, through the C-ABI.
Sizes span several tiles and a ragged tail; the oracle finishes each in well under a second."""
import numpy as np
import pytest
import torch

from oracle import stage_fp64 as O
from paper_2510_05186_amd import binding as B
from gpu_util import TOL, dev, host, ok, q, rel_err, rms_err, stream

pytestmark = pytest.mark.gpu
RNG = np.random.default_rng(42)
FP32, BF16 = 0, 1


def lib():
    return B.lib()


# ------------------------------------------------------------------ GEMM
@pytest.mark.parametrize("dtype,M,N,K", [
    (BF16, 520, 776, 328),        # 128x128 tiles, ragged in M, N and K
    (BF16, 2824, 3080, 264),      # 256x256 tiles (12 x 13), ragged
    (BF16, 2824, 3080, 320),      # same, K a multiple of 64: direct global->LDS tile loads, ragged M and N
    (BF16, 4096, 2048, 64),       # direct path, a single k-tile
    (BF16, 3000, 4096, 128),      # direct path, two k-tiles
    (BF16, 2824, 3080, 192),      # direct path: 3, 6, 7 and 11 k-tiles walk the ring of five LDS slots through every
    (BF16, 2824, 3080, 384),      # alignment of a tile's two slots, with and without a wrap inside the tile
    (BF16, 2824, 3080, 448),
    (BF16, 2824, 3080, 704),
    (BF16, 256, 256, 64),
    (BF16, 8, 8, 8),
    (FP32, 130, 77, 50),
    (FP32, 128, 256, 1024),
])
def test_gemm_nt_store_and_residual(dtype, M, N, K):
    a = q(RNG.standard_normal((M, K)), dtype)
    w = q(0.05 * RNG.standard_normal((N, K)), dtype)
    r = q(RNG.standard_normal((M, N)), dtype)
    A, W, R = dev(a, dtype), dev(w, dtype), dev(r, dtype)
    C = torch.empty_like(R)
    ok(lib().optstage_op_gemm(dtype, B.GEMM_NT, B.EPI_STORE, A.data_ptr(), W.data_ptr(), C.data_ptr(), 0, M, N, K, K, K, N, stream()))
    torch.cuda.synchronize()
    assert rel_err(host(C), O.linear_fwd(a, w)) < TOL[dtype]
    ok(lib().optstage_op_gemm(dtype, B.GEMM_NT, B.EPI_RESID, A.data_ptr(), W.data_ptr(), C.data_ptr(), R.data_ptr(), M, N, K, K, K, N, stream()))
    torch.cuda.synchronize()
    assert rel_err(host(C), r + O.linear_fwd(a, w)) < TOL[dtype]


@pytest.mark.parametrize("dtype,M,N,K", [
    (BF16, 520, 776, 333),        # K (tokens) need not be a multiple of anything
    (BF16, 2824, 3080, 200),
    (BF16, 2824, 3080, 64),       # direct path (whole 64-token k-tiles, 156 tiles): 1, 2, 5, 7 and 11 k-tiles
    (BF16, 2824, 3080, 128),
    (BF16, 2824, 3080, 320),
    (BF16, 2824, 3080, 448),
    (BF16, 2824, 3080, 704),
    (BF16, 8, 16, 1),
    (FP32, 130, 76, 50),
])
def test_gemm_tn_accumulate(dtype, M, N, K):
    # dW[M,N] += dY^T X with dY [K,M], X [K,N]
    dy = q(RNG.standard_normal((K, M)), dtype)
    x = q(RNG.standard_normal((K, N)), dtype)
    c0 = RNG.standard_normal((M, N)).astype(np.float32)
    DY, X = dev(dy, dtype), dev(x, dtype)
    C = torch.from_numpy(c0.copy()).cuda()
    for rep in range(2):
        ok(lib().optstage_op_gemm(dtype, B.GEMM_TN, B.EPI_ACCUM, DY.data_ptr(), X.data_ptr(), C.data_ptr(), 0, M, N, K, M, N, N, stream()))
    torch.cuda.synchronize()
    ref = c0.astype(np.float64) + 2 * O.linear_bwd_weight(dy, x)
    assert rel_err(host(C), ref) < (1e-5 if dtype == FP32 else 1e-4)    # fp32 accumulators: no bf16 rounding of C


def test_gemm_grouped_equals_one_by_one_and_the_oracle():
    """The weight-gradient products of a W op in one launch (shapes of the Llama stage's four linears at a
    shorter token count, including a ragged 200-row edge tile): bitwise the same as launching each on its
    own, and within tolerance of dY^T X from the oracle on sampled rows."""
    import ctypes as C
    K = 768
    shapes = [(1024, 2752), (5504, 1024), (1024, 1024), (3072, 1024), (200, 1024)]
    probs = (B.GemmProblem * len(shapes))()
    keep = []
    for i, (M, N) in enumerate(shapes):
        dy = q(RNG.standard_normal((K, M)), BF16)
        x = q(RNG.standard_normal((K, N)), BF16)
        c0 = torch.from_numpy(RNG.standard_normal((M, N)).astype(np.float32)).cuda()
        DY, X = dev(dy, BF16), dev(x, BF16)
        grouped, single = c0.clone(), c0.clone()
        ok(lib().optstage_op_gemm(BF16, B.GEMM_TN, B.EPI_ACCUM, DY.data_ptr(), X.data_ptr(), single.data_ptr(), 0, M, N, K, M, N, N, stream()))
        probs[i].A, probs[i].B, probs[i].C, probs[i].R = DY.data_ptr(), X.data_ptr(), grouped.data_ptr(), 0
        probs[i].M, probs[i].N, probs[i].lda, probs[i].ldb, probs[i].ldc = M, N, M, N, N
        keep.append((dy, x, c0, DY, X, grouped, single))
    ok(lib().optstage_op_gemm_grouped(B.GEMM_TN, B.EPI_ACCUM, len(shapes), C.cast(probs, C.c_void_p), K, stream()))
    torch.cuda.synchronize()
    for dy, x, c0, DY, X, grouped, single in keep:
        assert torch.equal(grouped, single)
        rows = RNG.choice(dy.shape[1], size=min(16, dy.shape[1]), replace=False)
        ref = host(c0)[rows] + dy[:, rows].T.astype(np.float64) @ x.astype(np.float64)
        assert rel_err(host(grouped)[rows], ref) < 1e-4
    # a set that does not qualify (K not a multiple of 64) is refused and nothing runs
    assert lib().optstage_op_gemm_grouped(B.GEMM_TN, B.EPI_ACCUM, len(shapes), C.cast(probs, C.c_void_p), 72, stream()) == B.E_ARG


def slabs_of(w):
    """[N, K] -> the slab layout of layout code 2: slab (n // 256, k // 64) holds rows 256 x columns 64, row-major,
    slabs ordered by (n // 256, k // 64); rows padded to a multiple of 256."""
    n, k = w.shape
    n_pad = (n + 255) // 256 * 256
    wp = np.zeros((n_pad, k), dtype=w.dtype)
    wp[:n] = w
    return np.ascontiguousarray(wp.reshape(n_pad // 256, 256, k // 64, 64).transpose(0, 2, 1, 3))


@pytest.mark.parametrize("M,N,K,epi", [(2816, 3072, 192, B.EPI_STORE), (2817, 3000, 256, B.EPI_RESID), (4096, 2048, 64, B.EPI_STORE)])
def test_gemm_with_b_in_slabs(M, N, K, epi):
    """The layout the stage keeps its weight copies in: bitwise the row-major product, and the oracle's on
    sampled rows (ragged edges in both directions)."""
    a = q(RNG.standard_normal((M, K)), BF16)
    w = q(RNG.standard_normal((N, K)), BF16)
    r = q(RNG.standard_normal((M, N)), BF16)
    A, W, WS, R = dev(a, BF16), dev(w, BF16), dev(slabs_of(w), BF16), dev(r, BF16)
    rp = R.data_ptr() if epi == B.EPI_RESID else 0
    C0 = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    C1 = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    ok(lib().optstage_op_gemm(BF16, B.GEMM_NT, epi, A.data_ptr(), W.data_ptr(), C0.data_ptr(), rp, M, N, K, K, K, N, stream()))
    ok(lib().optstage_op_gemm(BF16, B.GEMM_NT_SLAB, epi, A.data_ptr(), WS.data_ptr(), C1.data_ptr(), rp, M, N, K, K, 0, N, stream()))
    torch.cuda.synchronize()
    assert torch.equal(C0, C1)
    rows = RNG.choice(M, size=24, replace=False)
    ref = a[rows].astype(np.float64) @ w.astype(np.float64).T + (r[rows] if epi == B.EPI_RESID else 0.0)
    assert rel_err(host(C1)[rows], ref) < TOL[BF16]
    # too few tiles for the kernel that reads slabs, a contraction that is not whole slabs, fp32: refused
    f = lib().optstage_op_gemm
    assert f(BF16, B.GEMM_NT_SLAB, epi, A.data_ptr(), WS.data_ptr(), C1.data_ptr(), rp, 512, 512, K, K, 0, N, stream()) == B.E_ARG
    assert f(BF16, B.GEMM_NT_SLAB, epi, A.data_ptr(), WS.data_ptr(), C1.data_ptr(), rp, M, N, K - 8, K, 0, N, stream()) == B.E_ARG
    assert f(FP32, B.GEMM_NT_SLAB, epi, A.data_ptr(), WS.data_ptr(), C1.data_ptr(), rp, M, N, K, K, 0, N, stream()) == B.E_ARG
    assert f(BF16, B.GEMM_NT_SLAB, B.EPI_ACCUM, A.data_ptr(), WS.data_ptr(), C1.data_ptr(), 0, M, N, K, K, 0, N, stream()) == B.E_ARG


@pytest.mark.parametrize("N,K", [(512, 128), (300, 64), (1000, 448)])
def test_weight_slabs_match_the_host_layout(N, K):
    w = q(RNG.standard_normal((N, K)), BF16)
    want = torch.from_numpy(slabs_of(w).astype(np.float32)).bfloat16().reshape(-1)
    n_pad = (N + 255) // 256 * 256
    for transposed, src in ((0, w), (1, np.ascontiguousarray(w.T))):
        S = dev(src, BF16)
        D = torch.full((n_pad * K,), 3.0, dtype=torch.bfloat16, device="cuda")
        ok(lib().optstage_op_weight_slabs(S.data_ptr(), D.data_ptr(), N, K, transposed, stream()))
        torch.cuda.synchronize()
        assert torch.equal(D.cpu(), want), transposed
    assert lib().optstage_op_weight_slabs(S.data_ptr(), D.data_ptr(), N, K + 8, 0, stream()) == B.E_ARG


def test_gemm_rejects_bad_shapes():
    A = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    f = lib().optstage_op_gemm
    assert f(BF16, 0, 0, A.data_ptr(), A.data_ptr(), A.data_ptr(), 0, 64, 64, 60, 60, 60, 64, stream()) == B.E_ARG   # K % 8
    assert f(BF16, 0, 0, A.data_ptr(), A.data_ptr(), A.data_ptr(), 0, 64, 62, 64, 64, 64, 62, stream()) == B.E_ARG   # N % 4
    assert f(BF16, 0, 0, 0, A.data_ptr(), A.data_ptr(), 0, 64, 64, 64, 64, 64, 64, stream()) == B.E_ARG              # null
    assert f(BF16, 0, 1, A.data_ptr(), A.data_ptr(), A.data_ptr(), 0, 64, 64, 64, 64, 64, 64, stream()) == B.E_ARG   # residual missing
    assert f(BF16, 0, 0, A.data_ptr(), A.data_ptr(), A.data_ptr(), 0, 64, 64, 64, 32, 64, 64, stream()) == B.E_ARG   # lda < K
    assert f(BF16, 1, 2, A.data_ptr(), A.data_ptr(), A.data_ptr(), 0, 60, 64, 64, 64, 64, 64, stream()) == B.E_ARG   # TN: M % 8
    torch.cuda.synchronize()


# ------------------------------------------------------------------ norms
@pytest.mark.parametrize("dtype,family,rows,h", [
    (BF16, O.LLAMA, 300, 4096), (BF16, O.LLAMA, 37, 520), (BF16, O.GPT, 64, 1024), (BF16, O.LLAMA, 700, 8192),
    (FP32, O.GPT, 128, 256), (FP32, O.LLAMA, 130, 1000), (BF16, O.GPT, 2100, 2048), (FP32, O.GPT, 8200, 256), (BF16, O.LLAMA, 2500, 1024),
])
def test_norm_fwd_bwd(dtype, family, rows, h):
    eps = 1e-5
    x = q(2.0 * RNG.standard_normal((rows, h)) + 0.3, dtype)
    g = q(1 + 0.1 * RNG.standard_normal(h), dtype)
    b = q(0.1 * RNG.standard_normal(h), dtype)
    dn = q(RNG.standard_normal((rows, h)), dtype)
    dres = q(RNG.standard_normal((rows, h)), dtype)
    X, G, Bt, DN, DR = (dev(a, dtype) for a in (x, g, b, dn, dres))
    OUT = torch.empty_like(X)
    nst = 1 if family == O.LLAMA else 2
    ST = torch.empty(rows * nst, dtype=torch.float32, device="cuda")
    ok(lib().optstage_op_norm_fwd(dtype, family, X.data_ptr(), G.data_ptr(), Bt.data_ptr(), OUT.data_ptr(), ST.data_ptr(), rows, h, eps, stream()))
    DX = torch.empty_like(X)
    part = torch.empty(2 * min(rows, 512) * h, dtype=torch.float32, device="cuda")
    dg0 = RNG.standard_normal(h).astype(np.float32)
    DG, DB = torch.from_numpy(dg0.copy()).cuda(), torch.zeros(h, dtype=torch.float32, device="cuda")
    ok(lib().optstage_op_norm_bwd(dtype, family, DN.data_ptr(), X.data_ptr(), ST.data_ptr(), G.data_ptr(), DR.data_ptr(), DX.data_ptr(), part.data_ptr(), DG.data_ptr(), DB.data_ptr(), rows, h, stream()))
    torch.cuda.synchronize()
    if family == O.LLAMA:
        n, r = O.rmsnorm_fwd(x, g, eps)
        dx, dgam = O.rmsnorm_bwd(dn, x, r, g)
        assert rel_err(host(ST), r[:, 0]) < 1e-5
    else:
        n, mu, r = O.layernorm_fwd(x, g, b, eps)
        dx, dgam, dbeta = O.layernorm_bwd(dn, x, mu, r, g)
        st = host(ST).reshape(rows, 2)
        assert rel_err(st[:, 0], mu[:, 0]) < 1e-5 and rel_err(st[:, 1], r[:, 0]) < 1e-5
        assert rel_err(host(DB), dbeta) < 1e-5
    assert rel_err(host(OUT), n) < TOL[dtype]
    assert rel_err(host(DX), dres + dx) < TOL[dtype]
    assert rel_err(host(DG), dg0 + dgam) < 1e-5      # fp32 accumulation of exactly representable inputs


# ------------------------------------------------------------------ activations
@pytest.mark.parametrize("dtype,family,rows,f", [(BF16, O.LLAMA, 333, 1376), (BF16, O.GPT, 50, 1024),
                                                  (FP32, O.GPT, 128, 1024), (FP32, O.LLAMA, 17, 100)])
def test_activation_fwd_bwd(dtype, family, rows, f):
    w = 2 * f if family == O.LLAMA else f
    gu = q(1.5 * RNG.standard_normal((rows, w)), dtype)
    da = q(RNG.standard_normal((rows, f)), dtype)
    GU, DA = dev(gu, dtype), dev(da, dtype)
    A = torch.empty(rows, f, dtype=GU.dtype, device="cuda")
    ok(lib().optstage_op_act_fwd(dtype, family, GU.data_ptr(), A.data_ptr(), rows, f, stream()))
    ok(lib().optstage_op_act_bwd(dtype, family, DA.data_ptr(), GU.data_ptr(), GU.data_ptr(), rows, f, stream()))   # in place
    torch.cuda.synchronize()
    if family == O.LLAMA:
        a, dgu = O.swiglu_fwd(gu), O.swiglu_bwd(da, gu)
    else:
        a, dgu = O.gelu_fwd(gu), O.gelu_bwd(da, gu)
    assert rel_err(host(A), a) < TOL[dtype]
    assert rel_err(host(GU), dgu) < TOL[dtype]


# ------------------------------------------------------------------ rotary
@pytest.mark.parametrize("dtype,seq,batch,nq,nkv,d", [(BF16, 300, 1, 4, 2, 128), (FP32, 70, 2, 3, 3, 64), (BF16, 4096, 1, 2, 1, 128),
                                                       (BF16, 333, 2, 6, 2, 128), (FP32, 70, 1, 2, 2, 64)])   # q + k heads a multiple of 4
def test_rotary(dtype, seq, batch, nq, nkv, d):
    base = 10000.0
    rows = seq * batch
    w = (nq + 2 * nkv) * d
    qkv = q(RNG.standard_normal((rows, w)), dtype)
    table = torch.empty(seq * d, dtype=torch.float32, device="cuda")
    ok(lib().optstage_op_rope_table(table.data_ptr(), seq, d, base, stream()))
    SRC = dev(qkv, dtype)
    DST = torch.zeros_like(SRC)
    ok(lib().optstage_op_rope(dtype, SRC.data_ptr(), DST.data_ptr(), table.data_ptr(), rows, seq, nq, nkv, d, 1, stream()))   # backward, out of place
    ok(lib().optstage_op_rope(dtype, SRC.data_ptr(), SRC.data_ptr(), table.data_ptr(), rows, seq, nq, nkv, d, 0, stream()))   # forward, in place
    torch.cuda.synchronize()
    # table against fp64
    k = np.arange(d // 2)
    ang = np.arange(seq)[:, None] * base ** (-2.0 * k / d)[None, :]
    tb = host(table).reshape(seq, d // 2, 2)
    assert np.max(np.abs(tb[..., 0] - np.cos(ang))) < 1e-7 and np.max(np.abs(tb[..., 1] - np.sin(ang))) < 1e-7

    def ref(sign):
        out = qkv.copy().reshape(batch, seq, w)
        for b in range(batch):
            qq = out[b, :, : nq * d].reshape(seq, nq, d)
            kk = out[b, :, nq * d: (nq + nkv) * d].reshape(seq, nkv, d)
            out[b, :, : nq * d] = O.rope_apply(qq, base, sign).reshape(seq, -1)
            out[b, :, nq * d: (nq + nkv) * d] = O.rope_apply(kk, base, sign).reshape(seq, -1)
        return out.reshape(rows, w)
    assert rel_err(host(SRC), ref(1.0)) < TOL[dtype]
    assert rel_err(host(DST), ref(-1.0)) < TOL[dtype]


# ------------------------------------------------------------------ attention
@pytest.mark.parametrize("dtype,seq,batch,nq,nkv,d", [
    (FP32, 128, 1, 4, 4, 64), (FP32, 67, 2, 4, 2, 64), (BF16, 200, 1, 4, 2, 128), (BF16, 130, 1, 2, 2, 64),
    (BF16, 512, 1, 8, 2, 128), (BF16, 1, 1, 2, 1, 128), (BF16, 384, 2, 2, 2, 128), (BF16, 1000, 1, 4, 1, 128),
    (BF16, 65, 1, 1, 1, 128), (BF16, 129, 3, 2, 2, 128),
])
def test_attention_fwd_bwd(dtype, seq, batch, nq, nkv, d):
    rows = seq * batch
    w = (nq + 2 * nkv) * d
    qkv = q(RNG.standard_normal((rows, w)), dtype)
    do = q(RNG.standard_normal((rows, nq * d)), dtype)
    QKV, DO = dev(qkv, dtype), dev(do, dtype)
    Ot = torch.empty(rows, nq * d, dtype=QKV.dtype, device="cuda")
    LSE = torch.empty(batch * nq * seq, dtype=torch.float32, device="cuda")
    ok(lib().optstage_op_attn_fwd(dtype, QKV.data_ptr(), Ot.data_ptr(), LSE.data_ptr(), seq, batch, nq, nkv, d, stream()))
    DQKV = torch.zeros_like(QKV)
    nws = lib().optstage_op_attn_bwd_ws_floats(seq, batch, nq, nkv, d)
    WS = torch.empty(max(1, nws), dtype=torch.float32, device="cuda")
    ok(lib().optstage_op_attn_bwd(dtype, QKV.data_ptr(), Ot.data_ptr(), DO.data_ptr(), LSE.data_ptr(), DQKV.data_ptr(), WS.data_ptr(), seq, batch, nq, nkv, d, stream()))
    torch.cuda.synchronize()
    o_g, lse_g, dq_g = host(Ot), host(LSE).reshape(batch, nq, seq), host(DQKV)
    for b in range(batch):
        sl = slice(b * seq, (b + 1) * seq)
        qq = qkv[sl, : nq * d].reshape(seq, nq, d)
        kk = qkv[sl, nq * d: (nq + nkv) * d].reshape(seq, nkv, d)
        vv = qkv[sl, (nq + nkv) * d:].reshape(seq, nkv, d)
        o, lse = O.attention_fwd(qq, kk, vv)
        assert rel_err(o_g[sl], o.reshape(seq, -1)) < TOL[dtype]
        assert np.max(np.abs(lse_g[b] - lse)) < (1e-4 if dtype == FP32 else 2e-2)
        # backward is fed the GPU's own (stored-precision) o, as in the stage
        dq, dk, dv = O.attention_bwd(qq, kk, vv, o_g[sl].reshape(seq, nq, d), do[sl].reshape(seq, nq, d))
        ref = np.concatenate([dq.reshape(seq, -1), dk.reshape(seq, -1), dv.reshape(seq, -1)], axis=1)
        for lo, hi in ((0, nq * d), (nq * d, (nq + nkv) * d), ((nq + nkv) * d, w)):
            assert rel_err(dq_g[sl, lo:hi], ref[:, lo:hi]) < TOL[dtype], (lo, hi)


@pytest.mark.parametrize("gain", [6.0, 0.05])
def test_attention_forward_with_peaked_and_flat_scores(gain):
    """Scores far larger than usual (the softmax reference has to be raised again and again, and most
    probabilities underflow) and far smaller (the reference is set once and never raised)."""
    seq, nq, nkv, d = 700, 2, 1, 128
    w = (nq + 2 * nkv) * d
    qkv = RNG.standard_normal((seq, w))
    qkv[:, : (nq + nkv) * d] *= gain
    qkv = q(qkv, BF16)
    QKV = dev(qkv, BF16)
    Ot = torch.empty(seq, nq * d, dtype=QKV.dtype, device="cuda")
    LSE = torch.empty(nq * seq, dtype=torch.float32, device="cuda")
    ok(lib().optstage_op_attn_fwd(BF16, QKV.data_ptr(), Ot.data_ptr(), LSE.data_ptr(), seq, 1, nq, nkv, d, stream()))
    torch.cuda.synchronize()
    qq = qkv[:, : nq * d].reshape(seq, nq, d)
    kk = qkv[:, nq * d: (nq + nkv) * d].reshape(seq, nkv, d)
    vv = qkv[:, (nq + nkv) * d:].reshape(seq, nkv, d)
    o, lse = O.attention_fwd(qq, kk, vv)
    assert np.isfinite(host(Ot)).all() and np.isfinite(host(LSE)).all()
    assert rel_err(host(Ot), o.reshape(seq, -1)) < TOL[BF16]
    assert np.max(np.abs(host(LSE).reshape(nq, seq) - lse) / np.maximum(1.0, np.abs(lse))) < 2e-2


# ------------------------------------------------------------------ checksum
def test_checksum_matches_host_arithmetic():
    for n in (0, 8, 4096, 1 << 20, (1 << 20) + 8):
        a = RNG.integers(0, 2**63, size=max(1, n // 8), dtype=np.uint64)[: n // 8]
        t = torch.from_numpy(a.view(np.int64).copy()).cuda() if n else torch.zeros(1, dtype=torch.int64, device="cuda")
        out = torch.zeros(2, dtype=torch.int64, device="cuda")
        ok(lib().optstage_op_checksum(t.data_ptr(), n, out.data_ptr(), stream()))
        torch.cuda.synchronize()
        got = out.cpu().numpy().view(np.uint64)
        s = int(np.sum(a, dtype=np.uint64)) if n else 0
        x = int(np.bitwise_xor.reduce(a)) if n else 0
        assert int(got[0]) == s and int(got[1]) == x


def test_empty_inputs_are_refused_not_launched():
    """A zero extent anywhere is an argument error of the call (nothing is launched, nothing is written)."""
    L_ = lib()
    a = torch.zeros(4096, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(4096, dtype=torch.float32, device="cuda")
    p, q = a.data_ptr(), f.data_ptr()
    for M, N, K in ((0, 64, 64), (64, 0, 64), (64, 64, 0)):
        assert L_.optstage_op_gemm(BF16, B.GEMM_NT, B.EPI_STORE, p, p, p, 0, M, N, K, 64, 64, 64, stream()) == B.E_ARG
        assert L_.optstage_op_gemm(BF16, B.GEMM_TN, B.EPI_ACCUM, p, p, q, 0, M, N, K, 64, 64, 64, stream()) == B.E_ARG
    assert L_.optstage_op_norm_fwd(BF16, O.LLAMA, p, p, 0, p, q, 0, 64, 1e-5, stream()) == B.E_ARG
    assert L_.optstage_op_norm_fwd(BF16, O.LLAMA, p, p, 0, p, q, 8, 0, 1e-5, stream()) == B.E_ARG
    assert L_.optstage_op_norm_bwd(BF16, O.LLAMA, p, p, q, p, 0, p, q, q, 0, 0, 64, stream()) == B.E_ARG
    assert L_.optstage_op_act_fwd(BF16, O.LLAMA, p, p, 0, 64, stream()) == B.E_ARG
    assert L_.optstage_op_act_bwd(BF16, O.LLAMA, p, p, p, 8, 0, stream()) == B.E_ARG
    assert L_.optstage_op_rope(BF16, p, p, q, 0, 8, 2, 2, 128, 0, stream()) == B.E_ARG
    assert L_.optstage_op_attn_fwd(BF16, p, p, q, 0, 1, 2, 2, 128, stream()) == B.E_ARG
    assert L_.optstage_op_attn_bwd(BF16, p, p, p, q, q, q, 0, 1, 2, 2, 128, stream()) == B.E_ARG
    assert L_.optstage_op_weight_slabs(p, q, 0, 64, 0, stream()) == B.E_ARG
    torch.cuda.synchronize()
    assert float(a.float().abs().sum()) == 0.0 and float(f.abs().sum()) == 0.0


# ------------------------------------------------------------------ projections with a fused epilogue
@pytest.mark.parametrize("layout,M,N,K,seq,rot", [(B.GEMM_NT, 2000, 4096, 256, 500, 3072), (2, 2048, 4096, 192, 2048, 4096),
                                                  (B.GEMM_NT, 4096, 2048, 128, 1024, 1024)])
def test_gemm_with_rotary_in_the_epilogue(layout, M, N, K, seq, rot):
    d = 128
    a = q(RNG.standard_normal((M, K)), BF16)
    w = q(0.1 * RNG.standard_normal((N, K)), BF16)
    A, W = dev(a, BF16), dev(w, BF16)
    L_ = lib()
    Wop = W
    if layout == 2:
        Wop = torch.empty((N + 255) // 256 * 256 * K, dtype=torch.bfloat16, device="cuda")
        ok(L_.optstage_op_weight_slabs(W.data_ptr(), Wop.data_ptr(), N, K, 0, stream()))
    table = torch.empty(seq * (d // 2) * 2, dtype=torch.float32, device="cuda")
    ok(L_.optstage_op_rope_table(table.data_ptr(), seq, d, 10000.0, stream()))
    C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    ok(L_.optstage_op_gemm_rope(layout, A.data_ptr(), Wop.data_ptr(), C.data_ptr(), M, N, K, K, K, N, table.data_ptr(), seq, rot, stream()))
    # the unfused pair of kernels on the same operands
    C2 = torch.empty_like(C)
    ok(L_.optstage_op_gemm(BF16, B.GEMM_NT, B.EPI_STORE, A.data_ptr(), W.data_ptr(), C2.data_ptr(), 0, M, N, K, K, K, N, stream()))
    packed = (N // d) % 4 == 0 and rot == N // 4 * 3          # a packed qkv row: n_q = 2 n_kv query heads, n_kv key and value heads
    if packed:
        ok(L_.optstage_op_rope(BF16, C2.data_ptr(), C2.data_ptr(), table.data_ptr(), M, seq, N // d // 2, N // d // 4, d, 0, stream()))
    torch.cuda.synchronize()
    ref = a @ w.T
    heads = ref.reshape(M, N // d, d).copy()
    for s0 in range(0, M, seq):
        s1 = min(M, s0 + seq)
        heads[s0:s1, : rot // d] = O.rope_apply(heads[s0:s1, : rot // d], 10000.0)[: s1 - s0]
    ref = heads.reshape(M, N)
    assert rel_err(host(C), ref) < TOL[BF16] / 4 and rms_err(host(C), ref) < TOL[BF16] / 8
    if packed:            # against the two separate kernels: the same numbers up to the one extra rounding those make
        assert rms_err(host(C), host(C2)) < TOL[BF16] / 8
    # a shape the direct kernel does not serve, a head split by a tile, a missing table: refused, nothing written
    Z = torch.zeros(64, 256, dtype=torch.bfloat16, device="cuda")
    assert L_.optstage_op_gemm_rope(0, A.data_ptr(), W.data_ptr(), Z.data_ptr(), 64, 256, K, K, K, 256, table.data_ptr(), seq, 256, stream()) == B.E_ARG
    assert L_.optstage_op_gemm_rope(0, A.data_ptr(), W.data_ptr(), C.data_ptr(), M, N, K, K, K, N, table.data_ptr(), seq, 192, stream()) == B.E_ARG
    assert L_.optstage_op_gemm_rope(0, A.data_ptr(), W.data_ptr(), C.data_ptr(), M, N, K, K, K, N, 0, seq, rot, stream()) == B.E_ARG
    torch.cuda.synchronize()
    assert float(Z.float().abs().sum()) == 0.0


@pytest.mark.parametrize("M,f,K", [(2000, 2048, 192), (4096, 1024, 256), (2048, 2304, 64)])
def test_gate_up_projection_with_the_activation_in_the_epilogue(M, f, K):
    a = q(RNG.standard_normal((M, K)), BF16)
    w = q(0.15 * RNG.standard_normal((2 * f, K)), BF16)
    A, W = dev(a, BF16), dev(w, BF16)
    L_ = lib()
    Wp = torch.empty(2 * f * K, dtype=torch.bfloat16, device="cuda")
    ok(L_.optstage_op_weight_slabs(W.data_ptr(), Wp.data_ptr(), 2 * f, K, 2, stream()))
    GU = torch.full((M, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    ACT = torch.full((M, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    ok(L_.optstage_op_gemm_swiglu(A.data_ptr(), Wp.data_ptr(), GU.data_ptr(), ACT.data_ptr(), M, f, K, K, stream()))
    torch.cuda.synchronize()
    gu = a @ w.T
    assert rel_err(host(GU), gu) < TOL[BF16] / 4 and rms_err(host(GU), gu) < TOL[BF16] / 8       # plain [gate | up] layout
    act = O.swiglu_fwd(gu)
    assert rel_err(host(ACT), act) < TOL[BF16] / 4 and rms_err(host(ACT), act) < TOL[BF16] / 8
    # the stored gate / up tensor is what the separate projection stores, bit for bit
    GU2 = torch.empty_like(GU)
    ok(L_.optstage_op_gemm(BF16, B.GEMM_NT, B.EPI_STORE, A.data_ptr(), W.data_ptr(), GU2.data_ptr(), 0, M, 2 * f, K, K, K, 2 * f, stream()))
    torch.cuda.synchronize()
    assert torch.equal(GU, GU2)
    assert L_.optstage_op_gemm_swiglu(A.data_ptr(), Wp.data_ptr(), GU.data_ptr(), ACT.data_ptr(), M, f + 64, K, K, stream()) == B.E_ARG
    assert L_.optstage_op_gemm_swiglu(A.data_ptr(), Wp.data_ptr(), GU.data_ptr(), 0, M, f, K, K, stream()) == B.E_ARG
    assert L_.optstage_op_weight_slabs(W.data_ptr(), Wp.data_ptr(), 2 * f - 128, K, 2, stream()) == B.E_ARG
