"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the exact GEMM,
attention and stage launches of the Llama bf16 workload (hidden 4096, 32 heads x 128, ffn 11008, seq 4096),
checked on outputs the oracle can compute one by one (sampled GEMM elements, whole attention heads, one
whole layer), plus properties that hold at any size (schedule independence, accounting)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import schedule as S
from oracle import stage_fp64 as O
from paper_2510_05186_amd import binding as B
from paper_2510_05186_amd.stage import Stage
from stage_inputs import configs as CFG
from stage_inputs import schedules as G
from stage_inputs import tensors as T
from gpu_util import TOL, close, report, host, ok, oracle_shape, oracle_weights, rel_err, stream

pytestmark = pytest.mark.gpu
BF16 = 1


def dev_randn(shape, seed, scale=1.0):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * scale).bfloat16().contiguous()


@pytest.mark.parametrize("name,M,N,K,epi", [
    ("qkv", 4096, 12288, 4096, B.EPI_STORE), ("gate_up", 4096, 22016, 4096, B.EPI_STORE),
    ("down_resid", 4096, 4096, 11008, B.EPI_RESID), ("dn2", 4096, 4096, 22016, B.EPI_STORE),
    ("cfg4_up", 4096, 57344, 8192, B.EPI_STORE), ("cfg5_qkv", 16384, 15360, 5120, B.EPI_STORE),
])
def test_gemm_nt_full_size_sampled(name, M, N, K, epi):
    A, W = dev_randn((M, K), 1), dev_randn((N, K), 2, 0.02)
    R = dev_randn((M, N), 3) if epi == B.EPI_RESID else None
    C = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    ok(B.lib().optstage_op_gemm(BF16, B.GEMM_NT, epi, A.data_ptr(), W.data_ptr(), C.data_ptr(), R.data_ptr() if R is not None else 0, M, N, K, K, K, N, stream()))
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    # whole rows / columns at the tile corners and edges plus random elements
    ms = np.concatenate([[0, 255, 256, M - 1], rng.integers(0, M, 28)])
    ns = np.concatenate([[0, 255, 256, N - 1], rng.integers(0, N, 28)])
    a = host(A[torch.as_tensor(ms, device="cuda")])
    w = host(W[torch.as_tensor(ns, device="cuda")])
    ref = a @ w.T
    got = host(C[torch.as_tensor(ms, device="cuda")][:, torch.as_tensor(ns, device="cuda")])
    if R is not None:
        ref = ref + host(R[torch.as_tensor(ms, device="cuda")][:, torch.as_tensor(ns, device="cuda")])
    assert rel_err(got, ref) < TOL[BF16]
    assert torch.isfinite(C.float()).all()


@pytest.mark.parametrize("name,layout,M,N,K", [
    ("nt_a_3gib", B.GEMM_NT, 98304, 512, 16384),      # byte offsets past 2^31 on the direct path (32-bit buffer offsets)
    ("nt_a_5gib", B.GEMM_NT, 163840, 512, 16384),     # operand beyond the direct path's 4 GiB reach: register-staged kernel
    ("tn_a_3gib", B.GEMM_TN, 393216, 256, 4096),      # dY [K, M] of 3 GiB, rows 768 KiB apart
    ("tn_a_5gib", B.GEMM_TN, 655360, 256, 4096),
])
def test_gemm_operands_of_several_gib_sampled(name, layout, M, N, K):
    """Largest operands the kernels address: sampled output rows (first, last, tile edges, random) against fp64
    products of the same rows; for TN with a non-zero accumulator to start from."""
    rng = np.random.default_rng(17)
    ms = np.unique(np.concatenate([[0, 255, 256, M - 257, M - 256, M - 1], rng.integers(0, M, 26)]))
    mt = torch.as_tensor(ms, device="cuda")
    if layout == B.GEMM_NT:
        A, W = dev_randn((M, K), 21), dev_randn((N, K), 22, 0.02)
        C = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
        ok(B.lib().optstage_op_gemm(BF16, layout, B.EPI_STORE, A.data_ptr(), W.data_ptr(), C.data_ptr(), 0, M, N, K, K, K, N, stream()))
        torch.cuda.synchronize()
        ref = host(A[mt]) @ host(W).T
        assert rel_err(host(C[mt]), ref) < TOL[BF16]
        assert torch.isfinite(C.float()).all()
    else:
        DY, X = dev_randn((K, M), 23, 1e-3), dev_randn((K, N), 24)
        C = torch.full((M, N), 0.25, dtype=torch.float32, device="cuda")
        ok(B.lib().optstage_op_gemm(BF16, layout, B.EPI_ACCUM, DY.data_ptr(), X.data_ptr(), C.data_ptr(), 0, M, N, K, M, N, N, stream()))
        torch.cuda.synchronize()
        ref = 0.25 + host(DY[:, mt]).T @ host(X)
        assert rel_err(host(C[mt]), ref) < 1e-4
        assert torch.isfinite(C).all()


@pytest.mark.parametrize("name,M,N,K", [("dW_gu", 22016, 4096, 4096), ("dW_d", 4096, 11008, 4096), ("cfg5_dW_qkv", 15360, 5120, 16384)])
def test_gemm_tn_full_size_sampled(name, M, N, K):
    DY, X = dev_randn((K, M), 11, 1e-3), dev_randn((K, N), 12)
    C = torch.zeros(M, N, dtype=torch.float32, device="cuda")
    ok(B.lib().optstage_op_gemm(BF16, B.GEMM_TN, B.EPI_ACCUM, DY.data_ptr(), X.data_ptr(), C.data_ptr(), 0, M, N, K, M, N, N, stream()))
    torch.cuda.synchronize()
    rng = np.random.default_rng(6)
    ms = np.concatenate([[0, 255, 256, M - 1], rng.integers(0, M, 28)])
    ns = np.concatenate([[0, 255, 256, N - 1], rng.integers(0, N, 28)])
    dy = host(DY[:, torch.as_tensor(ms, device="cuda")])
    x = host(X[:, torch.as_tensor(ns, device="cuda")])
    got = host(C[torch.as_tensor(ms, device="cuda")][:, torch.as_tensor(ns, device="cuda")])
    assert rel_err(got, dy.T @ x) < 1e-4


@pytest.mark.parametrize("seq,nq,nkv,heads", [(4096, 32, 32, (0, 31)), (4096, 64, 8, (8, 15, 63)), (16384, 40, 40, (39,))])
def test_attention_full_size_whole_heads(seq, nq, nkv, heads):
    d = 128
    w = (nq + 2 * nkv) * d
    QKV, DO = dev_randn((seq, w), 21), dev_randn((seq, nq * d), 22, 1e-2)
    Ot = torch.empty(seq, nq * d, dtype=torch.bfloat16, device="cuda")
    LSE = torch.empty(nq * seq, dtype=torch.float32, device="cuda")
    lib = B.lib()
    ok(lib.optstage_op_attn_fwd(BF16, QKV.data_ptr(), Ot.data_ptr(), LSE.data_ptr(), seq, 1, nq, nkv, d, stream()))
    DQKV = torch.zeros_like(QKV)
    WS = torch.empty(lib.optstage_op_attn_bwd_ws_floats(seq, 1, nq, nkv, d), dtype=torch.float32, device="cuda")
    ok(lib.optstage_op_attn_bwd(BF16, QKV.data_ptr(), Ot.data_ptr(), DO.data_ptr(), LSE.data_ptr(), DQKV.data_ptr(), WS.data_ptr(), seq, 1, nq, nkv, d, stream()))
    torch.cuda.synchronize()
    rep = nq // nkv
    chunk = 2048
    for a in heads:
        g = a * nkv // nq
        q = host(QKV[:, a * d:(a + 1) * d]).reshape(seq, 1, d)
        k = host(QKV[:, (nq + g) * d:(nq + g + 1) * d]).reshape(seq, 1, d)
        v = host(QKV[:, (nq + nkv + g) * d:(nq + nkv + g + 1) * d]).reshape(seq, 1, d)
        o_g = host(Ot[:, a * d:(a + 1) * d])
        o, lse = O.attention_fwd(q, k, v, attn_chunk=chunk)
        assert rel_err(o_g, o[:, 0]) < TOL[BF16]
        assert np.max(np.abs(host(LSE).reshape(nq, seq)[a] - lse[0])) < 2e-2
        do = host(DO[:, a * d:(a + 1) * d]).reshape(seq, 1, d)
        dq, _, _ = O.attention_bwd(q, k, v, o_g.reshape(seq, 1, d), do, attn_chunk=chunk)
        assert rel_err(host(DQKV[:, a * d:(a + 1) * d]), dq[:, 0]) < TOL[BF16]
    # dK / dV of one kv head need every q head of its group
    g = heads[-1] * nkv // nq
    qs = host(QKV[:, g * rep * d:(g + 1) * rep * d]).reshape(seq, rep, d)
    k = host(QKV[:, (nq + g) * d:(nq + g + 1) * d]).reshape(seq, 1, d)
    v = host(QKV[:, (nq + nkv + g) * d:(nq + nkv + g + 1) * d]).reshape(seq, 1, d)
    og = host(Ot[:, g * rep * d:(g + 1) * rep * d]).reshape(seq, rep, d)
    dog = host(DO[:, g * rep * d:(g + 1) * rep * d]).reshape(seq, rep, d)
    _, dk, dv = O.attention_bwd(qs, k, v, og, dog, attn_chunk=chunk)
    assert rel_err(host(DQKV[:, (nq + g) * d:(nq + g + 1) * d]), dk[:, 0]) < TOL[BF16]
    assert rel_err(host(DQKV[:, (nq + nkv + g) * d:(nq + nkv + g + 1) * d]), dv[:, 0]) < TOL[BF16]


@pytest.mark.parametrize("base", [CFG.CFG2, CFG.CFG6, CFG.CFG4, CFG.CFG5], ids=lambda c: c.name)
def test_one_whole_layer_at_full_shape_against_oracle(base):
    """cfg 4 (hidden 8192, 64 query heads on 8 kv heads, MLP 28672) takes the oracle about 22 TFLOP in fp64, the
    long-sequence stage (16384 tokens, hidden 5120) about 41."""
    print(f"whole layer of {base.name}: GPU F/B/W, then the fp64 oracle on the host", flush=True)
    cfg = replace(base, name=base.name + "_one_layer", n_layers=1, n_microbatches=1)
    ws = T.stage_weights(cfg)
    st = Stage(cfg)
    st.set_weights(ws)
    x, dy = T.stage_input(cfg, 0), T.output_grad(cfg, 0)
    st.bind(0, x, dy)
    st.run([("F", 0), ("B", 0), ("W", 0)])
    st.synchronize()
    y, dx, dW, dn = O.stage_fbw(oracle_shape(cfg), oracle_weights(ws), x.astype(np.float64), dy.astype(np.float64), attn_chunk=1024)
    close(host(st.y[0]), y, BF16, f"{base.name} one layer y")
    close(host(st.dx[0]), dx, BF16, f"{base.name} one layer dx")
    for name in ("wqkv", "wo", "wgu", "wd"):
        close(host(st.grads[0][name]), dW[0][name], BF16, f"{base.name} one layer dW {name}")
    for name in dn[0]:                     # norm gains (and biases for LayerNorm)
        close(host(st.grads[0][name]), dn[0][name], BF16, f"{base.name} one layer d{name}")
    report()
    assert st.stats().live_bytes == 0
    st.close()


def test_full_size_schedule_independence_and_accounting():
    # the benchmark's stage (4 layers, full shapes) with 3 micro-batches under two different valid orders:
    # bitwise identical results, and the library's accounting equals the oracle's for both lists
    cfg = replace(CFG.CFG2, name="cfg2_m3", n_microbatches=3)
    t = S.memory_table(cfg.family, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn, cfg.seq, 2)
    lists = [G.split_bw_greedy(cfg.n_stages, 3)[cfg.stage_index],
             [("F", 0), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("F", 2), ("W", 1), ("B", 2), ("W", 2)]]
    g = torch.Generator(device="cuda")
    weights = []
    for l in range(cfg.n_layers):
        w = {}
        for i, (name, shape) in enumerate(T.weight_shapes(cfg).items()):
            g.manual_seed(1000 + 10 * l + i)
            tns = torch.randn(shape, generator=g, device="cuda") * 0.02
            w[name] = (tns + 1.0 if name in ("g1", "g2") else tns).bfloat16().contiguous()
        weights.append(w)
    xs = [dev_randn((cfg.seq, cfg.hidden), 50 + j) for j in range(3)]
    dys = [dev_randn((cfg.seq, cfg.hidden), 60 + j, 1e-3) for j in range(3)]
    outs = []
    for ev in lists:
        S.check_order(ev, 3, cfg.n_layers)
        peak, trace = S.account_memory(ev, cfg.n_layers, t)
        st = Stage(cfg)
        st.set_weights_device(weights)
        for j in range(3):
            st.bind(j, xs[j], dys[j])
        st.run(ev)
        st.synchronize()
        s = st.stats()
        assert s.peak_bytes == peak and s.live_bytes == 0
        outs.append(([st.y[j].clone() for j in range(3)], [st.dx[j].clone() for j in range(3)],
                     {(l, n): v.clone() for l in range(cfg.n_layers) for n, v in st.grads[l].items()}))
        assert all(torch.isfinite(y.float()).all() for y in outs[-1][0])
        st.close()
        del st
        torch.cuda.empty_cache()
    for j in range(3):
        assert torch.equal(outs[0][0][j], outs[1][0][j]) and torch.equal(outs[0][1][j], outs[1][1][j])
    for key in outs[0][2]:
        # W ops run in the same micro-batch order in both lists, so even the fp32 accumulation order is equal
        assert torch.equal(outs[0][2][key], outs[1][2][key]), key
