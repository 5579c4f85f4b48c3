"""Pins for oracle/stage_fp64.py — none of them re-types the oracle's formulas.

* central finite differences of <y, dy> for every gradient (x, every weight, norm params)
* torch CPU float64 autograd of the same block built from stock library ops
  (layer_norm, rms_norm, scaled_dot_product_attention, gelu, silu) — an independent
  unsplit backward, so "B then W equals the unsplit backward" is checked against it
* invariants / closed forms of every non-linear piece
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import stage_fp64 as O

RNG = np.random.default_rng(1234)


def tiny_shape(family, n_q=2, n_kv=2, L=2):
    return O.StageShape(family=family, n_layers=L, hidden=16, n_q_heads=n_q, n_kv_heads=n_kv,
                        head_dim=8, ffn=24, seq=8)


def rand_weights(sh, scale=0.3):
    h, f = sh.hidden, sh.ffn
    up = 2 * f if sh.family == O.LLAMA else f
    ws = []
    for _ in range(sh.n_layers):
        w = {"g1": 1 + 0.1 * RNG.standard_normal(h), "g2": 1 + 0.1 * RNG.standard_normal(h),
             "wqkv": scale * RNG.standard_normal((sh.qkv_width, h)),
             "wo": scale * RNG.standard_normal((h, sh.n_q_heads * sh.head_dim)),
             "wgu": scale * RNG.standard_normal((up, h)),
             "wd": scale * RNG.standard_normal((h, f))}
        if sh.family == O.GPT:
            w["b1"] = 0.1 * RNG.standard_normal(h)
            w["b2"] = 0.1 * RNG.standard_normal(h)
        ws.append(w)
    return ws


# ---------------------------------------------------------------- finite differences
@pytest.mark.parametrize("family,n_q,n_kv", [(O.GPT, 2, 2), (O.LLAMA, 2, 2), (O.LLAMA, 4, 2)])
def test_finite_differences(family, n_q, n_kv):
    sh = tiny_shape(family, n_q, n_kv)
    ws = rand_weights(sh)
    x = RNG.standard_normal((sh.seq, sh.hidden))
    dy = RNG.standard_normal((sh.seq, sh.hidden))
    _, dx, dW, dnorm = O.stage_fbw(sh, ws, x, dy)

    def loss():
        y, _ = O.stage_forward(sh, ws, x)
        return float(np.sum(y * dy))

    def fd(arr, idx, eps=1e-6):
        old = arr[idx]
        arr[idx] = old + eps
        lp = loss()
        arr[idx] = old - eps
        lm = loss()
        arr[idx] = old
        return (lp - lm) / (2 * eps)

    def check(arr, grad, n=6):
        flat = [np.unravel_index(i, arr.shape) for i in RNG.choice(arr.size, size=min(n, arr.size), replace=False)]
        for idx in flat:
            num = fd(arr, idx)
            assert abs(num - grad[idx]) <= 1e-6 * max(1.0, abs(num)) + 1e-7, (idx, num, grad[idx])

    check(x, dx, n=10)
    for l in range(sh.n_layers):
        for name in ("wqkv", "wo", "wgu", "wd"):
            check(ws[l][name], dW[l][name])
        for name, g in dnorm[l].items():
            check(ws[l][name], g)


# ---------------------------------------------------------------- torch autograd (library routines)
def torch_rope(u, base):
    # complex-multiplication form: pair (k, k + d/2) is one complex number rotated by t * theta_k
    s, n, d = u.shape
    theta = base ** (-torch.arange(0, d // 2, dtype=torch.float64) * 2.0 / d)
    ang = torch.outer(torch.arange(s, dtype=torch.float64), theta)
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    z = torch.complex(u[..., : d // 2], u[..., d // 2:]) * rot
    return torch.cat([z.real, z.imag], dim=-1)


def torch_stage(sh, tw, x, st=lambda t: t):
    """st: applied to the output of every op (identity by default)."""
    nq, nkv, d = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    s = x.shape[0]
    x = st(x)
    for w in tw:
        if sh.family == O.LLAMA:
            n1 = st(F.rms_norm(x, (sh.hidden,), w["g1"], sh.norm_eps))
        else:
            n1 = st(F.layer_norm(x, (sh.hidden,), w["g1"], w["b1"], sh.norm_eps))
        qkv = st(F.linear(n1, w["wqkv"]))
        q = qkv[:, : nq * d].reshape(s, nq, d)
        k = qkv[:, nq * d: (nq + nkv) * d].reshape(s, nkv, d)
        v = qkv[:, (nq + nkv) * d:].reshape(s, nkv, d)
        if sh.family == O.LLAMA:
            q, k = st(torch_rope(q, sh.rope_base)), st(torch_rope(k, sh.rope_base))
        rep = nq // nkv
        kk = k.repeat_interleave(rep, dim=1)
        vv = v.repeat_interleave(rep, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], kk.transpose(0, 1)[None],
                                           vv.transpose(0, 1)[None], is_causal=True)[0]
        o = st(o.transpose(0, 1).reshape(s, nq * d))
        xm = st(x + F.linear(o, w["wo"]))
        if sh.family == O.LLAMA:
            n2 = st(F.rms_norm(xm, (sh.hidden,), w["g2"], sh.norm_eps))
            gu = st(F.linear(n2, w["wgu"]))
            a = st(F.silu(gu[:, : sh.ffn]) * gu[:, sh.ffn:])
        else:
            n2 = st(F.layer_norm(xm, (sh.hidden,), w["g2"], w["b2"], sh.norm_eps))
            a = st(F.gelu(st(F.linear(n2, w["wgu"]))))
        x = st(xm + F.linear(a, w["wd"]))
    return x


@pytest.mark.parametrize("family,n_q,n_kv", [(O.GPT, 2, 2), (O.LLAMA, 2, 2), (O.LLAMA, 4, 1), (O.LLAMA, 4, 2)])
def test_matches_torch_autograd_unsplit_backward(family, n_q, n_kv):
    sh = tiny_shape(family, n_q, n_kv)
    ws = rand_weights(sh)
    x = RNG.standard_normal((sh.seq, sh.hidden))
    dy = RNG.standard_normal((sh.seq, sh.hidden))
    y, dx, dW, dnorm = O.stage_fbw(sh, ws, x, dy)

    tw = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in w.items()} for w in ws]
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = torch_stage(sh, tw, tx)
    ty.backward(torch.tensor(dy))
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    for l in range(sh.n_layers):
        for name in ("wqkv", "wo", "wgu", "wd"):
            np.testing.assert_allclose(dW[l][name], tw[l][name].grad.numpy(), rtol=1e-10, atol=1e-12)
        for name, g in dnorm[l].items():
            np.testing.assert_allclose(g, tw[l][name].grad.numpy(), rtol=1e-10, atol=1e-12)


def test_w_is_order_independent_and_sums_over_microbatches():
    # dW of the iteration is the sum of per-micro-batch dW, whatever the order W ops run in
    sh = tiny_shape(O.LLAMA, 4, 2)
    ws = rand_weights(sh)
    xs = [RNG.standard_normal((sh.seq, sh.hidden)) for _ in range(3)]
    dys = [RNG.standard_normal((sh.seq, sh.hidden)) for _ in range(3)]
    stashes = []
    for x, dy in zip(xs, dys):
        _, saved = O.stage_forward(sh, ws, x)
        _, st, _ = O.stage_backward_input(sh, ws, saved, dy)
        stashes.append(st)
    tot_a = None
    for j in (2, 0, 1):
        dW = O.stage_backward_weight(stashes[j])
        tot_a = dW if tot_a is None else [{k: a[k] + b[k] for k in a} for a, b in zip(tot_a, dW)]
    # torch: one backward over the summed loss
    tw = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in w.items()} for w in ws]
    loss = sum((torch_stage(sh, tw, torch.tensor(x)) * torch.tensor(dy)).sum() for x, dy in zip(xs, dys))
    loss.backward()
    for l in range(sh.n_layers):
        for name in ("wqkv", "wo", "wgu", "wd"):
            np.testing.assert_allclose(tot_a[l][name], tw[l][name].grad.numpy(), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("family", [O.GPT, O.LLAMA])
def test_micro_batch_of_several_sequences_is_the_sequences_side_by_side(family):
    """A micro-batch of size b is b sequences stored one after the other: nothing couples them (attention is
    causal within a sequence, rotary positions restart), so y and dx are the per-sequence results stacked and
    every parameter gradient is the sum over the sequences.  torch autograd on the stacked loss agrees."""
    sh = tiny_shape(family, 4, 2)
    ws = rand_weights(sh)
    b = 3
    x = RNG.standard_normal((b * sh.seq, sh.hidden))
    dy = RNG.standard_normal((b * sh.seq, sh.hidden))
    y, dx, dW, dn = O.stage_fbw(sh, ws, x, dy)
    parts = [O.stage_fbw(sh, ws, x[i * sh.seq:(i + 1) * sh.seq], dy[i * sh.seq:(i + 1) * sh.seq]) for i in range(b)]
    np.testing.assert_allclose(y, np.concatenate([p[0] for p in parts]), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dx, np.concatenate([p[1] for p in parts]), rtol=1e-12, atol=1e-13)
    for l in range(sh.n_layers):
        for name in dW[l]:
            np.testing.assert_allclose(dW[l][name], sum(p[2][l][name] for p in parts), rtol=1e-11, atol=1e-12)
        for name in dn[l]:
            np.testing.assert_allclose(dn[l][name], sum(p[3][l][name] for p in parts), rtol=1e-11, atol=1e-12)
    # the saved softmax statistics are laid out [sequence, head, position]
    saved = O.stage_forward(sh, ws, x)[1]
    for i in range(b):
        one = O.stage_forward(sh, ws, x[i * sh.seq:(i + 1) * sh.seq])[1]
        for l in range(sh.n_layers):
            assert saved[l]["lse"].shape == (b, sh.n_q_heads, sh.seq)
            np.testing.assert_allclose(saved[l]["lse"][i], one[l]["lse"][0], rtol=1e-12)
    # coupling test: changing the last sequence leaves the first one's output alone, changing the first token of a
    # sequence changes the rest of that sequence
    x2 = x.copy()
    x2[2 * sh.seq] += 1.0
    y2 = O.stage_forward(sh, ws, x2)[0]
    assert np.array_equal(y2[:2 * sh.seq], y[:2 * sh.seq])
    assert np.all(np.abs(y2[2 * sh.seq:] - y[2 * sh.seq:]).max(axis=1) > 0)
    tw = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in w.items()} for w in ws]
    loss = sum((torch_stage(sh, tw, torch.tensor(x[i * sh.seq:(i + 1) * sh.seq])) * torch.tensor(dy[i * sh.seq:(i + 1) * sh.seq])).sum()
               for i in range(b))
    loss.backward()
    for l in range(sh.n_layers):
        for name in ("wqkv", "wo", "wgu", "wd"):
            np.testing.assert_allclose(dW[l][name], tw[l][name].grad.numpy(), rtol=1e-10, atol=1e-12)
    with pytest.raises(ValueError):
        O.stage_forward(sh, ws, x[:sh.seq + 1])


# ---------------------------------------------------------------- storage precision
def test_round_bf16_is_round_to_nearest_even_on_eight_significant_bits():
    # by hand: the spacing of bf16 in [1, 2) is 2^-7; halfway cases go to the even neighbour
    u = 2.0 ** -7
    cases = {1.0: 1.0, 1.0 + u / 2: 1.0, 1.0 + 3 * u / 2: 1.0 + 2 * u, 1.0 + u / 2 + 1e-9: 1.0 + u, 1.0 + 0.49 * u: 1.0,
             -(1.0 + 3 * u / 2): -(1.0 + 2 * u), 0.0: 0.0, 255.5: 256.0}
    for a, want in cases.items():
        assert O.round_bf16(np.array([a]))[0] == want, a
    # against two independent routines on random single-precision values: the bit-pattern rounding of the input
    # generators and torch's cast
    from stage_inputs import tensors as T
    a = (RNG.standard_normal(200000) * np.exp(RNG.uniform(-20, 20, 200000))).astype(np.float32)
    got = O.round_bf16(a.astype(np.float64))
    np.testing.assert_array_equal(got, T.quantize(a, 1).astype(np.float64))
    np.testing.assert_array_equal(got, torch.from_numpy(a).bfloat16().double().numpy())
    np.testing.assert_array_equal(O.round_bf16(got), got)                    # idempotent


class _RoundBoth(torch.autograd.Function):
    """bf16 rounding of a tensor on the way forward and of its gradient on the way back (torch's own cast)."""
    @staticmethod
    def forward(ctx, t):
        return t.to(torch.bfloat16).to(torch.float64)

    @staticmethod
    def backward(ctx, g):
        return g.to(torch.bfloat16).to(torch.float64)


@pytest.mark.parametrize("family,n_q,n_kv", [(O.GPT, 2, 2), (O.LLAMA, 2, 2), (O.LLAMA, 4, 2)])
def test_storage_rounding_sits_at_every_op_boundary_and_nowhere_else(family, n_q, n_kv):
    """store=round_bf16 against an independently built model: the stock-op torch block with a node after every op
    that rounds the tensor going forward and its gradient going back.  A rounding the oracle misses, adds or puts
    elsewhere moves the results by 2^-9 relative somewhere; the two agree to 1e-10."""
    sh = tiny_shape(family, n_q, n_kv)
    ws = [{k: O.round_bf16(v) for k, v in w.items()} for w in rand_weights(sh)]
    x = O.round_bf16(RNG.standard_normal((sh.seq, sh.hidden)))
    dy = O.round_bf16(RNG.standard_normal((sh.seq, sh.hidden)))
    y, dx, dW, dnorm = O.stage_fbw(sh, ws, x, dy, store=O.round_bf16)
    for t in (y, dx):
        np.testing.assert_array_equal(O.round_bf16(t), t)                    # what leaves the stage is bf16
    tw = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in w.items()} for w in ws]
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = torch_stage(sh, tw, tx, st=_RoundBoth.apply)
    ty.backward(torch.tensor(dy))
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    for l in range(sh.n_layers):
        for name in ("wqkv", "wo", "wgu", "wd"):
            np.testing.assert_allclose(dW[l][name], tw[l][name].grad.numpy(), rtol=1e-10, atol=1e-12)
        for name, g in dnorm[l].items():
            np.testing.assert_allclose(g, tw[l][name].grad.numpy(), rtol=1e-10, atol=1e-12)
    # the rounded chain is a different function from the exact one, and not far from it
    y0, dx0, _, _ = O.stage_fbw(sh, ws, x, dy)
    for a, b in ((y, y0), (dx, dx0)):
        rel = np.max(np.abs(a - b)) / np.max(np.abs(b))
        assert 1e-5 < rel < 5e-2
    # every saved activation is a bf16 value
    _, saved = O.stage_forward(sh, ws, x, store=O.round_bf16)
    for sv in saved:
        for k in ("n1", "qkv", "o", "x_mid", "n2", "gu", "a"):
            np.testing.assert_array_equal(O.round_bf16(sv[k]), sv[k])


# ---------------------------------------------------------------- attention invariants
def test_attention_invariants():
    s, nq, nkv, d = 12, 4, 2, 8
    q = RNG.standard_normal((s, nq, d))
    k = RNG.standard_normal((s, nkv, d))
    v = RNG.standard_normal((s, nkv, d))
    o, lse = O.attention_fwd(q, k, v)
    # row 0 attends only to itself
    for a in range(nq):
        np.testing.assert_allclose(o[0, a], v[0, a * nkv // nq], rtol=1e-14)
    # probabilities: rows sum to 1, strictly causal zeros, consistent with lse
    P = O.attention_probs(q, k, 3, 1)
    np.testing.assert_allclose(P.sum(1), 1.0, rtol=1e-13)
    assert np.all(np.triu(P, 1) == 0)
    S = (q[:, 3] @ k[:, 1].T) / math.sqrt(d)
    np.testing.assert_allclose(np.diag(P), np.exp(np.diag(S) - lse[3]), rtol=1e-12)
    # query-chunked evaluation equals the full-matrix evaluation
    o2, lse2 = O.attention_fwd(q, k, v, attn_chunk=5)
    np.testing.assert_allclose(o2, o, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(lse2, lse, rtol=1e-13)
    do = RNG.standard_normal(o.shape)
    g1 = O.attention_bwd(q, k, v, o, do)
    g2 = O.attention_bwd(q, k, v, o, do, attn_chunk=5)
    for a_, b_ in zip(g1, g2):
        np.testing.assert_allclose(a_, b_, rtol=1e-12, atol=1e-14)
    # grouped kv == multi-head attention on replicated kv heads, with dK/dV summed per group
    kk, vv = np.repeat(k, nq // nkv, axis=1), np.repeat(v, nq // nkv, axis=1)
    o3, _ = O.attention_fwd(q, kk, vv)
    np.testing.assert_allclose(o3, o, rtol=1e-13)
    dq3, dk3, dv3 = O.attention_bwd(q, kk, vv, o3, do)
    np.testing.assert_allclose(dq3, g1[0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dk3.reshape(s, nkv, nq // nkv, d).sum(2), g1[1], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dv3.reshape(s, nkv, nq // nkv, d).sum(2), g1[2], rtol=1e-12, atol=1e-14)


def test_attention_single_token_is_identity_on_v():
    q = RNG.standard_normal((1, 2, 4))
    k = RNG.standard_normal((1, 2, 4))
    v = RNG.standard_normal((1, 2, 4))
    o, lse = O.attention_fwd(q, k, v)
    np.testing.assert_allclose(o, v)
    np.testing.assert_allclose(lse[:, 0], np.einsum("hd,hd->h", q[0], k[0]) / 2.0)


def test_attention_uniform_scores_average_prefix():
    # zero queries -> uniform causal probabilities -> o_t is the running mean of v
    s, d = 9, 4
    q = np.zeros((s, 1, d))
    k = RNG.standard_normal((s, 1, d))
    v = RNG.standard_normal((s, 1, d))
    o, lse = O.attention_fwd(q, k, v)
    np.testing.assert_allclose(o[:, 0], np.cumsum(v[:, 0], 0) / np.arange(1, s + 1)[:, None], rtol=1e-13)
    np.testing.assert_allclose(lse[0], np.log(np.arange(1, s + 1)), rtol=1e-13, atol=1e-15)


def test_attention_backward_row_term_by_definition_equals_the_output_form():
    # D_t = sum_t' P_tt' dP_tt' (o=None) and D_t = <dO_t, o_t> with the exact forward output are the same number
    s, nq, nkv, d = 12, 4, 2, 8
    q, do = RNG.standard_normal((s, nq, d)), RNG.standard_normal((s, nq, d))
    k, v = RNG.standard_normal((s, nkv, d)), RNG.standard_normal((s, nkv, d))
    o, _ = O.attention_fwd(q, k, v)
    for a, b in zip(O.attention_bwd(q, k, v, o, do), O.attention_bwd(q, k, v, None, do, attn_chunk=5)):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- rotary
def test_rotary_properties():
    s, n, d = 10, 3, 8
    u = RNG.standard_normal((s, n, d))
    r = O.rope_apply(u, 10000.0)
    # per-pair norm preserved, position 0 untouched
    np.testing.assert_allclose(r[..., : d // 2] ** 2 + r[..., d // 2:] ** 2,
                               u[..., : d // 2] ** 2 + u[..., d // 2:] ** 2, rtol=1e-13)
    np.testing.assert_allclose(r[0], u[0])
    # relative-position property: <rot_t q, rot_t' k> depends only on t - t'
    qv, kv = RNG.standard_normal(d), RNG.standard_normal(d)
    Q = O.rope_apply(np.tile(qv, (s, 1, 1)), 10000.0)[:, 0]
    K = O.rope_apply(np.tile(kv, (s, 1, 1)), 10000.0)[:, 0]
    G = Q @ K.T
    for off in range(-3, 4):
        diag = np.diagonal(G, off)
        np.testing.assert_allclose(diag, diag[0], rtol=1e-12, atol=1e-13)
    # explicit value: angle t * base^(-2k/d) for the pair (k, k + d/2)
    t, kk = 7, 2
    ang = t * 10000.0 ** (-2 * kk / d)
    e = np.zeros((s, 1, d))
    e[t, 0, kk] = 1.0
    out = O.rope_apply(e, 10000.0)[t, 0]
    assert abs(out[kk] - math.cos(ang)) < 1e-15 and abs(out[kk + d // 2] - math.sin(ang)) < 1e-15
    # backward map is the transpose (= inverse) of the forward rotation
    np.testing.assert_allclose(O.rope_apply(r, 10000.0, sign=-1.0), u, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- norms
def test_norm_invariants():
    x = 3.0 * RNG.standard_normal((6, 32)) + 0.7
    n, r = O.rmsnorm_fwd(x, np.ones(32), 0.0)
    np.testing.assert_allclose(np.mean(n * n, 1), 1.0, rtol=1e-13)
    n, mu, r = O.layernorm_fwd(x, np.ones(32), np.zeros(32), 0.0)
    np.testing.assert_allclose(n.mean(1), 0.0, atol=1e-14)
    np.testing.assert_allclose(n.var(1), 1.0, rtol=1e-13)
    # with eps = 0 the normalised output is scale invariant, so dx is orthogonal to x
    g = 1 + 0.1 * RNG.standard_normal(32)
    dn = RNG.standard_normal(x.shape)
    _, r = O.rmsnorm_fwd(x, g, 0.0)
    dx, _ = O.rmsnorm_bwd(dn, x, r, g)
    np.testing.assert_allclose(np.sum(dx * x, 1), 0.0, atol=1e-12)
    _, mu, r = O.layernorm_fwd(x, g, np.zeros(32), 0.0)
    dx, _, db = O.layernorm_bwd(dn, x, mu, r, g)
    np.testing.assert_allclose(np.sum(dx * (x - mu), 1), 0.0, atol=1e-12)
    np.testing.assert_allclose(dx.sum(1), 0.0, atol=1e-12)       # shift invariance
    np.testing.assert_allclose(db, dn.sum(0))


# ---------------------------------------------------------------- activations
def test_activation_closed_forms():
    g = RNG.standard_normal((5, 7))
    a = O.swiglu_fwd(np.concatenate([g, np.ones_like(g)], 1))
    np.testing.assert_allclose(a, F.silu(torch.tensor(g)).numpy(), rtol=1e-13)
    assert O.gelu_fwd(np.array([0.0]))[0] == 0.0
    assert O.gelu_bwd(np.array([1.0]), np.array([0.0]))[0] == 0.5
    z = np.array([1.0])
    assert abs(O.gelu_fwd(z)[0] - 0.8413447460685429) < 1e-15      # Phi(1)
    np.testing.assert_allclose(O.gelu_fwd(g), F.gelu(torch.tensor(g)).numpy(), rtol=1e-13)
    # large |z| limits
    assert abs(O.gelu_fwd(np.array([10.0]))[0] - 10.0) < 1e-12
    assert abs(O.gelu_fwd(np.array([-10.0]))[0]) < 1e-12


def test_flop_formula_matches_workload_table():
    # 4 layers, hidden 4096, 32 heads x 128, ffn 11008, seq 4096: 1.795 / 2.002 / 1.658 TFLOP per layer
    sh = O.StageShape(O.LLAMA, 4, 4096, 32, 32, 128, 11008, 4096)
    fl = O.flops_per_microbatch(sh)
    assert abs(fl["F"] / 4 / 1e12 - 1.795) < 1e-3
    assert abs(fl["B"] / 4 / 1e12 - 2.002) < 1e-3
    assert abs(fl["W"] / 4 / 1e12 - 1.658) < 1e-3


def test_attention_with_large_scores_stays_finite_and_equals_library_softmax():
    """Scores of magnitude several hundred (exp overflows in fp64 beyond 709): the running-maximum shift keeps the
    result finite and equal to scipy's softmax of the same masked scores; lse equals scipy's logsumexp."""
    from scipy.special import logsumexp, softmax
    rng = np.random.default_rng(11)
    s, d = 12, 8
    q = 40.0 * rng.standard_normal((s, 1, d))
    k = 40.0 * rng.standard_normal((s, 1, d))
    v = rng.standard_normal((s, 1, d))
    o, lse = O.attention_fwd(q, k, v)
    sc = (q[:, 0, :] @ k[:, 0, :].T) / np.sqrt(d)
    assert np.abs(sc).max() > 800
    sc = np.where(np.tril(np.ones((s, s), dtype=bool)), sc, -np.inf)
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))
    np.testing.assert_allclose(o[:, 0, :], softmax(sc, axis=1) @ v[:, 0, :], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(lse[0], logsumexp(sc, axis=1), rtol=1e-12)
    np.testing.assert_allclose(O.attention_probs(q, k, 0, 0), softmax(sc, axis=1), rtol=1e-12, atol=1e-300)
    do = rng.standard_normal((s, 1, d))
    dq, dk, dv = O.attention_bwd(q, k, v, o, do)
    assert np.all(np.isfinite(dq)) and np.all(np.isfinite(dk)) and np.all(np.isfinite(dv))
    np.testing.assert_allclose(dv[:, 0, :], softmax(sc, axis=1).T @ do[:, 0, :], rtol=1e-10, atol=1e-12)
