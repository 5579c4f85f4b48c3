"""fp64 CPU oracle for one pipeline stage's F / B / W numerics.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module;
it is used by tests/, by __graft_entry__.smoke() and by bench.py's
cpu_baseline leg.  It shares no code with the HIP path.

What it computes (paper Sec. 2.2): a stage is a chain of layers; the forward
pass F maps the stage input to the stage output; the backward pass is split
into B (gradient w.r.t. the stage input, "backward for activation") and W
(gradient w.r.t. the weights, "backward for weights").  Sec. 2.2 writes a
stage as z = W x followed by a non-linearity; a real stage (Sec. 2.1) is N/P
consecutive transformer layers, so every linear map below follows
    forward  Y  = X W^T          (z = W x, one token per row)
    B        dX = dY W           (grad_x = W^T grad_z)
    W        dW = dY^T X         (grad_W = grad_z x^T)
and the non-linear parts (norms, rotary, attention, SwiGLU / GELU) are the
textbook definitions, written out plainly.  The paper is silent on the block
details; the readings taken here (pre-norm residual blocks, no linear biases,
eps, exact-erf GELU, half-split rotary with base 10000, 1/sqrt(d) softmax
scale, q-head a uses kv-head floor(a * n_kv / n_q)) are listed in the design
notes of this repository.

Everything is numpy float64, whole-matrix, no tiling, no fusion.  The only
concession to size is `attn_chunk`: the s x s score matrix may be evaluated
in blocks of query rows (each block still uses the plain definition).

Storage precision (`store`).  The bf16 workloads name a storage type: the
tensors that pass from one op of the layer graph to the next (each z and
sigma(z) of Sec. 2.2 and each gradient of them, which is also what the
activation-memory parameters Delta and Gamma of Eq. 7 count at two bytes per
element) are bf16 values, while the arithmetic inside an op is not limited
by it.  With store=None (default) the oracle keeps every tensor in float64:
the exact function.  With store=round_bf16 the output of every op (norm,
linear map, rotary, attention, residual add, activation, and the backward
counterpart of each) is rounded to the nearest bf16 value (ties to even)
before the next op reads it, and everything inside an op stays float64: the
exact function OF THE STORED VALUES, which is what an executor with that
storage type can be held to far more tightly than to the float64 chain (a
gradient four layers deep moves by about 1.5 % RMS under storage rounding
alone).  Norm statistics and the attention log-sum-exp stay unrounded (the
memory table holds them as fp32).

Layouts: activations are [tokens, features] row-major; linear weights are
[out_features, in_features].  The packed qkv row is [q heads | k heads |
v heads], each head `d` wide.  The packed gate/up row is [gate f | up f].

Pins (tests/test_oracle_numerics.py): central finite differences for every
gradient, B then W equals an independently written unsplit backward, torch
CPU float64 autograd of the same block built from stock library ops, and the
closed-form / invariant checks for each non-linear piece.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

try:  # exact erf for GELU; scipy is only used for this one special function
    from scipy.special import erf as _erf
except Exception:  # pragma: no cover
    _erf = np.vectorize(math.erf)

GPT = 0
LLAMA = 1


def round_bf16(a):
    """Nearest bf16 value (8 significant bits, ties to even) of every element, returned as float64.
    Written on the value, not on bit patterns: a = m 2^e with 0.5 <= |m| < 1, and m is rounded to a
    multiple of 2^-8.  The workloads' values are far from bf16's exponent limits; none are handled."""
    m, e = np.frexp(np.asarray(a, dtype=np.float64))
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def _keep(x):
    return x


@dataclass(frozen=True)
class StageShape:
    family: int          # GPT (LayerNorm, GELU, no rotary) or LLAMA (RMSNorm, rotary, SwiGLU)
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    seq: int
    norm_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def qkv_width(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim


# --------------------------------------------------------------------------
# linear maps (Sec. 2.2)
# --------------------------------------------------------------------------
def linear_fwd(x, w):
    return x @ w.T


def linear_bwd_input(dy, w):
    return dy @ w


def linear_bwd_weight(dy, x):
    return dy.T @ x


# --------------------------------------------------------------------------
# norms
# --------------------------------------------------------------------------
def rmsnorm_fwd(x, gamma, eps):
    r = 1.0 / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + eps)
    return x * r * gamma, r


def rmsnorm_bwd(dn, x, r, gamma):
    xh = x * r
    g = dn * gamma
    dx = r * (g - xh * np.mean(g * xh, axis=1, keepdims=True))
    dgamma = np.sum(dn * xh, axis=0)
    return dx, dgamma


def layernorm_fwd(x, gamma, beta, eps):
    mu = np.mean(x, axis=1, keepdims=True)
    xc = x - mu
    r = 1.0 / np.sqrt(np.mean(xc * xc, axis=1, keepdims=True) + eps)
    return xc * r * gamma + beta, mu, r


def layernorm_bwd(dn, x, mu, r, gamma):
    xh = (x - mu) * r
    g = dn * gamma
    dx = r * (g - np.mean(g, axis=1, keepdims=True) - xh * np.mean(g * xh, axis=1, keepdims=True))
    return dx, np.sum(dn * xh, axis=0), np.sum(dn, axis=0)


# --------------------------------------------------------------------------
# rotary position embedding, half-split pairing (k, k + d/2), positions 0..s-1
# --------------------------------------------------------------------------
def _rope_angles(seq, d, base):
    k = np.arange(d // 2, dtype=np.float64)
    theta = base ** (-2.0 * k / d)
    ang = np.arange(seq, dtype=np.float64)[:, None] * theta[None, :]
    return np.cos(ang), np.sin(ang)


def rope_apply(u, base, sign=1.0):
    """u: [s, n_heads, d].  sign=+1 rotates by +t*theta (forward); sign=-1 is the
    transpose of that rotation, i.e. the backward map for gradients."""
    s, _, d = u.shape
    c, sn = _rope_angles(s, d, base)
    c = c[:, None, :]
    sn = sign * sn[:, None, :]
    lo, hi = u[..., : d // 2], u[..., d // 2:]
    return np.concatenate([lo * c - hi * sn, hi * c + lo * sn], axis=-1)


# --------------------------------------------------------------------------
# causal attention with grouped kv heads
# --------------------------------------------------------------------------
def _kv_head(a, n_q, n_kv):
    return (a * n_kv) // n_q


def attention_fwd(q, k, v, attn_chunk=None):
    """q: [s, n_q, d]; k, v: [s, n_kv, d].  Returns o [s, n_q, d] and
    lse [n_q, s] (natural-log sum-exp of the scaled, masked scores)."""
    s, n_q, d = q.shape
    n_kv = k.shape[1]
    scale = 1.0 / math.sqrt(d)
    o = np.empty_like(q)
    lse = np.empty((n_q, s))
    step = s if attn_chunk is None else attn_chunk
    for a in range(n_q):
        g = _kv_head(a, n_q, n_kv)
        K, V = k[:, g, :], v[:, g, :]
        for t0 in range(0, s, step):
            t1 = min(s, t0 + step)
            S = (q[t0:t1, a, :] @ K[:t1].T) * scale
            rows = np.arange(t0, t1)[:, None]
            cols = np.arange(t1)[None, :]
            S = np.where(cols <= rows, S, -np.inf)
            m = S.max(axis=1, keepdims=True)
            e = np.exp(S - m)
            z = e.sum(axis=1, keepdims=True)
            o[t0:t1, a, :] = (e / z) @ V[:t1]
            lse[a, t0:t1] = (m + np.log(z))[:, 0]
    return o, lse


def attention_probs(q, k, a, g):
    """Full s x s probability matrix of q-head a against kv-head g."""
    s, _, d = q.shape
    S = (q[:, a, :] @ k[:, g, :].T) / math.sqrt(d)
    mask = np.tril(np.ones((s, s), dtype=bool))
    S = np.where(mask, S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    e = np.exp(S)
    return e / e.sum(axis=1, keepdims=True)


def attention_bwd(q, k, v, o, do, attn_chunk=None):
    """Softmax-attention backward by the definition dS = P o (dP - D), D_t = sum_t' P_tt' dP_tt'.
    o=None: D from that definition.  o given: D_t = <dO_t, o_t>, the same number when o is the exact forward
    output (sum_t' P_tt' dP_tt' = <dO_t, sum_t' P_tt' V_t'>); tests that feed a kernel's own stored, rounded
    output use this form to check the kernel against the inputs it really had."""
    s, n_q, d = q.shape
    n_kv = k.shape[1]
    scale = 1.0 / math.sqrt(d)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    step = s if attn_chunk is None else attn_chunk
    for a in range(n_q):
        g = _kv_head(a, n_q, n_kv)
        K, V = k[:, g, :], v[:, g, :]
        for t0 in range(0, s, step):
            t1 = min(s, t0 + step)
            S = (q[t0:t1, a, :] @ K[:t1].T) * scale
            rows = np.arange(t0, t1)[:, None]
            cols = np.arange(t1)[None, :]
            S = np.where(cols <= rows, S, -np.inf)
            S = S - S.max(axis=1, keepdims=True)
            e = np.exp(S)
            P = e / e.sum(axis=1, keepdims=True)
            dO = do[t0:t1, a, :]
            dv[:t1, g, :] += P.T @ dO
            dP = dO @ V[:t1].T
            if o is None:
                D = np.sum(P * dP, axis=1, keepdims=True)
            else:
                D = np.sum(dO * o[t0:t1, a, :], axis=1, keepdims=True)
            dS = P * (dP - D)
            dq[t0:t1, a, :] = (dS @ K[:t1]) * scale
            dk[:t1, g, :] += (dS.T @ q[t0:t1, a, :]) * scale
    return dq, dk, dv


# --------------------------------------------------------------------------
# MLP activations
# --------------------------------------------------------------------------
def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def swiglu_fwd(gu):
    f = gu.shape[1] // 2
    g, u = gu[:, :f], gu[:, f:]
    return g * _sigmoid(g) * u


def swiglu_bwd(da, gu):
    f = gu.shape[1] // 2
    g, u = gu[:, :f], gu[:, f:]
    sg = _sigmoid(g)
    dg = da * u * sg * (1.0 + g * (1.0 - sg))
    du = da * g * sg
    return np.concatenate([dg, du], axis=1)


def gelu_fwd(z):
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


def gelu_bwd(da, z):
    Phi = 0.5 * (1.0 + _erf(z / math.sqrt(2.0)))
    phi = np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)
    return da * (Phi + z * phi)


# --------------------------------------------------------------------------
# one layer
# --------------------------------------------------------------------------
def _split_qkv(sh: StageShape, qkv):
    s = qkv.shape[0]
    nq, nkv, d = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    q = qkv[:, : nq * d].reshape(s, nq, d)
    k = qkv[:, nq * d: (nq + nkv) * d].reshape(s, nkv, d)
    v = qkv[:, (nq + nkv) * d:].reshape(s, nkv, d)
    return q, k, v


def _merge_qkv(q, k, v):
    s = q.shape[0]
    return np.concatenate([q.reshape(s, -1), k.reshape(s, -1), v.reshape(s, -1)], axis=1)


def _sequences(sh: StageShape, rows: int):
    """Row ranges of the sequences of one micro-batch: a micro-batch of size b holds b
    sequences of sh.seq tokens, stored one after the other; attention and rotary
    positions are per sequence."""
    if rows % sh.seq:
        raise ValueError(f"{rows} rows are not a whole number of sequences of {sh.seq} tokens")
    return [slice(b * sh.seq, (b + 1) * sh.seq) for b in range(rows // sh.seq)]


def layer_forward(sh: StageShape, w: dict, x, attn_chunk=None, store=None):
    """Returns (y, saved).  saved holds every tensor the store-all inventory keeps:
    x_in, n1, qkv (after rotary), o, lse, x_mid, n2, gu, a and the norm statistics.
    store: rounding applied to every op's output (see the module header); None keeps float64."""
    st = store or _keep
    sv = {"x_in": x}
    if sh.family == LLAMA:
        n1, r1 = rmsnorm_fwd(x, w["g1"], sh.norm_eps)
        sv["r1"] = r1
    else:
        n1, mu1, r1 = layernorm_fwd(x, w["g1"], w["b1"], sh.norm_eps)
        sv["mu1"], sv["r1"] = mu1, r1
    n1 = st(n1)
    qkv = st(linear_fwd(n1, w["wqkv"]))
    q, k, v = _split_qkv(sh, qkv)
    seqs = _sequences(sh, x.shape[0])
    if sh.family == LLAMA:
        q = np.concatenate([rope_apply(q[sl], sh.rope_base) for sl in seqs], axis=0)
        k = np.concatenate([rope_apply(k[sl], sh.rope_base) for sl in seqs], axis=0)
        qkv = st(_merge_qkv(q, k, v))
        q, k, v = _split_qkv(sh, qkv)
    per_seq = [attention_fwd(q[sl], k[sl], v[sl], attn_chunk) for sl in seqs]
    o = np.concatenate([o_b for o_b, _ in per_seq], axis=0)
    lse = np.stack([l_b for _, l_b in per_seq], axis=0)          # [sequence, head, position]
    o = st(o.reshape(x.shape[0], -1))
    x_mid = st(x + linear_fwd(o, w["wo"]))
    if sh.family == LLAMA:
        n2, r2 = rmsnorm_fwd(x_mid, w["g2"], sh.norm_eps)
        sv["r2"] = r2
    else:
        n2, mu2, r2 = layernorm_fwd(x_mid, w["g2"], w["b2"], sh.norm_eps)
        sv["mu2"], sv["r2"] = mu2, r2
    n2 = st(n2)
    gu = st(linear_fwd(n2, w["wgu"]))
    a = st(swiglu_fwd(gu) if sh.family == LLAMA else gelu_fwd(gu))
    y = st(x_mid + linear_fwd(a, w["wd"]))
    sv.update(n1=n1, qkv=qkv, o=o, lse=lse, x_mid=x_mid, n2=n2, gu=gu, a=a)
    return y, sv


def layer_backward_input(sh: StageShape, w: dict, sv: dict, dy, attn_chunk=None, store=None):
    """B for one layer.  Returns (dx_in, stash, dnorm) where stash holds, for each
    of the four linears, the pair (grad of its output, its input) that W needs,
    and dnorm the norm-parameter gradients (they are produced in B because B
    releases x_in / x_mid and the statistics they depend on)."""
    st = store or _keep
    s = dy.shape[0]
    da = st(linear_bwd_input(dy, w["wd"]))
    dgu = st(swiglu_bwd(da, sv["gu"]) if sh.family == LLAMA else gelu_bwd(da, sv["gu"]))
    dn2 = st(linear_bwd_input(dgu, w["wgu"]))
    dnorm = {}
    if sh.family == LLAMA:
        dxm, dnorm["g2"] = rmsnorm_bwd(dn2, sv["x_mid"], sv["r2"], w["g2"])
    else:
        dxm, dnorm["g2"], dnorm["b2"] = layernorm_bwd(dn2, sv["x_mid"], sv["mu2"], sv["r2"], w["g2"])
    dx_mid = st(dy + dxm)
    do = st(linear_bwd_input(dx_mid, w["wo"]))
    q, k, v = _split_qkv(sh, sv["qkv"])
    nq, d = sh.n_q_heads, sh.head_dim
    o3, do3 = sv["o"].reshape(s, nq, d), do.reshape(s, nq, d)
    parts = []
    for sl in _sequences(sh, s):
        # with a storage type the stored o is no longer the exact output: D then comes from its definition
        dq, dk, dv = attention_bwd(q[sl], k[sl], v[sl], o3[sl] if store is None else None, do3[sl], attn_chunk)
        dq, dk, dv = st(dq), st(dk), st(dv)                       # what the attention op hands on
        if sh.family == LLAMA:
            dq = st(rope_apply(dq, sh.rope_base, sign=-1.0))
            dk = st(rope_apply(dk, sh.rope_base, sign=-1.0))
        parts.append(_merge_qkv(dq, dk, dv))
    dqkv = np.concatenate(parts, axis=0)
    dn1 = st(linear_bwd_input(dqkv, w["wqkv"]))
    if sh.family == LLAMA:
        dxi, dnorm["g1"] = rmsnorm_bwd(dn1, sv["x_in"], sv["r1"], w["g1"])
    else:
        dxi, dnorm["g1"], dnorm["b1"] = layernorm_bwd(dn1, sv["x_in"], sv["mu1"], sv["r1"], w["g1"])
    dx_in = st(dx_mid + dxi)
    stash = {"wd": (dy, sv["a"]), "wgu": (dgu, sv["n2"]), "wo": (dx_mid, sv["o"]), "wqkv": (dqkv, sv["n1"])}
    return dx_in, stash, dnorm


def layer_backward_weight(stash: dict):
    """W for one layer: dW = dY^T X for each of the four linears."""
    return {name: linear_bwd_weight(dyx[0], dyx[1]) for name, dyx in stash.items()}


# --------------------------------------------------------------------------
# the stage: L layers in sequence
# --------------------------------------------------------------------------
def stage_forward(sh: StageShape, weights: list, x, attn_chunk=None, store=None):
    saved = []
    for l in range(sh.n_layers):
        x, sv = layer_forward(sh, weights[l], x, attn_chunk, store)
        saved.append(sv)
    return x, saved


def stage_backward_input(sh: StageShape, weights: list, saved: list, dy, attn_chunk=None, store=None):
    stashes = [None] * sh.n_layers
    dnorms = [None] * sh.n_layers
    for l in reversed(range(sh.n_layers)):
        dy, stashes[l], dnorms[l] = layer_backward_input(sh, weights[l], saved[l], dy, attn_chunk, store)
    return dy, stashes, dnorms


def stage_backward_weight(stashes: list):
    return [layer_backward_weight(st) for st in stashes]


def stage_fbw(sh: StageShape, weights: list, x, dy, attn_chunk=None, store=None):
    """F, then B, then W of one micro-batch.  Returns y, dx, dW (per layer dict),
    dnorm (per layer dict).  Parameter gradients are sums held in fp32 by the workloads
    and are never rounded to the storage type."""
    y, saved = stage_forward(sh, weights, x, attn_chunk, store)
    dx, stashes, dnorms = stage_backward_input(sh, weights, saved, dy, attn_chunk, store)
    return y, dx, stage_backward_weight(stashes), dnorms


def flops_per_microbatch(sh: StageShape):
    """Algorithmic flop count of F, B, W for one micro-batch: 2*tokens*N*K per GEMM
    in each of F / B / W; causal attention 2*s^2*n_q*d forward and 5*s^2*n_q*d
    backward (lower triangle only); elementwise work not counted."""
    s, h, f = sh.seq, sh.hidden, sh.ffn
    nq, d = sh.n_q_heads, sh.head_dim
    up = 2 * f if sh.family == LLAMA else f
    gemm = 2 * s * (sh.qkv_width * h + h * nq * d + up * h + h * f)
    fwd = gemm + 2 * s * s * nq * d
    bwd = gemm + 5 * s * s * nq * d
    return {"F": fwd * sh.n_layers, "B": bwd * sh.n_layers, "W": gemm * sh.n_layers}
