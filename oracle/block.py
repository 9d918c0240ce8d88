"""Oracle: one pre-norm transformer block over a packed variable-length mini-batch, fwd + bwd.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain numpy, plain definitions.

The paper (Sec. 3 "Data Imbalance", Sec. 4.1) only requires that samples stay whole and that a
mini-batch carries no padding; the block itself is the textbook pre-norm transformer block named
by the benchmark configurations:

    x1 = x  + Attn(N1(x)) W_o^T (+ b_o)
    y  = x1 + MLP(N2(x1))

with attention confined to each segment of the packed batch (a ViT image tile, or one LLM
sample), bidirectional or causal inside the segment.

Layouts: activations [T, H]; weights [out_features, in_features]; q [T, nq, d], k/v [T, nkv, d];
cu = int32 segment offsets, cu[0] = 0, cu[-1] = T.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

NORM_LAYERNORM, NORM_RMSNORM = 0, 1
MLP_GELU, MLP_SWIGLU = 0, 1
MASK_BIDIR, MASK_CAUSAL = 0, 1


# ------------------------------------------------------------------------------------------
# helpers
# ------------------------------------------------------------------------------------------

def segment_ids(cu, T):
    """seg[t] = index j of the segment with cu[j] <= t < cu[j+1]."""
    cu = np.asarray(cu, dtype=np.int64)
    assert cu[0] == 0 and cu[-1] == T and np.all(np.diff(cu) > 0)
    return np.repeat(np.arange(len(cu) - 1), np.diff(cu))


def allowed_mask(cu, T, mask_kind):
    """allowed[i, j] <=> seg(i) == seg(j) and (j <= i if causal).  bool [T, T]."""
    seg = segment_ids(cu, T)
    allowed = seg[:, None] == seg[None, :]
    if mask_kind == MASK_CAUSAL:
        idx = np.arange(T)
        allowed &= idx[None, :] <= idx[:, None]
    return allowed


def linear(a, w, b=None):
    """a [T, in] , w [out, in] -> a w^T (+ b)."""
    out = a @ w.T
    if b is not None:
        out = out + b
    return out


# ------------------------------------------------------------------------------------------
# norms
# ------------------------------------------------------------------------------------------

def layernorm_fwd(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)          # biased variance
    rstd = 1.0 / np.sqrt(var + eps)
    h = xc * rstd * g
    if b is not None:
        h = h + b
    return h


def layernorm_bwd(dh, x, g, eps):
    """returns dx, dgamma, dbeta"""
    H = x.shape[-1]
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = xc * rstd
    dxhat = dh * g
    dx = rstd * (dxhat - dxhat.sum(-1, keepdims=True) / H
                 - xhat * (dxhat * xhat).sum(-1, keepdims=True) / H)
    return dx, (dh * xhat).sum(axis=0), dh.sum(axis=0)


def rmsnorm_fwd(x, g, eps):
    rstd = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    return x * rstd * g


def rmsnorm_bwd(dh, x, g, eps):
    """returns dx, dgamma"""
    H = x.shape[-1]
    rstd = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    xhat = x * rstd
    dxhat = dh * g
    dx = rstd * (dxhat - xhat * (dxhat * xhat).sum(-1, keepdims=True) / H)
    return dx, (dh * xhat).sum(axis=0)


def norm_fwd(kind, x, g, b, eps):
    return layernorm_fwd(x, g, b, eps) if kind == NORM_LAYERNORM else rmsnorm_fwd(x, g, eps)


def norm_bwd(kind, dh, x, g, eps):
    if kind == NORM_LAYERNORM:
        return layernorm_bwd(dh, x, g, eps)
    dx, dg = rmsnorm_bwd(dh, x, g, eps)
    return dx, dg, None


# ------------------------------------------------------------------------------------------
# rotary position embedding, positions restart at 0 in every segment
# ------------------------------------------------------------------------------------------

def rotary_angles(cu, T, d, base, dtype=np.float64):
    """angle[t, i] = pos(t) * base^(-2 i / d), pos(t) = t - cu[seg(t)], i in [0, d/2)."""
    cu = np.asarray(cu, dtype=np.int64)
    seg = segment_ids(cu, T)
    pos = (np.arange(T) - cu[seg]).astype(np.float64)
    theta = np.float64(base) ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)
    return (pos[:, None] * theta[None, :]).astype(dtype)


def rotary_apply(x, angle, sign=1.0):
    """x [T, n, d]; pairs (i, i + d/2) rotated by sign * angle[t, i]."""
    d = x.shape[-1]
    c = np.cos(angle)[:, None, :]
    s = (sign * np.sin(angle))[:, None, :]
    x1, x2 = x[..., : d // 2], x[..., d // 2:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


# ------------------------------------------------------------------------------------------
# attention
# ------------------------------------------------------------------------------------------

def _softmax_rows(S, allowed):
    S = np.where(allowed, S, -np.inf)
    m = S.max(axis=-1, keepdims=True)
    E = np.exp(S - m)
    l = E.sum(axis=-1, keepdims=True)
    return E / l, (m + np.log(l))[:, 0]


def attention_fwd_masked(q, k, v, cu, mask_kind, scale, return_probs=False):
    """The definition: full [T, T] scores per head with the segment (and causal) mask.

    returns o [T, nq, d], lse [nq, T] (natural-log-sum-exp of the scaled, masked scores).
    """
    T, nq, d = q.shape
    nkv = k.shape[1]
    group = nq // nkv
    allowed = allowed_mask(cu, T, mask_kind)
    o = np.zeros_like(q)
    lse = np.zeros((nq, T), dtype=q.dtype)
    probs = []
    for a in range(nq):
        kvh = a // group
        S = (q[:, a, :] @ k[:, kvh, :].T) * scale
        P, lse[a] = _softmax_rows(S, allowed)
        o[:, a, :] = P @ v[:, kvh, :]
        if return_probs:
            probs.append(P)
    if return_probs:
        return o, lse, probs
    return o, lse


def attention_fwd_per_segment(q, k, v, cu, mask_kind, scale):
    """Textbook (full or causal) attention run on each segment alone."""
    T, nq, d = q.shape
    o = np.zeros_like(q)
    lse = np.zeros((nq, T), dtype=q.dtype)
    cu = np.asarray(cu, dtype=np.int64)
    for j in range(len(cu) - 1):
        a, b = int(cu[j]), int(cu[j + 1])
        oj, lj = attention_fwd_masked(q[a:b], k[a:b], v[a:b], [0, b - a], mask_kind, scale)
        o[a:b] = oj
        lse[:, a:b] = lj
    return o, lse


def attention_bwd_masked(d_o, q, k, v, cu, mask_kind, scale):
    """Analytic gradient of attention_fwd_masked: returns dq, dk, dv."""
    T, nq, d = q.shape
    nkv = k.shape[1]
    group = nq // nkv
    allowed = allowed_mask(cu, T, mask_kind)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for a in range(nq):
        kvh = a // group
        S = (q[:, a, :] @ k[:, kvh, :].T) * scale
        P, _ = _softmax_rows(S, allowed)
        dO = d_o[:, a, :]
        dv[:, kvh, :] += P.T @ dO
        dP = dO @ v[:, kvh, :].T
        delta = (dP * P).sum(axis=-1, keepdims=True)
        dS = P * (dP - delta)
        dq[:, a, :] = (dS @ k[:, kvh, :]) * scale
        dk[:, kvh, :] += (dS.T @ q[:, a, :]) * scale
    return dq, dk, dv


def attention_bwd_per_segment(d_o, q, k, v, cu, mask_kind, scale):
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    cu = np.asarray(cu, dtype=np.int64)
    for j in range(len(cu) - 1):
        a, b = int(cu[j]), int(cu[j + 1])
        r = attention_bwd_masked(d_o[a:b], q[a:b], k[a:b], v[a:b], [0, b - a], mask_kind, scale)
        dq[a:b], dk[a:b], dv[a:b] = r
    return dq, dk, dv


# Above this many tokens the [T, T] form is replaced by the per-segment form, which the tests
# pin to be the same function (tests/test_oracle_block.py::test_masked_equals_per_segment).
_MASKED_MAX_T = 1536


def attention_fwd(q, k, v, cu, mask_kind, scale):
    if q.shape[0] <= _MASKED_MAX_T:
        return attention_fwd_masked(q, k, v, cu, mask_kind, scale)
    return attention_fwd_per_segment(q, k, v, cu, mask_kind, scale)


def attention_bwd(d_o, q, k, v, cu, mask_kind, scale):
    if q.shape[0] <= _MASKED_MAX_T:
        return attention_bwd_masked(d_o, q, k, v, cu, mask_kind, scale)
    return attention_bwd_per_segment(d_o, q, k, v, cu, mask_kind, scale)


# ------------------------------------------------------------------------------------------
# MLP activations
# ------------------------------------------------------------------------------------------

def gelu(z):
    """exact GELU: z/2 (1 + erf(z / sqrt 2))"""
    return 0.5 * z * (1.0 + _erf(z / np.sqrt(2.0)))


def gelu_grad(z):
    return 0.5 * (1.0 + _erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


# ------------------------------------------------------------------------------------------
# the block
# ------------------------------------------------------------------------------------------

def _cast(w, dtype):
    return {k: (None if a is None else np.asarray(a, dtype=dtype)) for k, a in w.items()}


def block_fwd(shape, w, x, cu, dtype=np.float64):
    """Forward of one block.  `shape` has the fields of synth_inputs.BlockShape.

    returns y [T, H] and a cache of every intermediate (for the backward and for tests).
    """
    w = _cast(w, dtype)
    x = np.asarray(x, dtype=dtype)
    T, H = x.shape
    nq, nkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    F = shape.mlp_dim
    scale = 1.0 / np.sqrt(np.float64(d))
    g = lambda name: w.get(name)

    h1 = norm_fwd(shape.norm, x, w["n1_g"], g("n1_b"), shape.norm_eps)
    qkv = linear(h1, w["w_qkv"], g("b_qkv"))
    q = qkv[:, : nq * d].reshape(T, nq, d)
    k = qkv[:, nq * d: (nq + nkv) * d].reshape(T, nkv, d)
    v = qkv[:, (nq + nkv) * d:].reshape(T, nkv, d)
    angle = None
    if shape.use_rotary:
        angle = rotary_angles(cu, T, d, shape.rotary_base, dtype)
        q = rotary_apply(q, angle)
        k = rotary_apply(k, angle)
    o, lse = attention_fwd(q, k, v, cu, shape.mask, dtype(scale))
    x1 = x + linear(o.reshape(T, nq * d), w["w_o"], g("b_o"))
    h2 = norm_fwd(shape.norm, x1, w["n2_g"], g("n2_b"), shape.norm_eps)
    up = linear(h2, w["w_up"], g("b_up"))
    if shape.mlp == MLP_GELU:
        act = gelu(up)
    else:
        act = up[:, :F] * sigmoid(up[:, :F]) * up[:, F:]
    y = x1 + linear(act, w["w_down"], g("b_down"))
    cache = dict(x=x, h1=h1, q=q, k=k, v=v, angle=angle, o=o, lse=lse, x1=x1, h2=h2, up=up,
                 act=act, scale=dtype(scale))
    return y.astype(dtype), cache


def block_bwd(shape, w, cache, dy, cu, dtype=np.float64):
    """Analytic backward of block_fwd.  returns dx [T, H] and a dict of weight gradients."""
    w = _cast(w, dtype)
    dy = np.asarray(dy, dtype=dtype)
    c = cache
    T, H = dy.shape
    nq, nkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    F = shape.mlp_dim
    grads = {}

    # y = x1 + act W_down^T + b_down
    grads["w_down"] = dy.T @ c["act"]
    if shape.has_bias:
        grads["b_down"] = dy.sum(axis=0)
    dact = dy @ w["w_down"]
    up = c["up"]
    if shape.mlp == MLP_GELU:
        dup = dact * gelu_grad(up)
    else:
        gte, u = up[:, :F], up[:, F:]
        sg = sigmoid(gte)
        silu = gte * sg
        dgate = dact * u * (sg * (1.0 + gte * (1.0 - sg)))
        dupp = dact * silu
        dup = np.concatenate([dgate, dupp], axis=1)
    grads["w_up"] = dup.T @ c["h2"]
    if shape.has_bias:
        grads["b_up"] = dup.sum(axis=0)
    dh2 = dup @ w["w_up"]
    dx1_n, grads["n2_g"], db = norm_bwd(shape.norm, dh2, c["x1"], w["n2_g"], shape.norm_eps)
    if shape.norm == NORM_LAYERNORM and shape.has_bias:
        grads["n2_b"] = db
    dx1 = dy + dx1_n

    # x1 = x + o W_o^T + b_o
    o2 = c["o"].reshape(T, nq * d)
    grads["w_o"] = dx1.T @ o2
    if shape.has_bias:
        grads["b_o"] = dx1.sum(axis=0)
    d_o = (dx1 @ w["w_o"]).reshape(T, nq, d)
    dq, dk, dv = attention_bwd(d_o, c["q"], c["k"], c["v"], cu, shape.mask, c["scale"])
    if shape.use_rotary:
        dq = rotary_apply(dq, c["angle"], sign=-1.0)
        dk = rotary_apply(dk, c["angle"], sign=-1.0)
    dqkv = np.concatenate([dq.reshape(T, -1), dk.reshape(T, -1), dv.reshape(T, -1)], axis=1)
    grads["w_qkv"] = dqkv.T @ c["h1"]
    if shape.has_bias:
        grads["b_qkv"] = dqkv.sum(axis=0)
    dh1 = dqkv @ w["w_qkv"]
    dx_n, grads["n1_g"], db = norm_bwd(shape.norm, dh1, c["x"], w["n1_g"], shape.norm_eps)
    if shape.norm == NORM_LAYERNORM and shape.has_bias:
        grads["n1_b"] = db
    dx = dx1 + dx_n
    inter = dict(dact=dact, dup=dup, dh2=dh2, dx1=dx1, d_o=d_o, dq=dq, dk=dk, dv=dv, dqkv=dqkv,
                 dh1=dh1)
    return dx.astype(dtype), grads, inter


def stack_fwd_bwd(shape, weights_per_block, x, dy, cu, dtype=np.float64):
    """L blocks forward then backward (the whole hot path for one mini-batch)."""
    caches = []
    a = np.asarray(x, dtype=dtype)
    for w in weights_per_block:
        a, c = block_fwd(shape, w, a, cu, dtype)
        caches.append(c)
    y = a
    g = np.asarray(dy, dtype=dtype)
    all_grads = [None] * len(weights_per_block)
    for i in reversed(range(len(weights_per_block))):
        g, all_grads[i], _ = block_bwd(shape, weights_per_block[i], caches[i], g, cu, dtype)
    return y, g, all_grads


# ------------------------------------------------------------------------------------------
# algorithmic FLOP count (what the method must compute; masked-out score entries, the backward's
# recomputation of the scores and all elementwise work are not counted; backward = 2 x forward)
# ------------------------------------------------------------------------------------------

def algorithmic_flops(shape, cu, n_blocks=None):
    cu = np.asarray(cu, dtype=np.int64)
    T = int(cu[-1])
    s = np.diff(cu).astype(np.float64)
    H, d, nq = shape.hidden, shape.head_dim, shape.n_q_heads
    dqkv = (shape.n_q_heads + 2 * shape.n_kv_heads) * d
    gemm = 2.0 * H * dqkv + 2.0 * H * nq * d + 2.0 * H * shape.mlp_dim * \
        (3 if shape.mlp == MLP_SWIGLU else 2)
    area = (s * (s + 1) / 2).sum() if shape.mask == MASK_CAUSAL else (s * s).sum()
    attn = 4.0 * nq * d * area
    L = shape.n_blocks if n_blocks is None else n_blocks
    return 3.0 * L * (T * gemm + attn)
