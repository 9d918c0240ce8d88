"""Oracle: the hand-over between the ViT stack and the LLM stack of a mixed pipeline stage
(App. A shows stages that hold both kinds of layer; Sec. 5.4 names the vision model's "token
sub-sampling" as the point after which less data crosses a stage boundary).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain numpy, plain definitions, fp64.

The paper fixes neither the sub-sampling nor the connector; the reading taken here is the one the
benchmark configurations imply (1025 ViT tokens per tile = class token + 32 x 32 patches; 256
LLM-side tokens per tile):

  c1  sub-sampling: drop the class token; token (r, c) of the (g/2) x (g/2) output grid is the
      concatenation along channels of the 2 x 2 patches (2r + dr, 2c + dc), channel block
      2 dr + dc;  [n_tiles (g^2 + 1), Hv] -> [n_tiles g^2 / 4, 4 Hv]
  c2  LayerNorm over the 4 Hv channels (gain, beta)
  c3  h = un W1^T + b1 ; a = GELU(h)                 W1 [Ht, 4 Hv]
  c4  z = a W2^T + b2                                W2 [Ht, Ht]
  c5  row i of z replaces row dst_rows[i] of the LLM stack's packed input (text rows stay)

Pins: tests/test_oracle_connector.py.
"""
import numpy as np

from oracle.block import gelu, gelu_grad, layernorm_bwd, layernorm_fwd, linear


def source_rows(n_tiles, g):
    """rows[i, b] = row of the ViT output that feeds channel block b of sub-sampled token i."""
    half = g // 2
    rows = np.empty((n_tiles * half * half, 4), dtype=np.int64)
    for t in range(n_tiles):
        for r in range(half):
            for c in range(half):
                i = (t * half + r) * half + c
                for dr in range(2):
                    for dc in range(2):
                        rows[i, 2 * dr + dc] = t * (g * g + 1) + 1 + (2 * r + dr) * g + (2 * c + dc)
    return rows


def subsample_fwd(v, n_tiles, g):
    Hv = v.shape[1]
    rows = source_rows(n_tiles, g)
    u = np.empty((rows.shape[0], 4 * Hv), dtype=v.dtype)
    for b in range(4):
        u[:, b * Hv:(b + 1) * Hv] = v[rows[:, b]]
    return u


def subsample_bwd(du, n_tiles, g):
    """Adjoint of subsample_fwd: every patch row receives its channel block, class rows zero."""
    Hv = du.shape[1] // 4
    rows = source_rows(n_tiles, g)
    dv = np.zeros((n_tiles * (g * g + 1), Hv), dtype=du.dtype)
    for b in range(4):
        dv[rows[:, b]] += du[:, b * Hv:(b + 1) * Hv]
    return dv


def connector_fwd(w, v, n_tiles, g, eps, x_llm, dst_rows):
    """returns the LLM input with the visual rows filled in, and the cache for the backward."""
    v = np.asarray(v, dtype=np.float64)
    w = {k: np.asarray(a, dtype=np.float64) for k, a in w.items()}
    u = subsample_fwd(v, n_tiles, g)
    un = layernorm_fwd(u, w["n_g"], w["n_b"], eps)
    h = linear(un, w["w1"], w["b1"])
    a = gelu(h)
    z = linear(a, w["w2"], w["b2"])
    out = np.array(x_llm, dtype=np.float64, copy=True)
    out[np.asarray(dst_rows)] = z
    return out, dict(u=u, un=un, h=h, a=a, z=z)


def connector_bwd(w, cache, dx_llm, n_tiles, g, eps, dst_rows):
    """Given the gradient of the LLM input, returns dv [n_tiles (g^2 + 1), Hv] and weight grads."""
    w = {k: np.asarray(a, dtype=np.float64) for k, a in w.items()}
    dz = np.asarray(dx_llm, dtype=np.float64)[np.asarray(dst_rows)]
    grads = {"w2": dz.T @ cache["a"], "b2": dz.sum(0)}
    da = dz @ w["w2"]
    dh = da * gelu_grad(cache["h"])
    grads["w1"] = dh.T @ cache["un"]
    grads["b1"] = dh.sum(0)
    dun = dh @ w["w1"]
    du, grads["n_g"], grads["n_b"] = layernorm_bwd(dun, cache["u"], w["n_g"], eps)
    return subsample_bwd(du, n_tiles, g), grads
