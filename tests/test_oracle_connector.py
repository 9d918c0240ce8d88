"""Pins for oracle/connector.py: brute force, a coordinate image, adjointness, finite differences."""
import numpy as np

import synth_inputs as si
from oracle import connector as oc


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def test_subsample_on_a_coordinate_image():
    # patch (y, x) of tile t carries the feature (t, y, x); the class token carries -1
    g, n_tiles = 6, 3
    v = np.full((n_tiles * (g * g + 1), 3), -1.0)
    for t in range(n_tiles):
        for y in range(g):
            for x in range(g):
                v[t * (g * g + 1) + 1 + y * g + x] = (t, y, x)
    u = oc.subsample_fwd(v, n_tiles, g)
    assert u.shape == (n_tiles * 9, 12)
    for t in range(n_tiles):
        for r in range(3):
            for c in range(3):
                row = u[(t * 3 + r) * 3 + c].reshape(4, 3)
                expect = [(t, 2 * r, 2 * c), (t, 2 * r, 2 * c + 1), (t, 2 * r + 1, 2 * c), (t, 2 * r + 1, 2 * c + 1)]
                np.testing.assert_array_equal(row, np.array(expect, dtype=float))
    assert not (u == -1.0).any()          # the class token is never picked


def test_every_patch_is_used_exactly_once():
    g, n_tiles = 8, 2
    rows = oc.source_rows(n_tiles, g)
    flat = np.sort(rows.ravel())
    patches = np.array([t * (g * g + 1) + 1 + p for t in range(n_tiles) for p in range(g * g)])
    np.testing.assert_array_equal(flat, patches)


def test_subsample_bwd_is_the_adjoint():
    g, n_tiles, Hv = 4, 2, 5
    v, du = _rand((n_tiles * (g * g + 1), Hv), 0), _rand((n_tiles * g * g // 4, 4 * Hv), 1)
    lhs = (oc.subsample_fwd(v, n_tiles, g) * du).sum()
    dv = oc.subsample_bwd(du, n_tiles, g)
    np.testing.assert_allclose(lhs, (v * dv).sum(), rtol=1e-13)
    for t in range(n_tiles):
        assert not dv[t * (g * g + 1)].any()      # class rows get no gradient


def _setup(seed=0, g=4, n_tiles=2, Hv=6, Ht=10, text=(3, 5)):
    w = {k: _rand(a.shape, seed + 10 + i, 0.3) + (1.0 if k == "n_g" else 0.0)
         for i, (k, a) in enumerate(si.connector_weights(Hv, Ht, seed).items())}
    v = _rand((n_tiles * (g * g + 1), Hv), seed + 1)
    dst, cu = si.visual_rows([1] * n_tiles, text, tokens_per_tile=g * g // 4)
    x_llm = _rand((int(cu[-1]), Ht), seed + 2)
    dx_llm = _rand((int(cu[-1]), Ht), seed + 3)
    return w, v, dst, cu, x_llm, dx_llm, g, n_tiles


def test_forward_is_the_composition_written_out_and_text_rows_stay():
    w, v, dst, cu, x_llm, _, g, n_tiles = _setup()
    out, cache = oc.connector_fwd(w, v, n_tiles, g, 1e-5, x_llm, dst)
    text = np.setdiff1d(np.arange(int(cu[-1])), dst)
    np.testing.assert_array_equal(out[text], x_llm[text])
    # first visual token of tile 1 by hand
    i = g * g // 4
    t0 = 1 * (g * g + 1) + 1
    u = np.concatenate([v[t0], v[t0 + 1], v[t0 + g], v[t0 + g + 1]])
    xh = (u - u.mean()) / np.sqrt(u.var() + 1e-5)
    h = (xh * w["n_g"] + w["n_b"]) @ w["w1"].T + w["b1"]
    from math import erf, sqrt
    a = np.array([0.5 * t * (1 + erf(t / sqrt(2))) for t in h])
    np.testing.assert_allclose(out[dst[i]], a @ w["w2"].T + w["b2"], rtol=1e-12, atol=1e-12)


def test_backward_matches_central_differences():
    w, v, dst, cu, x_llm, dx_llm, g, n_tiles = _setup(seed=5)
    eps = 1e-5

    def loss(w_, v_):
        out, _ = oc.connector_fwd(w_, v_, n_tiles, g, eps, x_llm, dst)
        return float((out * dx_llm).sum())

    _, cache = oc.connector_fwd(w, v, n_tiles, g, eps, x_llm, dst)
    dv, grads = oc.connector_bwd(w, cache, dx_llm, n_tiles, g, eps, dst)
    rng = np.random.default_rng(9)
    h = 1e-6
    for _ in range(12):     # input entries, class rows included
        i, j = rng.integers(v.shape[0]), rng.integers(v.shape[1])
        vp, vm = v.copy(), v.copy()
        vp[i, j] += h; vm[i, j] -= h
        np.testing.assert_allclose(dv[i, j], (loss(w, vp) - loss(w, vm)) / (2 * h), rtol=2e-6, atol=2e-8)
    for name in si.CONNECTOR_NAMES:
        for _ in range(4):
            idx = tuple(rng.integers(s) for s in w[name].shape)
            wp = {k: a.copy() for k, a in w.items()}; wm = {k: a.copy() for k, a in w.items()}
            wp[name][idx] += h; wm[name][idx] -= h
            np.testing.assert_allclose(grads[name][idx], (loss(wp, v) - loss(wm, v)) / (2 * h), rtol=2e-6, atol=2e-8)


def test_visual_rows_layout():
    dst, cu = si.visual_rows([2, 1], [3, 0], tokens_per_tile=4)
    np.testing.assert_array_equal(cu, [0, 11, 15])
    np.testing.assert_array_equal(dst, list(range(8)) + list(range(11, 15)))
