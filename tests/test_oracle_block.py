"""Pins for oracle/block.py: every check here compares the oracle with something other than
itself -- a textbook special case, a closed form, brute force, or finite differences."""
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import block as ob


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


# ------------------------------------------------------------------------------------------
# GEMM step: brute-force triple loop, sizes that are multiples of nothing
# ------------------------------------------------------------------------------------------

def test_linear_matches_triple_loop():
    a, w, b = _rand((5, 7), 0), _rand((3, 7), 1), _rand((3,), 2)
    ref = np.zeros((5, 3))
    for i in range(5):
        for j in range(3):
            acc = 0.0
            for k in range(7):
                acc += a[i, k] * w[j, k]
            ref[i, j] = acc + b[j]
    np.testing.assert_allclose(ob.linear(a, w, b), ref, rtol=0, atol=1e-13)


# ------------------------------------------------------------------------------------------
# norms, activations, rotary: closed forms
# ------------------------------------------------------------------------------------------

def test_layernorm_zero_mean_unit_variance():
    x = _rand((9, 33), 3, 2.0) + 5.0
    h = ob.layernorm_fwd(x, np.ones(33), np.zeros(33), 0.0)
    np.testing.assert_allclose(h.mean(-1), 0.0, atol=1e-12)
    np.testing.assert_allclose((h * h).mean(-1), 1.0, atol=1e-12)
    g, b = _rand((33,), 4), _rand((33,), 5)
    np.testing.assert_allclose(ob.layernorm_fwd(x, g, b, 0.0), h * g + b, atol=1e-12)


def test_layernorm_eps_enters_under_the_root():
    x = np.array([[1.0, 3.0]])            # mean 2, biased var 1
    h = ob.layernorm_fwd(x, np.ones(2), None, 3.0)
    np.testing.assert_allclose(h, [[-0.5, 0.5]], atol=1e-15)


def test_rmsnorm_constant_vector_gives_sign_times_gamma():
    g = _rand((16,), 6)
    for c in (3.5, -0.25):
        h = ob.rmsnorm_fwd(np.full((2, 16), c), g, 0.0)
        np.testing.assert_allclose(h, np.sign(c) * np.tile(g, (2, 1)), atol=1e-14)
    h = ob.rmsnorm_fwd(np.array([[3.0, 4.0]]), np.ones(2), 0.0)   # rms = sqrt(12.5)
    np.testing.assert_allclose(h, np.array([[3.0, 4.0]]) / math.sqrt(12.5), atol=1e-15)


def test_gelu_and_sigmoid_values():
    z = np.array([-3.0, -1.0, 0.0, 0.5, 2.0])
    ref = [0.5 * t * (1.0 + math.erf(t / math.sqrt(2.0))) for t in z]
    np.testing.assert_allclose(ob.gelu(z), ref, atol=1e-15)
    assert ob.gelu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(ob.gelu(np.array([1.0]))[0], 0.8413447460685429, atol=1e-12)
    np.testing.assert_allclose(ob.sigmoid(np.array([0.0, math.log(3.0)])), [0.5, 0.75],
                               atol=1e-15)
    h = 1e-6
    fd = (ob.gelu(z + h) - ob.gelu(z - h)) / (2 * h)
    np.testing.assert_allclose(ob.gelu_grad(z), fd, atol=1e-8)


def test_rotary_properties():
    d, T = 8, 11
    cu = [0, 4, 11]
    ang = ob.rotary_angles(cu, T, d, 10000.0)
    # positions restart at 0 in each segment -> identity there
    x = _rand((T, 2, d), 7)
    y = ob.rotary_apply(x, ang)
    np.testing.assert_array_equal(y[0], x[0])
    np.testing.assert_array_equal(y[4], x[4])
    # angle of pair i at position p is p * base^(-2i/d)
    assert ang[6, 0] == 2.0 and abs(ang[6, 1] - 2.0 * 10000.0 ** (-0.25)) < 1e-15
    # each (i, i + d/2) pair keeps its norm
    n_in = x[..., : d // 2] ** 2 + x[..., d // 2:] ** 2
    n_out = y[..., : d // 2] ** 2 + y[..., d // 2:] ** 2
    np.testing.assert_allclose(n_out, n_in, atol=1e-12)
    # q_m . k_n after rotation depends only on m - n
    q0, k0 = _rand((d,), 8), _rand((d,), 9)
    ang1 = ob.rotary_angles([0, 40], 40, d, 10000.0)
    qs = ob.rotary_apply(np.tile(q0, (40, 1, 1)), ang1)[:, 0]
    ks = ob.rotary_apply(np.tile(k0, (40, 1, 1)), ang1)[:, 0]
    assert abs(qs[7] @ ks[3] - qs[30] @ ks[26]) < 1e-12
    assert abs(qs[7] @ ks[3] - qs[7] @ ks[4]) > 1e-6
    # inverse rotation undoes it; a hand value: rotate (1, 0) by angle pi/2 -> (0, 1)
    np.testing.assert_allclose(ob.rotary_apply(y, ang, sign=-1.0), x, atol=1e-12)
    v = np.zeros((1, 1, 2)); v[0, 0, 0] = 1.0
    r = ob.rotary_apply(v, np.array([[math.pi / 2]]))
    np.testing.assert_allclose(r[0, 0], [0.0, 1.0], atol=1e-15)


# ------------------------------------------------------------------------------------------
# attention: segment masking == per-segment textbook attention; softmax rows; GQA
# ------------------------------------------------------------------------------------------

def _textbook_attention(q, k, v, causal, scale):
    """single sequence, single head, python loops"""
    T, d = q.shape
    o = np.zeros((T, v.shape[1]))
    for i in range(T):
        js = range(i + 1) if causal else range(T)
        s = np.array([q[i] @ k[j] * scale for j in js])
        p = np.exp(s - s.max())
        p /= p.sum()
        for p_j, j in zip(p, js):
            o[i] += p_j * v[j]
    return o


@pytest.mark.parametrize("mask", [ob.MASK_BIDIR, ob.MASK_CAUSAL])
def test_single_segment_is_textbook_attention(mask):
    T, d = 9, 4
    q, k, v = _rand((T, 1, d), 10), _rand((T, 1, d), 11), _rand((T, 1, d), 12)
    o, lse = ob.attention_fwd_masked(q, k, v, [0, T], mask, 0.5)
    ref = _textbook_attention(q[:, 0], k[:, 0], v[:, 0], mask == ob.MASK_CAUSAL, 0.5)
    np.testing.assert_allclose(o[:, 0], ref, atol=1e-13)
    # lse of the last row = log sum_j exp(s_j) over all T keys in both mask kinds
    s = (q[-1, 0] @ k[:, 0].T) * 0.5
    assert abs(lse[0, -1] - math.log(np.exp(s).sum())) < 1e-12


@pytest.mark.parametrize("mask", [ob.MASK_BIDIR, ob.MASK_CAUSAL])
def test_masked_equals_per_segment(mask):
    lens = [5, 1, 17, 8]
    cu = si.lengths_to_cu(lens)
    T, nq, nkv, d = int(cu[-1]), 4, 2, 8
    q, k, v, d_o = (_rand((T, n, d), s) for n, s in ((nq, 1), (nkv, 2), (nkv, 3), (nq, 4)))
    o1, l1 = ob.attention_fwd_masked(q, k, v, cu, mask, 0.3)
    o2, l2 = ob.attention_fwd_per_segment(q, k, v, cu, mask, 0.3)
    np.testing.assert_allclose(o1, o2, atol=1e-13)
    np.testing.assert_allclose(l1, l2, atol=1e-13)
    # and per segment it is the textbook loop (head 3 reads kv head 1)
    a, b = int(cu[2]), int(cu[3])
    ref = _textbook_attention(q[a:b, 3], k[a:b, 1], v[a:b, 1], mask == ob.MASK_CAUSAL, 0.3)
    np.testing.assert_allclose(o1[a:b, 3], ref, atol=1e-13)
    g1 = ob.attention_bwd_masked(d_o, q, k, v, cu, mask, 0.3)
    g2 = ob.attention_bwd_per_segment(d_o, q, k, v, cu, mask, 0.3)
    for x, y in zip(g1, g2):
        np.testing.assert_allclose(x, y, atol=1e-12)


def test_softmax_rows_sum_to_one_and_length_one_row_copies_v():
    cu = si.lengths_to_cu([6, 1, 9])
    T = 16
    q, k, v = _rand((T, 2, 4), 20), _rand((T, 2, 4), 21), _rand((T, 2, 4), 22)
    for mask in (ob.MASK_BIDIR, ob.MASK_CAUSAL):
        o, lse, probs = ob.attention_fwd_masked(q, k, v, cu, mask, 0.5, return_probs=True)
        allowed = ob.allowed_mask(cu, T, mask)
        for P in probs:
            np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-14)
            assert np.all(P[~allowed] == 0.0)
        np.testing.assert_array_equal(o[6], v[6])          # the one-token segment
    o, _ = ob.attention_fwd_masked(q, k, v, cu, ob.MASK_CAUSAL, 0.5)
    np.testing.assert_array_equal(o[0], v[0])              # first causal row of a segment
    np.testing.assert_array_equal(o[7], v[7])
    q32 = q.astype(np.float32)
    _, _, probs = ob.attention_fwd_masked(q32, k.astype(np.float32), v.astype(np.float32), cu,
                                          ob.MASK_BIDIR, np.float32(0.5), return_probs=True)
    assert max(abs(P.sum(-1) - 1).max() for P in probs) <= 1e-6


def test_mask_bits():
    cu = [0, 2, 5]
    m = ob.allowed_mask(cu, 5, ob.MASK_CAUSAL).astype(int)
    ref = [[1, 0, 0, 0, 0], [1, 1, 0, 0, 0], [0, 0, 1, 0, 0], [0, 0, 1, 1, 0], [0, 0, 1, 1, 1]]
    assert m.tolist() == ref
    m = ob.allowed_mask(cu, 5, ob.MASK_BIDIR).astype(int)
    ref = [[1, 1, 0, 0, 0], [1, 1, 0, 0, 0], [0, 0, 1, 1, 1], [0, 0, 1, 1, 1], [0, 0, 1, 1, 1]]
    assert m.tolist() == ref


def test_gqa_equals_mha_with_replicated_kv_heads():
    cu = si.lengths_to_cu([7, 12])
    T, nq, nkv, d = 19, 6, 2, 8
    q, k, v, d_o = (_rand((T, n, d), s) for n, s in ((nq, 30), (nkv, 31), (nkv, 32), (nq, 33)))
    k_rep, v_rep = np.repeat(k, nq // nkv, axis=1), np.repeat(v, nq // nkv, axis=1)
    o1, _ = ob.attention_fwd_masked(q, k, v, cu, ob.MASK_CAUSAL, 0.35)
    o2, _ = ob.attention_fwd_masked(q, k_rep, v_rep, cu, ob.MASK_CAUSAL, 0.35)
    np.testing.assert_allclose(o1, o2, atol=1e-14)
    dq1, dk1, dv1 = ob.attention_bwd_masked(d_o, q, k, v, cu, ob.MASK_CAUSAL, 0.35)
    dq2, dk2, dv2 = ob.attention_bwd_masked(d_o, q, k_rep, v_rep, cu, ob.MASK_CAUSAL, 0.35)
    np.testing.assert_allclose(dq1, dq2, atol=1e-13)
    # the gradient of a shared KV head is the sum over the heads that read it
    np.testing.assert_allclose(dk1, dk2.reshape(T, nkv, nq // nkv, d).sum(2), atol=1e-13)
    np.testing.assert_allclose(dv1, dv2.reshape(T, nkv, nq // nkv, d).sum(2), atol=1e-13)


# ------------------------------------------------------------------------------------------
# backward: central finite differences in fp64, for both block variants
# ------------------------------------------------------------------------------------------

def _fd_shapes():
    vit = si.small_shape(hidden=8, n_q_heads=2, n_kv_heads=2, head_dim=4, mlp_dim=12,
                         norm=si.NORM_LAYERNORM, mlp=si.MLP_GELU, mask=si.MASK_BIDIR,
                         use_rotary=False, has_bias=True)
    llm = si.small_shape(hidden=16, n_q_heads=4, n_kv_heads=2, head_dim=4, mlp_dim=10,
                         norm=si.NORM_RMSNORM, mlp=si.MLP_SWIGLU, mask=si.MASK_CAUSAL,
                         use_rotary=True, has_bias=False, norm_eps=1e-6)
    return [vit, llm]


@pytest.mark.parametrize("shape", _fd_shapes(), ids=["vit-like", "llm-like"])
def test_block_backward_matches_central_differences(shape):
    cu = si.lengths_to_cu([3, 5, 1])
    T = int(cu[-1])
    rng = np.random.default_rng(40)
    w = {n: rng.standard_normal(s) * 0.4 + (1.0 if n.endswith("_g") else 0.0)
         for n, s in si.weight_shapes(shape).items()}
    x = rng.standard_normal((T, shape.hidden))
    dy = rng.standard_normal((T, shape.hidden))
    y, cache = ob.block_fwd(shape, w, x, cu)
    dx, grads, _ = ob.block_bwd(shape, w, cache, dy, cu)
    assert set(grads) == set(w)

    def loss(w_, x_):
        return float((ob.block_fwd(shape, w_, x_, cu)[0] * dy).sum())

    h = 1e-5
    worst = 0.0
    # every element of x and a sample of every weight tensor
    for (i, j) in [(0, 0), (2, 3), (3, 1), (7, 5), (8, shape.hidden - 1)]:
        xp, xm = x.copy(), x.copy()
        xp[i, j] += h
        xm[i, j] -= h
        fd = (loss(w, xp) - loss(w, xm)) / (2 * h)
        worst = max(worst, abs(fd - dx[i, j]) / max(1.0, abs(fd)))
    for name, a in w.items():
        flat_idx = rng.choice(a.size, size=min(6, a.size), replace=False)
        for f in flat_idx:
            idx = np.unravel_index(f, a.shape)
            wp = {k: v.copy() for k, v in w.items()}
            wm = {k: v.copy() for k, v in w.items()}
            wp[name][idx] += h
            wm[name][idx] -= h
            fd = (loss(wp, x) - loss(wm, x)) / (2 * h)
            err = abs(fd - grads[name][idx]) / max(1.0, abs(fd))
            assert err < 1e-6, (name, idx, fd, grads[name][idx])
            worst = max(worst, err)
    assert worst < 1e-6


@pytest.mark.parametrize("shape", _fd_shapes(), ids=["vit-like", "llm-like"])
def test_stack_backward_matches_central_differences(shape):
    """Three chained blocks (the block stack the benchmark metric is quoted on): the input gradient and
    the gradients of each block's weights against central differences of <y, dy> through the whole
    stack; a backward that walked the blocks in the wrong order, or paired a block with another
    block's cache or weights, fails here."""
    cu = si.lengths_to_cu([4, 2, 3])
    T = int(cu[-1])
    rng = np.random.default_rng(41)
    ws = [{n: rng.standard_normal(sh) * 0.4 + (1.0 if n.endswith("_g") else 0.0)
           for n, sh in si.weight_shapes(shape).items()} for _ in range(3)]
    x = rng.standard_normal((T, shape.hidden))
    dy = rng.standard_normal((T, shape.hidden))
    y, dx, grads = ob.stack_fwd_bwd(shape, ws, x, dy, cu)
    assert len(grads) == 3 and all(set(g) == set(ws[0]) for g in grads)

    def loss(ws_, x_):
        a = x_
        for w_ in ws_:                       # the definition of a stack: block after block
            a = ob.block_fwd(shape, w_, a, cu)[0]
        return float((a * dy).sum())

    np.testing.assert_array_equal(y, _chain(shape, ws, x, cu))
    h, worst = 1e-5, 0.0
    for idx in [(0, 0), (T - 1, shape.hidden - 1), (3, 2), (5, 1)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd = (loss(ws, xp) - loss(ws, xm)) / (2 * h)
        worst = max(worst, abs(fd - dx[idx]) / max(abs(fd), 1e-3))
    for b in range(3):
        for name in ws[b]:
            flat = ws[b][name].reshape(-1)
            for e in sorted(set([0, flat.size // 2, flat.size - 1])):
                keep = flat[e]
                flat[e] = keep + h
                lp = loss(ws, x)
                flat[e] = keep - h
                lm = loss(ws, x)
                flat[e] = keep
                fd = (lp - lm) / (2 * h)
                got = grads[b][name].reshape(-1)[e]
                worst = max(worst, abs(fd - got) / max(abs(fd), 1e-3))
    assert worst < 1e-6, worst


def _chain(shape, ws, x, cu):
    a = x
    for w in ws:
        a = ob.block_fwd(shape, w, a, cu)[0]
    return a


def test_attention_backward_matches_central_differences():
    cu = si.lengths_to_cu([4, 6])
    T, nq, nkv, d = 10, 4, 2, 4
    rng = np.random.default_rng(41)
    q, k, v, d_o = (rng.standard_normal((T, n, d)) for n in (nq, nkv, nkv, nq))
    for mask in (ob.MASK_BIDIR, ob.MASK_CAUSAL):
        dq, dk, dv = ob.attention_bwd_masked(d_o, q, k, v, cu, mask, 0.5)
        f = lambda q_, k_, v_: float((ob.attention_fwd_masked(q_, k_, v_, cu, mask, 0.5)[0]
                                      * d_o).sum())
        h = 1e-5
        for arr, grad, pos in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
            for f_idx in rng.choice(arr.size, size=10, replace=False):
                idx = np.unravel_index(f_idx, arr.shape)
                args_p, args_m = [q.copy(), k.copy(), v.copy()], [q.copy(), k.copy(), v.copy()]
                args_p[pos][idx] += h
                args_m[pos][idx] -= h
                fd = (f(*args_p) - f(*args_m)) / (2 * h)
                assert abs(fd - grad[idx]) < 1e-7 * max(1.0, abs(fd))


# ------------------------------------------------------------------------------------------
# block level: packed == per-segment; fp32 instantiation == fp64; config-1 recipe
# ------------------------------------------------------------------------------------------

def test_block_packed_equals_each_segment_alone():
    shape = _fd_shapes()[1]          # rotary + causal + GQA: positions must restart per segment
    lens = [5, 9, 2]
    cu = si.lengths_to_cu(lens)
    T = int(cu[-1])
    rng = np.random.default_rng(42)
    w = {n: rng.standard_normal(s) * 0.3 + (1.0 if n.endswith("_g") else 0.0)
         for n, s in si.weight_shapes(shape).items()}
    x, dy = rng.standard_normal((T, 16)), rng.standard_normal((T, 16))
    y, c = ob.block_fwd(shape, w, x, cu)
    dx, grads, _ = ob.block_bwd(shape, w, c, dy, cu)
    gsum = {n: 0.0 for n in grads}
    for j in range(len(lens)):
        a, b = int(cu[j]), int(cu[j + 1])
        yj, cj = ob.block_fwd(shape, w, x[a:b], [0, b - a])
        dxj, gj, _ = ob.block_bwd(shape, w, cj, dy[a:b], [0, b - a])
        np.testing.assert_allclose(y[a:b], yj, atol=1e-12)
        np.testing.assert_allclose(dx[a:b], dxj, atol=1e-12)
        for n in gj:
            gsum[n] = gsum[n] + gj[n]
    for n in grads:
        np.testing.assert_allclose(grads[n], gsum[n], atol=1e-11)


def test_fp32_oracle_agrees_with_fp64_on_config1():
    shape = si.CONFIGS[1]
    lens = si.tiny_segment_lengths(seed=0)
    assert len(lens) == 4 and lens.min() >= 64 and lens.max() <= 384 and lens.sum() <= 1024
    cu = si.lengths_to_cu(lens)
    T = int(cu[-1])
    w = si.block_weights(shape, seed=0)
    x, dy = si.activations(T, shape.hidden, seed=0)
    y64, c64 = ob.block_fwd(shape, w, x, cu, np.float64)
    y32, c32 = ob.block_fwd(shape, w, x, cu, np.float32)
    assert y32.dtype == np.float32
    dx64, g64, _ = ob.block_bwd(shape, w, c64, dy, cu, np.float64)
    dx32, g32, _ = ob.block_bwd(shape, w, c32, dy, cu, np.float32)
    from conftest import rel_err
    assert rel_err(y32, y64) < 1e-5 and rel_err(dx32, dx64) < 1e-5
    for n in g64:
        assert rel_err(g32[n], g64[n]) < 1e-5, n


def test_algorithmic_flops_hand_count():
    shape = si.small_shape(hidden=64, n_q_heads=2, n_kv_heads=1, head_dim=32, mlp_dim=128,
                           mlp=si.MLP_SWIGLU, mask=si.MASK_CAUSAL)
    cu = [0, 3, 5]
    # per token: qkv 2*64*128, out 2*64*64, mlp 3 matrices 2*64*128 each
    gemm = 2 * 64 * 128 + 2 * 64 * 64 + 3 * 2 * 64 * 128
    attn = 4 * 2 * 32 * (3 * 4 // 2 + 2 * 3 // 2)
    assert ob.algorithmic_flops(shape, cu, n_blocks=2) == 3 * 2 * (5 * gemm + attn)
    shape_b = si.small_shape(hidden=64, n_q_heads=2, n_kv_heads=2, head_dim=32, mlp_dim=128,
                             mlp=si.MLP_GELU, mask=si.MASK_BIDIR)
    gemm_b = 2 * 64 * 192 + 2 * 64 * 64 + 2 * 2 * 64 * 128
    assert ob.algorithmic_flops(shape_b, cu, n_blocks=1) == 3 * (5 * gemm_b + 4 * 2 * 32 * 13)
