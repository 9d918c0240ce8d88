"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
rejects bad arguments without touching a device, and its host packer equals the oracle's."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2407_20761_amd as ob
import synth_inputs as si
from oracle import packer as op

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "omnibal.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ob_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 18
    for name in declared:
        assert hasattr(ob.lib, name), name
    assert declared == set(ob.EXPORTED)
    assert ob.lib.ob_has_device_code() == 1


# ---- packer: bit-exact against the oracle ---------------------------------------------------

@pytest.mark.parametrize("seed", [0, 3])
def test_pack_isf_equals_oracle(seed):
    tiles, tok = si.synthetic_dataset(2500, seed)
    for (Qv, Qt, Qvm, Qtm) in [(10 ** 9, 16384, 10 ** 9, 16384 - 128), (12, 10 ** 9, 12, 10 ** 9),
                               (42, 16384, 42, 16384 - 128), (14, 9000, 13, 8000)]:
        g, left, per = ob.ob_pack_isf(tiles, tok, Qv, Qt, Qvm, Qtm, 10, seed)
        P, L, pi = op.isf(tiles, tok, Qv, Qt, Qvm, Qtm, 10, seed)
        assert [a.tolist() for a in g] == P
        assert left.tolist() == L
        assert per.tolist()[:len(pi)] == pi and not per.tolist()[len(pi):].count(1)


def test_pack_isf_tiny_and_degenerate():
    img, tok = [1, 2, 1, 3, 1, 1], [4, 3, 5, 2, 8, 2]
    for seed in range(5):
        g, left, _ = ob.ob_pack_isf(img, tok, 4, 10, 4, 8, 3, seed)
        P, L, _ = op.isf(img, tok, 4, 10, 4, 8, 3, seed)
        assert [a.tolist() for a in g] == P and left.tolist() == L
    g, left, _ = ob.ob_pack_isf([], [], 4, 10, 4, 8, 3, 0)
    assert g == [] and left.tolist() == []
    g, left, _ = ob.ob_pack_isf([1], [5], 4, 10, 4, 8, 0, 0)       # zero iterations
    assert g == [] and left.tolist() == [0]
    with pytest.raises(ob.OmnibalError) as e:
        ob.ob_pack_isf(img, tok, 2, 10, 2, 8, 3, 0)                # sample 3 has 3 > 2 tiles
    assert e.value.status == ob.OB_EINVAL and "sample 3" in str(e.value)


def test_pack_random_and_cu_builders_equal_oracle():
    g, left = ob.ob_pack_random(1003, 7, 11)
    G, L = op.random_groups(1003, 7, 11)
    assert [a.tolist() for a in g] == G and left.tolist() == L
    tiles, tok = si.synthetic_dataset(50, 2)
    cu, mx = ob.ob_build_cu_seqlens_llm([4, 9, 1], tok)
    assert cu.tolist() == op.cu_seqlens_llm([4, 9, 1], tok) and mx == max(tok[[4, 9, 1]])
    assert ob.ob_build_cu_seqlens_vit(12, 1025).tolist() == op.cu_seqlens_vit(12, 1025)
    with pytest.raises(ob.OmnibalError):
        ob.ob_build_cu_seqlens_vit(0, 1025)


def test_metrics_equal_oracle():
    for v in ([2, 4], [5, 5, 5], [1, 2, 3, 6], [100, 50], [7]):
        assert ob.ob_pad_ratio(v) == pytest.approx(op.pad_ratio(v), abs=1e-15)
        assert ob.ob_dist_ratio(v) == pytest.approx(op.dist_ratio(v), abs=1e-15)


# ---- argument validation: every error path returns before any launch -----------------------

def _seg(cu, total=None, max_seqlen=None, fake_dev=True):
    cu = np.asarray(cu, dtype=np.int32)
    s = ob.Segments(cu, device=None, max_seqlen=max_seqlen)
    if fake_dev:
        s.c.cu_dev = 0x1000                     # never dereferenced: validation fails first
    if total is not None:
        s.c.total_tokens = total
    return s


def _attn_status(seg, nq=4, nkv=2, d=64, ldq=256, ldkv=128, ldo=256, mask=1, dtype=0, null_q=False):
    p = C.c_void_p(0x1000)
    return ob.lib.ob_varlen_attn_fwd(None if null_q else p, p, p, p, p, ldq, ldkv, ldo,
                                     C.byref(seg.c), nq, nkv, d, 0.125, mask, dtype, None)


def test_attention_argument_validation():
    good = _seg([0, 5, 9])
    assert _attn_status(good, null_q=True) == ob.OB_EINVAL
    assert _attn_status(_seg([1, 5, 9])) == ob.OB_ESEGMENTS               # cu[0] != 0
    assert "must be 0" in ob.ob_last_error()
    assert _attn_status(_seg([0, 5, 5, 9])) == ob.OB_ESEGMENTS            # empty segment
    assert _attn_status(_seg([0, 7, 5, 9])) == ob.OB_ESEGMENTS            # not monotone
    assert _attn_status(_seg([0, 5, 9], total=10)) == ob.OB_ESEGMENTS     # cu[n] != T
    assert _attn_status(_seg([0, 5, 9], max_seqlen=3)) == ob.OB_ESEGMENTS
    assert _attn_status(good, nq=4, nkv=3) == ob.OB_EINVAL
    assert _attn_status(good, d=96) == ob.OB_EUNSUPPORTED
    assert _attn_status(good, dtype=7) == ob.OB_EINVAL
    assert _attn_status(good, mask=7) == ob.OB_EINVAL
    assert _attn_status(good, ldq=100) == ob.OB_EINVAL
    assert _attn_status(_seg([0, 5, 9], fake_dev=False)) == ob.OB_EINVAL  # cu_dev null
    p = C.c_void_p(0x1000)
    st = ob.lib.ob_varlen_attn_bwd(p, p, p, p, p, p, p, p, p, 256, 128, 256, C.byref(good.c),
                                   4, 2, 64, 0.125, 1, 0, p, 16, None)
    assert st == ob.OB_EWORKSPACE
    # the variant with the library's static scratch: same checks, and sizes beyond its array are refused
    st = ob.lib.ob_varlen_attn_bwd_static(p, p, p, p, p, p, p, p, p, 256, 128, 256, C.byref(_seg([0, 7, 5, 9]).c),
                                          4, 2, 64, 0.125, 1, 0, None)
    assert st == ob.OB_ESEGMENTS
    st = ob.lib.ob_varlen_attn_bwd_static(None, p, p, p, p, p, p, p, p, 256, 128, 256, C.byref(good.c),
                                          4, 2, 64, 0.125, 1, 0, None)
    assert st == ob.OB_EINVAL
    big = _seg([0, 1 << 20])
    st = ob.lib.ob_varlen_attn_bwd_static(p, p, p, p, p, p, p, p, p, 512, 512, 512, C.byref(big.c),
                                          8, 8, 64, 0.125, 1, 0, None)
    assert st == ob.OB_EWORKSPACE and "static" in ob.ob_last_error()


def test_block_argument_validation_and_sizes():
    shape = si.CONFIGS[1]
    desc = ob.make_desc(shape)
    T = 777
    sb, wb = ob.ob_block_saved_bytes(desc, T), ob.ob_block_workspace_bytes(desc, T)
    # saved holds h1, qkv, o, x1, h2, up, act (bf16) + lse + two stat arrays (fp32)
    lower = T * (4 * 256 + 768 + 1024 + 1024) * 2 + 4 * T * 4 + 2 * T * 2 * 4
    assert lower <= sb <= lower + 10 * 256 and wb > 0
    offs = [ob.ob_block_saved_offset(desc, T, n) for n in
            ("h1", "qkv", "o", "lse", "x1", "h2", "up", "act", "stat1", "stat2")]
    assert offs == sorted(offs) and offs[0] == 0 and all(o % 256 == 0 for o in offs)
    assert ob.ob_block_saved_offset(desc, T, "nope") == C.c_size_t(-1).value
    # the fp32 debug path stores the same members with four-byte elements
    d32 = ob.make_desc(shape, dtype=ob.OB_FP32)
    sb32 = ob.ob_block_saved_bytes(d32, T)
    lower32 = T * (4 * 256 + 768 + 1024 + 1024) * 4 + 4 * T * 4 + 2 * T * 2 * 4
    assert lower32 <= sb32 <= lower32 + 10 * 256 and ob.ob_block_workspace_bytes(d32, T) > 0
    assert ob.ob_block_saved_offset(d32, T, "qkv") == (T * 256 * 4 + 255) // 256 * 256

    p = C.c_void_p(0x1000)
    w = ob.ob_block_weights(*[0x1000] * 12)
    seg = _seg([0, 300, 777])

    def fwd(desc_, w_=w, seg_=seg, sb_=sb, wb_=wb, x=p):
        return ob.lib.ob_block_fwd(C.byref(desc_), C.byref(w_), x, p, p, sb_, C.byref(seg_.c), p,
                                   wb_, None)

    assert fwd(desc, x=None) == ob.OB_EINVAL
    assert fwd(desc, sb_=sb - 1) == ob.OB_EWORKSPACE
    assert fwd(desc, wb_=wb - 1) == ob.OB_EWORKSPACE
    assert fwd(desc, seg_=_seg([0, 300, 776], total=777)) == ob.OB_ESEGMENTS
    w_missing = ob.ob_block_weights(*[0x1000] * 12)
    w_missing.b_qkv = None
    assert fwd(desc, w_=w_missing) == ob.OB_EINVAL            # has_bias but no bias pointer
    for field, val, status in (("head_dim", 96, ob.OB_EUNSUPPORTED), ("hidden", 250, ob.OB_EUNSUPPORTED),
                               ("n_kv_heads", 3, ob.OB_EINVAL), ("dtype", 7, ob.OB_EINVAL),
                               ("norm", 5, ob.OB_EINVAL), ("hidden", 16384, ob.OB_EUNSUPPORTED)):
        d2 = ob.make_desc(shape)
        setattr(d2, field, val)
        assert fwd(d2) == status, field
    g = ob.ob_block_grads(*[0x1000] * 12)
    g.w_o = None
    st = ob.lib.ob_block_bwd(C.byref(desc), C.byref(w), C.byref(g), 0, p, p, p, p, sb,
                             C.byref(seg.c), p, wb, None)
    assert st == ob.OB_EINVAL


def test_gemm_argument_validation():
    p = C.c_void_p(0x1000)
    call = lambda layout, M, N, K, ws=p, wsb=1 << 40: ob.lib.ob_gemm_bf16(layout, M, N, K, p, p, p,
                                                                         None, None, ws, wsb, None)
    assert call(3, 64, 64, 64) == ob.OB_EINVAL
    assert call(0, 64, 100, 64) == ob.OB_EUNSUPPORTED
    assert call(0, 64, 64, 100) == ob.OB_EUNSUPPORTED
    assert call(2, 100, 64, 77) == ob.OB_EUNSUPPORTED
    for layout in (0, 1, 2):                      # enough tiles, or a short contraction: no scratch
        assert ob.ob_gemm_workspace_bytes(layout, 128, 64, 128) == 0
        assert ob.ob_gemm_workspace_bytes(layout, 16384, 4096, 16384) == 0
    # 64 tiles of 128 x 128 over 193 K steps: 4 slices of fp32 sums, a tile on every CU
    assert ob.ob_gemm_workspace_bytes(2, 1024, 1024, 12300) == 4 * 1024 * 1024 * 4
    assert call(2, 1024, 1024, 12300, wsb=1024) == ob.OB_EWORKSPACE
    assert ob.lib.ob_debug_materialize_mask(C.byref(_seg([0, 4]).c), 1, None, None) == ob.OB_EINVAL


def test_gemm_workspace_is_bounded_and_tile_granular():
    """The split planner on arbitrary shapes: scratch is a whole number of 128 x 128 fp32 tile sums,
    never more than 8 slices of less than a round of 256 x 256 tiles, and a function of the shape only."""
    rng = np.random.default_rng(5)
    for _ in range(3000):
        M = int(rng.choice([1, 64, 255, 256, 257, 4096, 12300, 16384, 1 << 20, int(rng.integers(1, 1 << 21))]))
        N = 64 * int(rng.choice([1, 2, 16, 50, 64, 224, 448, int(rng.integers(1, 4096))]))
        K = int(rng.choice([64, 1000, 1024, 4096, 8192, 12300, 16325, 1 << 20, int(rng.integers(1, 1 << 21))]))
        layout = int(rng.integers(0, 3))
        b = ob.ob_gemm_workspace_bytes(layout, M, N, K)
        assert b % (128 * 128 * 4) == 0 and b <= 8 * 255 * 256 * 256 * 4, (layout, M, N, K, b)
        assert b == ob.ob_gemm_workspace_bytes(layout, M, N, K)


# ---- grouping arms, partition search and re-computation plan: library == oracle ----------------

@pytest.mark.parametrize("seed", [0, 4])
def test_size_grouping_arms_equal_oracle(seed):
    tiles, tok = si.synthetic_dataset(1234, seed)
    for B in (1, 6, 50):
        g, left = ob.ob_pack_length_group(tok, B, seed)
        G, Left = op.length_groups(tok, B, seed)
        assert [a.tolist() for a in g] == G and left.tolist() == Left
        g, left = ob.ob_pack_device_group(tok, B, seed)
        G, Left = op.device_groups(tok, B, seed)
        assert [a.tolist() for a in g] == G and left.tolist() == Left
    with pytest.raises(RuntimeError):
        ob.ob_pack_length_group(tok, 0, seed)


def test_bmp_anchor_and_search_equal_oracle():
    import random
    from oracle import planner as pl
    rng = random.Random(5)
    assert ob.ob_bmp_anchor([1.0] * 20, 4) == (6, 11, 16)
    ranked, n = ob.ob_bmp_search([1.0] * 20, [0.0] * 20, 4, 1, top_k=100)
    assert n == 27 and len(ranked) == 27                      # Sec. 4.2: r = 1, N = 4
    for _ in range(40):
        N = rng.randint(1, 5)
        L = rng.randint(N, 30)
        # integer-valued times and volumes: every score is exact in double, so ranks must agree exactly
        fwd = [float(rng.randint(1, 40)) for _ in range(L)]
        activ = [float(rng.randint(0, 9)) for _ in range(L)]
        r, w, k = rng.randint(0, 3), rng.choice([0.0, 1.0, 4.0]), rng.randint(1, 20)
        assert ob.ob_bmp_anchor(fwd, N) == pl.anchor(fwd, N)
        got, n_got = ob.ob_bmp_search(fwd, activ, N, r, w, k)
        want, n_want = pl.search(fwd, activ, N, r, w, k)
        assert n_got == n_want and got == want
    # real-valued profile: same candidates, scores equal to rounding
    fwd = [rng.uniform(0.5, 3.0) for _ in range(40)]
    activ = [rng.uniform(0.0, 2.0) for _ in range(40)]
    got, n_got = ob.ob_bmp_search(fwd, activ, 4, 2, 1.0, 125)
    want, n_want = pl.search(fwd, activ, 4, 2, 1.0, 125)
    assert n_got == n_want and sorted(P for _, P in got) == sorted(P for _, P in want)
    assert all(abs(a - b) <= 1e-9 * max(1.0, abs(b)) for (a, _), (b, _) in zip(got, want))
    for bad in (lambda: ob.ob_bmp_anchor([1.0, 2.0], 3), lambda: ob.ob_bmp_anchor([1.0, -2.0], 2),
                lambda: ob.ob_bmp_search([1.0] * 60, [0.0] * 60, 30, 3)):
        with pytest.raises(RuntimeError):
            bad()


def test_recompute_plan_equals_oracle():
    import random
    from oracle import planner as pl
    rng = random.Random(2)
    for _ in range(300):
        nv, nt = rng.randint(0, 8), rng.randint(0, 8)
        bv, bt = rng.randint(1, 30), rng.randint(1, 30)
        mv, mt = rng.choice([0.0, 1.0, 1.5, 2.0, 3.0]), rng.choice([0.0, 1.0, 1.5, 2.0, 3.0])
        free, e = rng.randint(0, 300), rng.randint(0, 3)
        assert ob.ob_recompute_plan(free, nv, bv, mv, nt, bt, mt, e) == pl.recompute_plan(free, nv, bv, mv, nt, bt, mt, e)
    # with the library's own byte counts: 8 config-3 blocks into 10 GiB
    desc = ob.make_desc(si.CONFIGS[3])
    per_block = ob.ob_block_saved_bytes(desc, 16384)
    assert ob.ob_recompute_plan(10 << 30, 0, 1, 0.0, 8, per_block, 5.0) == (0, min(8, (10 << 30) // per_block))
    with pytest.raises(RuntimeError):
        ob.ob_recompute_plan(-1, 1, 1, 1.0, 1, 1, 1.0)


# ---- ViT -> LLM hand-over: validation happens on the host, before anything is launched ---------

def test_connector_argument_validation_and_sizes():
    d = ob.make_connector_desc(128, 256, grid=4)
    n_tiles, n_tok = 3, 3 * 4
    sv, wk = ob.ob_connector_saved_bytes(d, n_tiles), ob.ob_connector_workspace_bytes(d, n_tiles)
    # un [n_tok, 4 Hv] + h, a [n_tok, Ht] bf16 + (mean, rstd) per token, each member padded to 256 bytes
    pad = lambda b: (b + 255) // 256 * 256
    assert sv == pad(n_tok * 512 * 2) + 2 * pad(n_tok * 256 * 2) + pad(n_tok * 8)
    assert wk >= pad(n_tok * 512 * 2) + 3 * pad(n_tok * 256 * 2)
    for bad in (ob.make_connector_desc(100, 256, 4), ob.make_connector_desc(128, 250, 4),
                ob.make_connector_desc(4160, 256, 4), ob.make_connector_desc(128, 256, 4, dtype=7)):
        assert ob.ob_connector_saved_bytes(bad, n_tiles) == 0
    # the fp32 debug variant keeps u as well, four bytes per element
    d32 = ob.make_connector_desc(128, 256, grid=4, dtype=ob.OB_FP32)
    assert ob.ob_connector_saved_bytes(d32, n_tiles) == 2 * pad(n_tok * 512 * 4) + 2 * pad(n_tok * 256 * 4) + pad(n_tok * 8)
    assert ob.ob_connector_workspace_bytes(d32, n_tiles) == 3 * pad(n_tok * 256 * 4) + 2 * pad(n_tok * 512 * 4)
    assert ob.ob_connector_saved_bytes(ob.make_connector_desc(128, 256, 5), n_tiles) == 0     # odd grid
    assert ob.ob_connector_saved_bytes(d, 0) == 0

    # pointer and row-list checks need no device: fake non-null addresses are never dereferenced
    class Fake:
        def __init__(self, n=1 << 30): self.n = n
        def data_ptr(self): return 0x1000
        def numel(self): return self.n
        def element_size(self): return 1
    w = {n: Fake() for n in ob.CONNECTOR_FIELDS}
    rows = ob.RowIndex(np.arange(n_tok), device=None)
    rows.dev = Fake()
    call = lambda **kw: ob.ob_connector_fwd(kw.get("d", d), kw.get("w", w), Fake(), n_tiles, kw.get("rows", rows),
                                            Fake(), kw.get("T", 40), kw.get("saved", Fake()), kw.get("ws", Fake()),
                                            stream=type("S", (), {"cuda_stream": 0})())
    def status(**kw):
        with pytest.raises(ob.OmnibalError) as e:
            call(**kw)
        return e.value.status
    assert status(w={**w, "b2": None}) == ob.OB_EINVAL
    assert status(T=n_tok - 1) == ob.OB_EINVAL                       # fewer LLM rows than visual tokens
    dup = ob.RowIndex(np.r_[np.arange(n_tok - 1), 0], device=None); dup.dev = Fake()
    assert status(rows=dup) == ob.OB_EINVAL and "twice" in ob.ob_last_error()
    far = ob.RowIndex(np.r_[np.arange(n_tok - 1), 40], device=None); far.dev = Fake()
    assert status(rows=far) == ob.OB_EINVAL and "outside" in ob.ob_last_error()
    assert status(saved=Fake(sv - 1)) == ob.OB_EWORKSPACE
    assert status(ws=Fake(wk - 1)) == ob.OB_EWORKSPACE
    bwd = lambda flags: ob.ob_connector_bwd(d, w, w, flags, Fake(), Fake(), Fake(), n_tiles, rows, 40, Fake(), Fake(),
                                            stream=type("S", (), {"cuda_stream": 0})())
    with pytest.raises(ob.OmnibalError) as e:
        bwd(ob.OB_BWD_RECOMPUTE)
    assert e.value.status == ob.OB_EINVAL
