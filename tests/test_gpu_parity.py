"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Tolerance: max|err| / max|ref| <= 2e-2 per tensor for the bf16 path (the benchmark contract's
bound; bf16 has 8 mantissa bits, every stored intermediate costs up to 2^-9 relative) and <= 1e-4
for the fp32 debug path.  Segment offsets and masks are compared bit for bit.
"""
import numpy as np
import pytest
import torch

import paper_2407_20761_amd as ob
import synth_inputs as si
from conftest import rel_err
from oracle import block as orc
from oracle import packer as orc_pack

pytestmark = pytest.mark.gpu
TOL = 2e-2
TOL_FP32 = 1e-4

if torch.cuda.is_available():
    from gpu_util import BlockRun, bytes_buf, run_block, saved_view, to_dev, to_np


def _say(msg):
    print(msg, flush=True)


# ---- GEMM ------------------------------------------------------------------------------------

@pytest.mark.parametrize("layout", [0, 1, 2])
@pytest.mark.parametrize("M,N,K", [(300, 192, 128), (1, 64, 64), (4100, 8192, 256),
                                   (1025, 3200, 448), (257, 256, 64), (130, 320, 192), (513, 512, 320),
                                   (4096, 8192, 8192)])      # 512 tiles over a long contraction: the round-robin patch order
def test_gemm_against_fp64_matmul(layout, M, N, K):
    if layout == 2 and M % 64:
        M = (M + 63) // 64 * 64          # the output rows of a weight gradient are a feature dim
    if layout == 2:
        K = K + 37                        # the token dimension is ragged
    _say(f"gemm layout={layout} M={M} N={N} K={K}")
    rng = np.random.default_rng(M + N + K + layout)
    A = si.round_to_bf16(rng.standard_normal((M, K), dtype=np.float32))
    B = si.round_to_bf16(rng.standard_normal((N, K), dtype=np.float32))
    bias = si.round_to_bf16(rng.standard_normal((N,), dtype=np.float32))
    R = si.round_to_bf16(rng.standard_normal((M, N), dtype=np.float32) * 4)
    ref = A.astype(np.float64) @ B.astype(np.float64).T
    a_dev = to_dev(A if layout != 2 else A.T.copy())
    b_dev = to_dev(B if layout == 0 else B.T.copy())
    ws = bytes_buf(ob.ob_gemm_workspace_bytes(layout, M, N, K))
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ob.ob_gemm_bf16(layout, M, N, K, a_dev, b_dev, c, None, None, ws)
    assert rel_err(to_np(c), ref) < 5e-3
    c2 = to_dev(R)
    ob.ob_gemm_bf16(layout, M, N, K, a_dev, b_dev, c2, to_dev(bias), c2, ws)   # in-place + bias
    assert rel_err(to_np(c2), ref + bias + R) < 5e-3


@pytest.mark.parametrize("layout,M,N,K", [(2, 1024, 1024, 12300), (2, 2048, 1024, 12300), (2, 512, 1024, 8219),
                                          (2, 64, 64, 1000), (0, 257, 256, 4096), (1, 700, 512, 2112),
                                          (2, 4096, 5120, 4100), (0, 4100, 4992, 4096), (1, 2500, 8192, 4160)])
def test_gemm_split_contraction(layout, M, N, K):
    """The tiles of an incomplete last round (all tiles, for the small weight gradients of config 2) have
    their contraction cut into slices whose fp32 sums a second kernel adds; the last slice is shorter
    than the rest, and the last three cases keep whole tiles beside the split ones."""
    _say(f"gemm split layout={layout} M={M} N={N} K={K}")
    need = ob.ob_gemm_workspace_bytes(layout, M, N, K)
    assert need > 0                                                  # this case does split
    rng = np.random.default_rng(M + N + K + layout)
    A = si.round_to_bf16(rng.standard_normal((M, K), dtype=np.float32))
    B = si.round_to_bf16(rng.standard_normal((N, K), dtype=np.float32))
    bias = si.round_to_bf16(rng.standard_normal((N,), dtype=np.float32))
    R = si.round_to_bf16(rng.standard_normal((M, N), dtype=np.float32) * 4)
    ref = A.astype(np.float64) @ B.astype(np.float64).T
    a_dev = to_dev(A if layout != 2 else A.T.copy())
    b_dev = to_dev(B if layout == 0 else B.T.copy())
    ws = bytes_buf(need)
    ws.fill_(0x7F)                                                   # stale contents must not matter
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ob.ob_gemm_bf16(layout, M, N, K, a_dev, b_dev, c, None, None, ws)
    assert rel_err(to_np(c), ref) < 5e-3
    c2 = to_dev(R)
    ob.ob_gemm_bf16(layout, M, N, K, a_dev, b_dev, c2, to_dev(bias), c2, ws)   # in-place + bias
    assert rel_err(to_np(c2), ref + bias + R) < 5e-3
    c3 = torch.empty_like(c)
    ob.ob_gemm_bf16(layout, M, N, K, a_dev, b_dev, c3, None, None, None)       # no scratch: unsplit
    assert rel_err(to_np(c3), ref) < 5e-3


def test_gemm_random_shapes():
    """Forty seeded shapes across the planner's cases (tile size, whole and split tiles, patch order,
    ragged edges), each with scratch (bias and in-place residual) and without (plain, unsplit)."""
    rng = np.random.default_rng(2024)
    done = split = 0
    while done < 40:
        layout = int(rng.integers(0, 3))
        M = int(rng.choice([64, 128, 192, 256, 320, 1024, 2048, 3200, 4096, int(rng.integers(1, 5000))]))
        N = 64 * int(rng.choice([1, 2, 3, 4, 8, 16, 20, 24, 32, 50, int(rng.integers(1, 64))]))
        K = int(rng.choice([64, 128, 1024, 2048, 4096, 8192, 8256, 12300, int(rng.integers(1, 20000))]))
        if layout == 2:
            M = (M + 63) // 64 * 64
        else:
            K = (K + 63) // 64 * 64
        if M * N * K > 3e10:
            continue
        A = si.round_to_bf16(rng.standard_normal((M, K), dtype=np.float32))
        B = si.round_to_bf16(rng.standard_normal((N, K), dtype=np.float32))
        bias = si.round_to_bf16(rng.standard_normal((N,), dtype=np.float32))
        R = si.round_to_bf16(rng.standard_normal((M, N), dtype=np.float32) * 4)
        ref = A.astype(np.float64) @ B.astype(np.float64).T
        a_dev = to_dev(A if layout != 2 else A.T.copy())
        b_dev = to_dev(B if layout == 0 else B.T.copy())
        need = ob.ob_gemm_workspace_bytes(layout, M, N, K)
        _say(f"gemm random layout={layout} M={M} N={N} K={K} scratch={need}")
        ws = bytes_buf(need)
        ws.fill_(0x7F)
        c = to_dev(R)
        ob.ob_gemm_bf16(layout, M, N, K, a_dev, b_dev, c, to_dev(bias), c, ws)
        assert rel_err(to_np(c), ref + bias + R) < 5e-3
        c2 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        ob.ob_gemm_bf16(layout, M, N, K, a_dev, b_dev, c2, None, None, None)
        assert rel_err(to_np(c2), ref) < 5e-3
        done += 1
        split += need > 0
    assert split >= 10          # the sweep does reach the split path


@pytest.mark.parametrize("layout,M,N,K", [(0, 16384, 28672, 4096), (1, 16384, 4096, 14336), (2, 4096, 14336, 16325)])
def test_gemm_full_size_sampled_outputs(layout, M, N, K):
    """Config 3's largest GEMMs in the launch shape the benchmark times (256x256 tiles, one per CU);
    the definition is evaluated for sampled outputs: corners, tile borders, random positions."""
    _say(f"gemm full size layout={layout} M={M} N={N} K={K}")
    rng = np.random.default_rng(7 + layout)
    A = si.round_to_bf16(rng.standard_normal((M, K), dtype=np.float32))
    B = si.round_to_bf16(rng.standard_normal((N, K), dtype=np.float32))
    a_dev = to_dev(A if layout != 2 else np.ascontiguousarray(A.T))
    b_dev = to_dev(B if layout == 0 else np.ascontiguousarray(B.T))
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ob.ob_gemm_bf16(layout, M, N, K, a_dev, b_dev, c, None, None, None)
    rows = np.concatenate([[0, 1, 15, 16, 127, 128, 255, 256, M - 257, M - 256, M - 1], rng.integers(0, M, 200)])
    cols = np.concatenate([[0, 3, 4, 16, 63, 64, 255, 256, N - 257, N - 129, N - 1], rng.integers(0, N, 200)])
    ref = A[rows].astype(np.float64) @ B[cols].astype(np.float64).T          # every sampled row x every sampled column
    got = to_np(c[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
    assert rel_err(got, ref) < 5e-3


@pytest.mark.parametrize("layout", [1, 2])
def test_gemm_k_major_operand_larger_than_4_gib(layout):
    """A k-major operand of more than 2^32 bytes: the 32-bit range of a buffer descriptor must not
    cut the contraction short (sampled outputs against fp64 numpy products of the same operand values,
    brought back to the host row by row)."""
    if layout == 2:
        M, N, K = 16384, 64, 262144 + 37         # A [K, M]: 8.6 GB, contraction in two slices, the second from 4.3 GB on
    else:
        M, N, K = 64, 196608 + 64, 16384         # B [K, N]: 6.4 GB
    _say(f"gemm >4 GiB operand layout={layout} M={M} N={N} K={K}")
    gen = torch.Generator(device="cuda").manual_seed(11 + layout)
    a = torch.randn((K, M) if layout == 2 else (M, K), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    b = torch.randn((K, N), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ws = bytes_buf(ob.ob_gemm_workspace_bytes(layout, M, N, K))
    assert layout != 2 or ob.ob_gemm_workspace_bytes(layout, M, N, K) > 0
    ob.ob_gemm_bf16(layout, M, N, K, a, b, c, None, None, ws)
    rows = torch.tensor([0, 1, M // 2 + 3, M - 1], device="cuda")
    cols = torch.tensor([0, 5, N // 2 + 1, N - 64, N - 1], device="cuda")
    a_rows = to_np(a[:, rows].T if layout == 2 else a[rows])                 # [4, K] on the host, float64
    b_cols = to_np(b[:, cols])                                               # [K, 5]
    ref = a_rows @ b_cols
    got = to_np(c[rows][:, cols])
    assert rel_err(got, ref) < 5e-3


# ---- attention ------------------------------------------------------------------------------

ATTN_CASES = [
    # lens, nq, nkv, d, mask
    ([1, 63, 64, 65, 130, 300], 4, 2, 64, orc.MASK_CAUSAL),
    ([1, 63, 64, 65, 130, 300], 4, 4, 64, orc.MASK_BIDIR),
    ([129, 7, 256, 1], 8, 2, 128, orc.MASK_CAUSAL),
    ([1025, 1025], 3, 3, 128, orc.MASK_BIDIR),
    ([700], 2, 1, 128, orc.MASK_CAUSAL),
]


@pytest.mark.parametrize("lens,nq,nkv,d,mask", ATTN_CASES)
def test_varlen_attention_fwd_bwd(lens, nq, nkv, d, mask):
    _check_attention(lens, nq, nkv, d, mask, seed=len(lens) + d)


def test_varlen_attention_random_cases():
    """Sixteen seeded cases: 1-8 segments of 1-900 tokens (half of them forced onto tile borders and
    their neighbours), GQA groups 1, 2, 4, 6, both head sizes, both masks."""
    rng = np.random.default_rng(77)
    for case in range(16):
        n = int(rng.integers(1, 9))
        lens = [int(rng.choice([63, 64, 65, 127, 128, 129, 191, 192, 193, 256, 257, 512, 513]))
                if rng.random() < 0.5 else int(rng.integers(1, 901)) for _ in range(n)]
        group = int(rng.choice([1, 2, 4, 6]))
        nkv = int(rng.integers(1, 3))
        _check_attention(lens, nkv * group, nkv, int(rng.choice([64, 128])),
                         orc.MASK_CAUSAL if case % 2 else orc.MASK_BIDIR, seed=100 + case)


def _check_attention(lens, nq, nkv, d, mask, seed, per_segment=False):
    _say(f"attention n_seg={len(lens)} lens={lens if len(lens) <= 40 else str(lens[:40]) + ' ...'} nq={nq} nkv={nkv} d={d} mask={mask}")
    cu = si.lengths_to_cu(lens)
    T = int(cu[-1])
    q, k, v, d_o = si.qkv_tensors(T, nq, nkv, d, seed=seed)
    scale = 1.0 / np.sqrt(d)
    if per_segment:
        # large batches: the oracle's per-segment form (pinned equal to the masked form), printing as it goes
        o_ref, lse_ref = np.empty((T, nq, d)), np.empty((nq, T))
        dq_ref, dk_ref, dv_ref = np.empty((T, nq, d)), np.empty((T, nkv, d)), np.empty((T, nkv, d))
        for j in range(len(lens)):
            a, b = int(cu[j]), int(cu[j + 1])
            sub = [t[a:b].astype(np.float64) for t in (d_o, q, k, v)]
            o_ref[a:b], lse_ref[:, a:b] = orc.attention_fwd_masked(sub[1], sub[2], sub[3], [0, b - a], mask, scale)
            dq_ref[a:b], dk_ref[a:b], dv_ref[a:b] = orc.attention_bwd_masked(*sub, [0, b - a], mask, scale)
            _say(f"    oracle segment {j} [{a},{b}) done")
    else:
        o_ref, lse_ref = orc.attention_fwd(*(a.astype(np.float64) for a in (q, k, v)), cu, mask, scale)
        dq_ref, dk_ref, dv_ref = orc.attention_bwd(*(a.astype(np.float64) for a in (d_o, q, k, v)),
                                                   cu, mask, scale)
    # q, k, v live as column slices of one [T, (nq + 2 nkv) d] buffer, as inside the block
    Dq = (nq + 2 * nkv) * d
    qkv = to_dev(np.concatenate([q.reshape(T, -1), k.reshape(T, -1), v.reshape(T, -1)], axis=1))
    qd, kd, vd = qkv[:, :nq * d], qkv[:, nq * d:(nq + nkv) * d], qkv[:, (nq + nkv) * d:]
    o = torch.empty((T, nq * d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((nq, T), dtype=torch.float32, device="cuda")
    seg = ob.Segments(cu)
    ob.ob_varlen_attn_fwd(qd, kd, vd, o, lse, Dq, Dq, nq * d, seg, nq, nkv, d, scale, mask)
    assert rel_err(to_np(o).reshape(T, nq, d), o_ref) < TOL
    assert np.abs(to_np(lse) - lse_ref).max() < 2e-2
    dqkv = torch.full((T, Dq), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = bytes_buf(ob.ob_varlen_attn_bwd_workspace_bytes(T, nq, nkv, d))
    dod = to_dev(d_o.reshape(T, -1))
    ob.ob_varlen_attn_bwd(dod, qd, kd, vd, o, lse, dqkv[:, :nq * d], dqkv[:, nq * d:(nq + nkv) * d],
                          dqkv[:, (nq + nkv) * d:], Dq, Dq, nq * d, seg, nq, nkv, d, scale, mask, ws)
    g = to_np(dqkv)
    assert np.isfinite(g).all()
    assert rel_err(g[:, :nq * d].reshape(T, nq, d), dq_ref) < TOL
    assert rel_err(g[:, nq * d:(nq + nkv) * d].reshape(T, nkv, d), dk_ref) < TOL
    assert rel_err(g[:, (nq + nkv) * d:].reshape(T, nkv, d), dv_ref) < TOL
    # bitwise reproducible (no atomics anywhere)
    dqkv2 = torch.empty_like(dqkv)
    ob.ob_varlen_attn_bwd(dod, qd, kd, vd, o, lse, dqkv2[:, :nq * d], dqkv2[:, nq * d:(nq + nkv) * d],
                          dqkv2[:, (nq + nkv) * d:], Dq, Dq, nq * d, seg, nq, nkv, d, scale, mask, ws)
    assert torch.equal(dqkv.view(torch.int16), dqkv2.view(torch.int16))


@pytest.mark.parametrize("mask", [orc.MASK_BIDIR, orc.MASK_CAUSAL])
def test_mask_and_offsets_bit_exact(mask):
    lens = si.tiny_segment_lengths(seed=0)
    cu = si.lengths_to_cu(lens)
    T = int(cu[-1])
    seg = ob.Segments(cu)
    out = torch.empty((T, T), dtype=torch.uint8, device="cuda")
    ob.ob_debug_materialize_mask(seg, mask, out)
    assert np.array_equal(out.cpu().numpy().astype(bool), orc.allowed_mask(cu, T, mask))
    # offsets produced by the library's builders equal the oracle's, bit for bit
    tiles, tok = si.synthetic_dataset(500, 0)
    groups, _, _ = ob.ob_pack_isf(tiles, tok, 10 ** 9, 16384, 10 ** 9, 16384 - 128, 10, 0)
    P, _, _ = orc_pack.isf(tiles, tok, 10 ** 9, 16384, 10 ** 9, 16384 - 128, 10, 0)
    for g, G in zip(groups[:5], P[:5]):
        assert ob.ob_build_cu_seqlens_llm(g, tok)[0].tolist() == orc_pack.cu_seqlens_llm(G, tok)


# ---- whole block ----------------------------------------------------------------------------

def _check_block(shape, cu, seed, intermediates=True, dtype=None, tol=TOL):
    dtype = dtype or torch.bfloat16
    T = int(cu[-1])
    w = si.block_weights(shape, seed=seed)
    x, dy = si.activations(T, shape.hidden, seed=seed)
    y_ref, cache = orc.block_fwd(shape, w, x, cu)
    dx_ref, g_ref, _ = orc.block_bwd(shape, w, cache, dy, cu)
    run, y, dx, g = run_block(shape, w, x, dy, cu, dtype)
    errs = {"y": rel_err(y, y_ref), "dx": rel_err(dx, dx_ref)}
    for n in g_ref:
        errs["d" + n] = rel_err(g[n], g_ref[n])
    if intermediates:
        nq, nkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
        qkv_ref = np.concatenate([cache["q"].reshape(T, -1), cache["k"].reshape(T, -1),
                                  cache["v"].reshape(T, -1)], axis=1)
        views = {"h1": (cache["h1"], (T, shape.hidden)), "qkv": (qkv_ref, (T, shape.d_qkv)),
                 "o": (cache["o"].reshape(T, -1), (T, nq * d)), "x1": (cache["x1"], (T, shape.hidden)),
                 "h2": (cache["h2"], (T, shape.hidden)), "up": (cache["up"], (T, shape.up_rows)),
                 "act": (cache["act"], (T, shape.mlp_dim))}
        for n, (ref, shp) in views.items():
            errs["saved." + n] = rel_err(to_np(saved_view(run.desc, T, run.saved, n, shp, dtype)), ref)
    _say("  " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    assert set(g_ref) == set(w)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad
    return run


def test_block_config1_fwd_bwd():
    shape = si.CONFIGS[1]
    cu = si.lengths_to_cu(si.tiny_segment_lengths(seed=0))
    _say(f"block config 1: T={int(cu[-1])} lens={np.diff(cu).tolist()}")
    _check_block(shape, cu, seed=0)


@pytest.mark.parametrize("variant", ["llm-like", "llm-many-segments", "vit-like", "vit-d128-rms", "vit-h768-long",
                                     "llm-h640-long"])
def test_block_small_variants(variant):
    if variant == "llm-many-segments":
        # more segments than a wavefront has lanes (the rotary kernel's segment lookup and the attention
        # kernels' tile lookup walk them in rounds), many of them shorter than a tile, token count odd
        shape = si.small_shape(hidden=256, n_q_heads=4, n_kv_heads=1, head_dim=64, mlp_dim=256,
                               norm=si.NORM_RMSNORM, mlp=si.MLP_SWIGLU, mask=si.MASK_CAUSAL,
                               use_rotary=True, has_bias=False, norm_eps=1e-6)
        lens = [1 + (7 * i) % 13 for i in range(150)] + [131, 2]
    elif variant == "llm-like":
        shape = si.small_shape(hidden=512, n_q_heads=4, n_kv_heads=2, head_dim=128, mlp_dim=320,
                               norm=si.NORM_RMSNORM, mlp=si.MLP_SWIGLU, mask=si.MASK_CAUSAL,
                               use_rotary=True, has_bias=False, norm_eps=1e-6)
        lens = [300, 1, 140, 259]
    elif variant == "vit-h768-long":
        # >= 2048 tokens of <= 1024 elements: the norm backward with eight row-walking waves per workgroup
        # whose column sums (norm parameters, and two bias gradients beside them) are folded in LDS; 96
        # 16-byte pieces per row, so the lanes' second piece exists only for half of them; tokens odd
        shape = si.small_shape(hidden=768, n_q_heads=12, n_kv_heads=12, head_dim=64, mlp_dim=512,
                               norm=si.NORM_LAYERNORM, mlp=si.MLP_GELU, mask=si.MASK_BIDIR,
                               use_rotary=False, has_bias=True)
        lens = [1025, 1025, 13]
    elif variant == "llm-h640-long":
        # the same path without biases (no sums beside the norm parameters') and with RMSNorm
        shape = si.small_shape(hidden=640, n_q_heads=5, n_kv_heads=5, head_dim=128, mlp_dim=384,
                               norm=si.NORM_RMSNORM, mlp=si.MLP_SWIGLU, mask=si.MASK_CAUSAL,
                               use_rotary=True, has_bias=False, norm_eps=1e-6)
        lens = [700, 1, 900, 448]
    elif variant == "vit-like":
        shape = si.small_shape(hidden=192, n_q_heads=3, n_kv_heads=3, head_dim=64, mlp_dim=768,
                               norm=si.NORM_LAYERNORM, mlp=si.MLP_GELU, mask=si.MASK_BIDIR,
                               use_rotary=False, has_bias=True)
        lens = [257, 257, 257]
    else:
        shape = si.small_shape(hidden=384, n_q_heads=3, n_kv_heads=3, head_dim=128, mlp_dim=1536,
                               norm=si.NORM_RMSNORM, mlp=si.MLP_GELU, mask=si.MASK_BIDIR,
                               use_rotary=False, has_bias=False, norm_eps=1e-6)
        lens = [1025, 130]
    _say(f"block {variant}: lens={lens}")
    _check_block(shape, si.lengths_to_cu(lens), seed=3)


@pytest.mark.parametrize("dtype_name", ["bf16", "fp32"])
def test_block_random_compositions(dtype_name):
    """Ten seeded blocks: every combination the descriptor allows is drawn from (norm, MLP, mask,
    rotary, biases, GQA group, head size, hidden sizes that are and are not multiples of 256); once on
    the bf16 path and once on the fp32 debug path at its own bar."""
    rng = np.random.default_rng(31)
    fp32 = dtype_name == "fp32"
    for case in range(10):
        d = int(rng.choice([64, 128]))
        nkv = int(rng.integers(1, 3))
        nq = nkv * int(rng.choice([1, 2, 4]))
        norm = si.NORM_LAYERNORM if rng.random() < 0.5 else si.NORM_RMSNORM
        shape = si.small_shape(hidden=64 * int(rng.integers(1, 13)), n_q_heads=nq, n_kv_heads=nkv, head_dim=d,
                               mlp_dim=64 * int(rng.integers(1, 17)), norm=norm,
                               mlp=si.MLP_GELU if rng.random() < 0.5 else si.MLP_SWIGLU,
                               mask=si.MASK_CAUSAL if rng.random() < 0.5 else si.MASK_BIDIR,
                               use_rotary=bool(rng.random() < 0.5), has_bias=bool(rng.random() < 0.5),
                               norm_eps=1e-5 if norm == si.NORM_LAYERNORM else 1e-6)
        lens = [int(rng.integers(1, 400)) for _ in range(int(rng.integers(1, 7)))]
        _say(f"block random {case}: hidden={shape.hidden} nq={nq} nkv={nkv} d={d} mlp={shape.mlp_dim} "
             f"norm={shape.norm} act={shape.mlp} mask={shape.mask} rotary={shape.use_rotary} bias={shape.has_bias} lens={lens}")
        _check_block(shape, si.lengths_to_cu(lens), seed=40 + case, dtype=torch.float32 if fp32 else None,
                     tol=TOL_FP32 if fp32 else TOL)


# ---- re-computation (Sec. 4.3): backward replays the forward into a scratch `saved` -----------

@pytest.mark.parametrize("variant", ["config1", "llm-like"])
def test_block_bwd_with_recompute_is_bit_identical(variant):
    if variant == "config1":
        shape, lens = si.CONFIGS[1], si.tiny_segment_lengths(seed=0)
    else:
        shape = si.small_shape(hidden=512, n_q_heads=4, n_kv_heads=2, head_dim=128, mlp_dim=320,
                               norm=si.NORM_RMSNORM, mlp=si.MLP_SWIGLU, mask=si.MASK_CAUSAL,
                               use_rotary=True, has_bias=False, norm_eps=1e-6)
        lens = [300, 1, 140, 259]
    cu = si.lengths_to_cu(lens)
    T = int(cu[-1])
    _say(f"recompute {variant}: T={T}")
    w = si.block_weights(shape, seed=1)
    x_np, dy_np = si.activations(T, shape.hidden, seed=1)
    seg = ob.Segments(cu)
    run = BlockRun(shape, w, T)
    x, dy = to_dev(x_np), to_dev(dy_np)
    run.fwd(x, seg)
    dx_ref = run.bwd(x, dy, seg)
    g_ref = {n: t.clone() for n, t in run.g.items()}
    # poison the saved buffer (as if another block had used it), then let the backward replay
    run.saved.fill_(0xFF)
    for t in run.g.values():
        t.zero_()
    dx = torch.empty_like(x)
    ob.ob_block_bwd(run.desc, run.w, run.g, ob.OB_BWD_RECOMPUTE, x, dy, dx, run.saved, seg, run.ws)
    torch.cuda.synchronize()
    assert torch.equal(dx.view(torch.int16), dx_ref.view(torch.int16))
    for n in g_ref:
        assert torch.equal(run.g[n].view(torch.int16), g_ref[n].view(torch.int16)), n
    # and it still matches the oracle
    y_ref, cache = orc.block_fwd(shape, w, x_np, cu)
    dx_o, _, _ = orc.block_bwd(shape, w, cache, dy_np, cu)
    assert rel_err(to_np(dx), dx_o) < TOL


# ---- fp32 debug path: same entry points, dtype = OB_FP32, tolerance 1e-4 ----------------------

@pytest.mark.parametrize("lens,nq,nkv,d,mask", ATTN_CASES[:3] + [([257, 130], 3, 3, 128, orc.MASK_BIDIR)])
def test_fp32_debug_attention(lens, nq, nkv, d, mask):
    _say(f"fp32 attention lens={lens} nq={nq} nkv={nkv} d={d} mask={mask}")
    cu = si.lengths_to_cu(lens)
    T = int(cu[-1])
    q, k, v, d_o = si.qkv_tensors(T, nq, nkv, d, seed=len(lens) + d)
    scale = 1.0 / np.sqrt(d)
    o_ref, lse_ref = orc.attention_fwd(*(a.astype(np.float64) for a in (q, k, v)), cu, mask, scale)
    dq_ref, dk_ref, dv_ref = orc.attention_bwd(*(a.astype(np.float64) for a in (d_o, q, k, v)),
                                               cu, mask, scale)
    f32 = torch.float32
    qd, kd, vd = (to_dev(a.reshape(T, -1), f32) for a in (q, k, v))
    o = torch.empty((T, nq * d), dtype=f32, device="cuda")
    lse = torch.empty((nq, T), dtype=f32, device="cuda")
    seg = ob.Segments(cu)
    ob.ob_varlen_attn_fwd(qd, kd, vd, o, lse, nq * d, nkv * d, nq * d, seg, nq, nkv, d, scale, mask,
                          dtype=ob.OB_FP32)
    assert rel_err(to_np(o).reshape(T, nq, d), o_ref) < TOL_FP32
    assert np.abs(to_np(lse) - lse_ref).max() < 1e-4
    dq, dk, dv = (torch.full_like(t, float("nan")) for t in (qd, kd, vd))
    ws = bytes_buf(ob.ob_varlen_attn_bwd_workspace_bytes(T, nq, nkv, d))
    ob.ob_varlen_attn_bwd(to_dev(d_o.reshape(T, -1), f32), qd, kd, vd, o, lse, dq, dk, dv, nq * d, nkv * d,
                          nq * d, seg, nq, nkv, d, scale, mask, ws, dtype=ob.OB_FP32)
    assert rel_err(to_np(dq).reshape(T, nq, d), dq_ref) < TOL_FP32
    assert rel_err(to_np(dk).reshape(T, nkv, d), dk_ref) < TOL_FP32
    assert rel_err(to_np(dv).reshape(T, nkv, d), dv_ref) < TOL_FP32


@pytest.mark.parametrize("variant", ["config1", "llm-like", "vit-d128-rms"])
def test_fp32_debug_block(variant):
    if variant == "config1":
        shape, lens = si.CONFIGS[1], si.tiny_segment_lengths(seed=0)
    elif variant == "llm-like":
        shape = si.small_shape(hidden=512, n_q_heads=4, n_kv_heads=2, head_dim=128, mlp_dim=320,
                               norm=si.NORM_RMSNORM, mlp=si.MLP_SWIGLU, mask=si.MASK_CAUSAL,
                               use_rotary=True, has_bias=False, norm_eps=1e-6)
        lens = [300, 1, 140, 259]
    else:
        shape = si.small_shape(hidden=384, n_q_heads=3, n_kv_heads=3, head_dim=128, mlp_dim=1536,
                               norm=si.NORM_RMSNORM, mlp=si.MLP_GELU, mask=si.MASK_BIDIR,
                               use_rotary=False, has_bias=False, norm_eps=1e-6)
        lens = [513, 130]
    _say(f"fp32 block {variant}: lens={list(lens)}")
    _check_block(shape, si.lengths_to_cu(lens), seed=3, dtype=torch.float32, tol=TOL_FP32)


def _subset_cu(cfg, max_tokens, seed=0):
    """Whole segments of one balanced mini-batch of `cfg`, up to about max_tokens tokens."""
    shape = si.CONFIGS[cfg]
    tiles, tok = si.synthetic_dataset(20000, seed)
    if shape.kind == "vit":
        n = max(1, max_tokens // si.VIT_TILE_TOKENS)
        return ob.ob_build_cu_seqlens_vit(n, si.VIT_TILE_TOKENS)
    groups, _, _ = ob.ob_pack_isf(tiles, tok, 10 ** 9, shape.budget, 10 ** 9, shape.budget - 128, 10, seed)
    cu, _ = ob.ob_build_cu_seqlens_llm(groups[0], tok)
    n = max(1, int(np.searchsorted(cu, max_tokens, side="right")) - 1)
    return cu[:n + 1].copy()


@pytest.mark.parametrize("cfg,max_tokens", [(2, 2100), (3, 2048), (4, 2100), (5, 1600), (2, 12300)])
def test_block_full_hidden_sizes_on_a_segment_subset(cfg, max_tokens):
    """Configs 2-5 at their full hidden sizes, one block, whole segments of a balanced batch; the last
    case is config 2's whole batch of 12 tiles, the launch configuration the bench times (weight
    gradients with split contractions, the column reductions of four biases and two norms)."""
    shape = si.CONFIGS[cfg]
    cu = _subset_cu(cfg, max_tokens)
    _say(f"block config {cfg} ({shape.name}): T={int(cu[-1])} n_seg={len(cu) - 1}")
    _check_block(shape, cu, seed=cfg, intermediates=False)


def test_block_is_bitwise_reproducible_and_accumulates():
    shape = si.CONFIGS[1]
    cu = si.lengths_to_cu([200, 333, 90])
    T = int(cu[-1])
    w = si.block_weights(shape, seed=9)
    x_np, dy_np = si.activations(T, shape.hidden, seed=9)
    seg = ob.Segments(cu)
    run = BlockRun(shape, w, T)
    x, dy = to_dev(x_np), to_dev(dy_np)
    y1 = run.fwd(x, seg).clone()
    dx1 = run.bwd(x, dy, seg).clone()
    g1 = {n: t.clone() for n, t in run.g.items()}
    y2 = run.fwd(x, seg)
    dx2 = run.bwd(x, dy, seg, accumulate=True)       # grads now hold g + g
    torch.cuda.synchronize()
    assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))
    assert torch.equal(dx1.view(torch.int16), dx2.view(torch.int16))
    for n in g1:
        assert torch.equal((2 * g1[n].float()).to(torch.bfloat16).view(torch.int16),
                           run.g[n].view(torch.int16)), n


def test_grouped_weight_gradients_of_a_narrow_block():
    """The 300M-class ViT block over its full batch of 12 tiles: its four weight gradients are less than a
    round of tiles each and go out as ONE grouped launch (9 GEMM launches per forward + backward instead of
    12).  Gradients against the oracle (in test_block_full_hidden_sizes_on_a_segment_subset); here: the
    launch count, bitwise reproducibility, and the accumulate flag through the grouped path."""
    shape = si.CONFIGS[2]
    cu = ob.ob_build_cu_seqlens_vit(shape.budget, si.VIT_TILE_TOKENS)
    T = int(cu[-1])
    w = si.block_weights(shape, seed=2)
    x_np, dy_np = si.activations(T, shape.hidden, seed=2)
    seg = ob.Segments(cu)
    run = BlockRun(shape, w, T)
    x, dy = to_dev(x_np), to_dev(dy_np)
    ob.ob_prof_begin(1000)
    run.fwd(x, seg)
    dx1 = run.bwd(x, dy, seg).clone()
    torch.cuda.synchronize()
    prof = ob.ob_prof_end()
    _say(f"grouped wgrad: gemm launches per fwd+bwd = {prof['gemm'][1]}")
    assert prof["gemm"][1] == 9
    g1 = {n: t.clone() for n, t in run.g.items()}
    dx2 = run.bwd(x, dy, seg, accumulate=True)
    torch.cuda.synchronize()
    assert torch.equal(dx1.view(torch.int16), dx2.view(torch.int16))
    for n in g1:
        assert torch.equal((2 * g1[n].float()).to(torch.bfloat16).view(torch.int16), run.g[n].view(torch.int16)), n


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_full_batch_one_segment_against_oracle(cfg):
    """The launch configurations the bench times (config 3: one full balanced 16K-token batch;
    config 4: 16 tiles; config 5: 32K tokens): the packed result restricted to one segment must equal
    the oracle run on that segment alone, and with dy zero outside the segment the weight gradients
    must equal the segment's own."""
    shape = si.CONFIGS[cfg]
    if shape.kind == "vit":
        cu = ob.ob_build_cu_seqlens_vit(shape.budget, si.VIT_TILE_TOKENS)
        j = shape.budget // 2 - 1
    else:
        tiles, tok = si.synthetic_dataset(20000, 0)
        groups, _, _ = ob.ob_pack_isf(tiles, tok, 10 ** 9, shape.budget, 10 ** 9, shape.budget - 128, 10, 0)
        cu, mx = ob.ob_build_cu_seqlens_llm(groups[0], tok)
        j = int(np.argmin(np.abs(np.diff(cu) - 700)))     # a mid-sized sample, not tile aligned
    T = int(cu[-1])
    lens = np.diff(cu)
    a, b = int(cu[j]), int(cu[j + 1])
    _say(f"config {cfg} full batch: T={T} n_seg={len(lens)} checking segment {j} [{a},{b})")
    w = si.block_weights(shape, seed=3)
    x, dy = si.activations(T, shape.hidden, seed=3)
    dy_masked = np.zeros_like(dy)
    dy_masked[a:b] = dy[a:b]
    run, y, dx, g = run_block(shape, w, x, dy_masked, cu)
    y_ref, cache = orc.block_fwd(shape, w, x[a:b], [0, b - a])
    dx_ref, g_ref, _ = orc.block_bwd(shape, w, cache, dy[a:b], [0, b - a])
    errs = {"y": rel_err(y[a:b], y_ref), "dx": rel_err(dx[a:b], dx_ref)}
    for n in g_ref:
        errs["d" + n] = rel_err(g[n], g_ref[n])
    _say("  " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    assert max(errs.values()) <= TOL, errs
    outside = np.ones(T, bool)
    outside[a:b] = False
    assert np.abs(dx[outside]).max() == 0.0


def _bench_batch_cu(cfg, batch=0, seed=0):
    """Segment offsets of balanced mini-batch `batch` of config `cfg`, built the way bench.py builds them."""
    shape = si.CONFIGS[cfg]
    if shape.kind == "vit":
        return ob.ob_build_cu_seqlens_vit(shape.budget, si.VIT_TILE_TOKENS)
    tiles, tok = si.synthetic_dataset(20000, seed)
    groups, _, _ = ob.ob_pack_isf(tiles, tok, 10 ** 9, shape.budget, 10 ** 9, shape.budget - 128, 10, seed)
    return ob.ob_build_cu_seqlens_llm(groups[batch], tok)[0]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_full_batch_every_row_and_gradient_against_oracle(cfg):
    """The launch configurations the bench times, compared whole: one full balanced batch (config 3:
    16K tokens, config 4: 16 tiles, config 5: 32K tokens), real dy on every row; every row of y and dx
    and every weight gradient against the oracle.  The oracle runs segment by segment (a packed batch
    is its segments run alone: pinned on the CPU) and its weight gradients are summed over the
    segments.  Config 5's oracle runs in fp32 (77 TFLOP of host work; fp32 and fp64 oracle agree to
    1e-5, pinned on the CPU), the others in fp64."""
    shape = si.CONFIGS[cfg]
    cu = _bench_batch_cu(cfg)
    T, lens = int(cu[-1]), np.diff(cu)
    odt = np.float32 if cfg == 5 else np.float64
    _say(f"config {cfg} whole batch: T={T} n_seg={len(lens)} lens={lens.tolist()} oracle dtype={odt.__name__}")
    w = si.block_weights(shape, seed=5)
    x, dy = si.activations(T, shape.hidden, seed=5)
    run, y, dx, g = run_block(shape, w, x, dy, cu)
    _say("  HIP path done; oracle, segment by segment:")
    w_o = {n: a.astype(odt) for n, a in w.items()}            # cast once, not per segment
    y_ref, dx_ref = np.empty((T, shape.hidden), odt), np.empty((T, shape.hidden), odt)
    g_ref = None
    for j in range(len(lens)):
        a, b = int(cu[j]), int(cu[j + 1])
        yj, cache = orc.block_fwd(shape, w_o, x[a:b], [0, b - a], dtype=odt)
        dxj, gj, _ = orc.block_bwd(shape, w_o, cache, dy[a:b], [0, b - a], dtype=odt)
        y_ref[a:b], dx_ref[a:b] = yj, dxj
        if g_ref is None:
            g_ref = {n: v.astype(np.float64) for n, v in gj.items()}
        else:
            for n, v in gj.items():
                g_ref[n] += v
        _say(f"    segment {j} [{a},{b}) done")
    errs = {"y": rel_err(y, y_ref), "dx": rel_err(dx, dx_ref)}
    for n in g_ref:
        errs["d" + n] = rel_err(g[n], g_ref[n])
    _say("  " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    assert set(g_ref) == set(w)
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, bad
    # no row may hide behind the largest one: every segment's rows on their own scale too
    for j in range(len(lens)):
        a, b = int(cu[j]), int(cu[j + 1])
        assert rel_err(y[a:b], y_ref[a:b]) <= TOL and rel_err(dx[a:b], dx_ref[a:b]) <= TOL, j


@pytest.mark.parametrize("variant", ["llm-like", "vit-like"])
def test_block_stack_of_three_against_oracle(variant):
    """Three blocks of one kind chained forward and then backward, as the bench chains them (each
    block with its own weights, `saved` and gradient buffers; activations handed from block to block,
    gradients alternating between two buffers), against the oracle's stack: y of the last block, dx of
    the first, and every block's weight gradients."""
    if variant == "llm-like":
        shape = si.small_shape(hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=64, mlp_dim=704,
                               norm=si.NORM_RMSNORM, mlp=si.MLP_SWIGLU, mask=si.MASK_CAUSAL,
                               use_rotary=True, has_bias=False, norm_eps=1e-6)
        lens = [300, 1, 140, 259, 77]
    else:
        shape = si.small_shape(hidden=384, n_q_heads=6, n_kv_heads=6, head_dim=64, mlp_dim=1536,
                               norm=si.NORM_LAYERNORM, mlp=si.MLP_GELU, mask=si.MASK_BIDIR,
                               use_rotary=False, has_bias=True)
        lens = [257, 257, 257]
    cu = si.lengths_to_cu(lens)
    T, L = int(cu[-1]), 3
    _say(f"stack {variant}: L={L} T={T} lens={lens}")
    ws = [si.block_weights(shape, seed=21, block=i) for i in range(L)]
    # activations of unit scale so that the three residual branches matter against the input
    x_np, dy_np = si.activations(T, shape.hidden, seed=21, std=1.0)
    y_ref, dx_ref, g_ref = orc.stack_fwd_bwd(shape, ws, x_np, dy_np, cu)

    seg = ob.Segments(cu)
    runs = [BlockRun(shape, w, T) for w in ws]
    acts = [to_dev(x_np)]
    for r in runs:
        acts.append(r.fwd(acts[-1], seg))
    gbuf = [torch.empty_like(acts[0]) for _ in range(2)]
    g_in = to_dev(dy_np)
    for i in reversed(range(L)):
        g_out = gbuf[i & 1]
        ob.ob_block_bwd(runs[i].desc, runs[i].w, runs[i].g, 0, acts[i], g_in, g_out, runs[i].saved, seg, runs[i].ws)
        g_in = g_out
    torch.cuda.synchronize()
    errs = {"y": rel_err(to_np(acts[-1]), y_ref), "dx": rel_err(to_np(g_in), dx_ref)}
    for i in range(L):
        assert set(g_ref[i]) == set(ws[i])
        for n in g_ref[i]:
            errs[f"block{i}.d{n}"] = rel_err(to_np(runs[i].g[n]), g_ref[i][n])
    _say("  " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, bad


@pytest.mark.timeout(600)
@pytest.mark.parametrize("cfg", [3, 5])
def test_attention_alone_at_full_size_on_the_bench_batch(cfg):
    """Varlen attention forward and backward alone at the full token count and head counts of the LLM
    configurations (32 / 8 and 48 / 8 heads of 128, causal), on the segment layout of the bench's first
    balanced batch; every segment, every head, against the oracle."""
    shape = si.CONFIGS[cfg]
    cu = _bench_batch_cu(cfg)
    _check_attention(np.diff(cu).tolist(), shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.mask, seed=cfg,
                     per_segment=True)


@pytest.mark.parametrize("d,mask", [(64, orc.MASK_BIDIR), (64, orc.MASK_CAUSAL), (128, orc.MASK_BIDIR),
                                    (128, orc.MASK_CAUSAL)])
def test_attention_packed_equals_each_segment_alone_bit_for_bit(d, mask):
    """What "samples stay whole" means for the kernels (Sec. 3, Sec. 4.1): tiles are aligned to segments,
    so running the packed batch and running every segment as a batch of its own must give the same
    bits, for o, lse, dq, dk and dv, for both masks and both head sizes.  This pins the masking of the
    product kernels themselves at bit level."""
    lens = [130, 1, 64, 257, 63, 200, 1025]
    nq, nkv = 4, 2
    cu = si.lengths_to_cu(lens)
    T = int(cu[-1])
    _say(f"packed vs alone d={d} mask={mask} lens={lens}")
    q, k, v, d_o = si.qkv_tensors(T, nq, nkv, d, seed=d + mask)
    scale = 1.0 / np.sqrt(d)
    qd, kd, vd, dod = (to_dev(a.reshape(T, -1)) for a in (q, k, v, d_o))

    def run(qs, ks, vs, dos, cu_):
        t = qs.shape[0]
        seg = ob.Segments(cu_)
        o = torch.empty((t, nq * d), dtype=torch.bfloat16, device="cuda")
        lse = torch.empty((nq, t), dtype=torch.float32, device="cuda")
        ob.ob_varlen_attn_fwd(qs, ks, vs, o, lse, nq * d, nkv * d, nq * d, seg, nq, nkv, d, scale, mask)
        dq, dk, dv = torch.empty_like(qs), torch.empty_like(ks), torch.empty_like(vs)
        ws = bytes_buf(ob.ob_varlen_attn_bwd_workspace_bytes(t, nq, nkv, d))
        ob.ob_varlen_attn_bwd(dos, qs, ks, vs, o, lse, dq, dk, dv, nq * d, nkv * d, nq * d, seg, nq, nkv, d,
                              scale, mask, ws)
        torch.cuda.synchronize()
        return o, lse, dq, dk, dv

    o, lse, dq, dk, dv = run(qd, kd, vd, dod, cu)
    for j in range(len(lens)):
        a, b = int(cu[j]), int(cu[j + 1])
        oj, lsej, dqj, dkj, dvj = run(qd[a:b], kd[a:b], vd[a:b], dod[a:b], np.array([0, b - a], dtype=np.int32))
        for name, whole, alone in (("o", o[a:b], oj), ("dq", dq[a:b], dqj), ("dk", dk[a:b], dkj), ("dv", dv[a:b], dvj)):
            assert torch.equal(whole.view(torch.int16), alone.view(torch.int16)), (name, j)
        assert torch.equal(lse[:, a:b].contiguous().view(torch.int32), lsej.view(torch.int32)), ("lse", j)


@pytest.mark.parametrize("n_seg", [257, 300, 520, 600])
def test_attention_with_hundreds_of_segments(n_seg):
    """More segments than one round of the kernels' in-workgroup segment scan covers (256), and more
    than two rounds: segments of 1-70 tokens, against the oracle."""
    rng = np.random.default_rng(n_seg)
    lens = rng.integers(1, 71, n_seg).tolist()
    _check_attention(lens, 4, 2, 64 if n_seg % 2 else 128, orc.MASK_CAUSAL if n_seg % 3 else orc.MASK_BIDIR, seed=n_seg)


def test_block_with_hundreds_of_segments():
    """The block's segment lookups (rotary positions, attention tiles) past 256 and past 512 segments."""
    shape = si.small_shape(hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, mlp_dim=256,
                           norm=si.NORM_RMSNORM, mlp=si.MLP_SWIGLU, mask=si.MASK_CAUSAL,
                           use_rotary=True, has_bias=False, norm_eps=1e-6)
    rng = np.random.default_rng(9)
    lens = rng.integers(1, 40, 530).tolist()
    _say(f"block with {len(lens)} segments, T={sum(lens)}")
    _check_block(shape, si.lengths_to_cu(lens), seed=8)


# ---- ViT -> LLM hand-over: sub-sampling + connector ---------------------------------------------

CONNECTOR_CASES = [
    # Hv, Ht, grid, tiles per sample, text tokens per sample
    (128, 256, 8, [2, 1], [5, 0]),
    (1024, 4096, 32, [1, 1], [37, 300]),       # the 300M-class encoder into the 7B-class decoder
    (3200, 6144, 32, [1], [129]),              # the 6B-class encoder into the 20B-class decoder
]


@pytest.mark.parametrize("Hv,Ht,grid,tiles,text", CONNECTOR_CASES)
def test_connector_fwd_bwd(Hv, Ht, grid, tiles, text):
    from oracle import connector as orc_conn
    _say(f"connector Hv={Hv} Ht={Ht} grid={grid} tiles={tiles} text={text}")
    n_tiles, per_tile = sum(tiles), grid * grid // 4
    w_np = si.connector_weights(Hv, Ht, seed=Hv + Ht)
    dst, cu = si.visual_rows(tiles, text, tokens_per_tile=per_tile)
    T = int(cu[-1])
    v_np, _ = si.activations(n_tiles * (grid * grid + 1), Hv, seed=1, std=1.0)
    x_np, dx_np = si.activations(T, Ht, seed=2, std=1.0)
    eps = 1e-5

    ref_out, cache = orc_conn.connector_fwd(w_np, v_np, n_tiles, grid, eps, x_np, dst)
    ref_dv, ref_g = orc_conn.connector_bwd(w_np, cache, dx_np, n_tiles, grid, eps, dst)

    desc = ob.make_connector_desc(Hv, Ht, grid, eps)
    w = {n: to_dev(a) for n, a in w_np.items()}
    g = {n: torch.zeros_like(t) for n, t in w.items()}
    saved = bytes_buf(ob.ob_connector_saved_bytes(desc, n_tiles))
    ws = bytes_buf(ob.ob_connector_workspace_bytes(desc, n_tiles))
    rows = ob.RowIndex(dst)
    v, x_llm, dx_llm = to_dev(v_np), to_dev(x_np), to_dev(dx_np)
    dv = torch.full((n_tiles * (grid * grid + 1), Hv), 7.0, dtype=torch.bfloat16, device="cuda")
    ob.ob_connector_fwd(desc, w, v, n_tiles, rows, x_llm, T, saved, ws)
    ob.ob_connector_bwd(desc, w, g, 0, v, dx_llm, dv, n_tiles, rows, T, saved, ws)
    torch.cuda.synchronize()

    out = to_np(x_llm)
    text_rows = np.setdiff1d(np.arange(T), dst)
    np.testing.assert_array_equal(out[text_rows], x_np[text_rows].astype(np.float64))   # untouched, bit for bit
    assert rel_err(out[dst], ref_out[dst]) < TOL
    dv_np = to_np(dv)
    cls = np.arange(n_tiles) * (grid * grid + 1)
    assert not dv_np[cls].any()                                                         # class rows: exact zeros
    assert rel_err(dv_np, ref_dv) < TOL
    for n in si.CONNECTOR_NAMES:
        assert rel_err(to_np(g[n]), ref_g[n]) < TOL, n

    # a second backward with the accumulate flag doubles every weight gradient (up to bf16 rounding)
    first = {n: to_np(t) for n, t in g.items()}
    ob.ob_connector_bwd(desc, w, g, ob.OB_BWD_ACCUMULATE, v, dx_llm, dv, n_tiles, rows, T, saved, ws)
    torch.cuda.synchronize()
    for n in si.CONNECTOR_NAMES:
        assert rel_err(to_np(g[n]), 2 * first[n]) < 1e-2, n


@pytest.mark.parametrize("Hv,Ht,grid,tiles,text", CONNECTOR_CASES[:2])
def test_fp32_debug_connector(Hv, Ht, grid, tiles, text):
    """The hand-over with every tensor in fp32: composition, gather / scatter and the analytic backward
    against the fp64 oracle at the tolerance bf16 storage cannot reach."""
    from oracle import connector as orc_conn
    _say(f"fp32 connector Hv={Hv} Ht={Ht} grid={grid} tiles={tiles} text={text}")
    n_tiles, per_tile = sum(tiles), grid * grid // 4
    w_np = si.connector_weights(Hv, Ht, seed=Hv + Ht)
    dst, cu = si.visual_rows(tiles, text, tokens_per_tile=per_tile)
    T = int(cu[-1])
    v_np, _ = si.activations(n_tiles * (grid * grid + 1), Hv, seed=1, std=1.0)
    x_np, dx_np = si.activations(T, Ht, seed=2, std=1.0)
    eps = 1e-5
    ref_out, cache = orc_conn.connector_fwd(w_np, v_np, n_tiles, grid, eps, x_np, dst)
    ref_dv, ref_g = orc_conn.connector_bwd(w_np, cache, dx_np, n_tiles, grid, eps, dst)

    f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    desc = ob.make_connector_desc(Hv, Ht, grid, eps, dtype=ob.OB_FP32)
    w = {n: f32(a) for n, a in w_np.items()}
    g = {n: torch.zeros_like(t) for n, t in w.items()}
    saved = bytes_buf(ob.ob_connector_saved_bytes(desc, n_tiles))
    ws = bytes_buf(ob.ob_connector_workspace_bytes(desc, n_tiles))
    rows = ob.RowIndex(dst)
    v, x_llm, dx_llm = f32(v_np), f32(x_np), f32(dx_np)
    dv = torch.full((n_tiles * (grid * grid + 1), Hv), 7.0, dtype=torch.float32, device="cuda")
    ob.ob_connector_fwd(desc, w, v, n_tiles, rows, x_llm, T, saved, ws)
    ob.ob_connector_bwd(desc, w, g, 0, v, dx_llm, dv, n_tiles, rows, T, saved, ws)
    torch.cuda.synchronize()
    out = x_llm.cpu().numpy().astype(np.float64)
    text_rows = np.setdiff1d(np.arange(T), dst)
    np.testing.assert_array_equal(out[text_rows], x_np[text_rows].astype(np.float32).astype(np.float64))
    assert rel_err(out[dst], ref_out[dst]) < TOL_FP32
    dv_np = dv.cpu().numpy().astype(np.float64)
    assert not dv_np[np.arange(n_tiles) * (grid * grid + 1)].any()
    assert rel_err(dv_np, ref_dv) < TOL_FP32
    for n in si.CONNECTOR_NAMES:
        assert rel_err(g[n].cpu().numpy(), ref_g[n]) < TOL_FP32, n


def test_mixed_stage_chain_vit_block_handover_llm_block():
    """One ViT block -> sub-sampling + connector -> one LLM block on one mini-batch, forward and backward,
    against the oracle's chain: checks that the entry points compose (row layouts, the visual rows of
    the packed LLM batch, the gradient handed from the LLM input back to the ViT output)."""
    from oracle import connector as orc_conn
    grid, tiles, text = 8, [2, 1, 1], [9, 40, 3]
    vs = si.small_shape(name="vit", hidden=128, n_q_heads=2, n_kv_heads=2, mlp_dim=256, mask=si.MASK_BIDIR)
    ts = si.small_shape(name="llm", hidden=256, n_q_heads=4, n_kv_heads=2, mlp_dim=512, norm=si.NORM_RMSNORM,
                        mlp=si.MLP_SWIGLU, mask=si.MASK_CAUSAL, use_rotary=True, has_bias=False, norm_eps=1e-6)
    n_tiles, per_tile, eps = sum(tiles), grid * grid // 4, 1e-5
    cu_v = orc_pack.cu_seqlens_vit(n_tiles, grid * grid + 1)
    dst, cu_t = si.visual_rows(tiles, text, tokens_per_tile=per_tile)
    Tv, Tt = int(cu_v[-1]), int(cu_t[-1])
    _say(f"mixed chain: {n_tiles} tiles, Tv={Tv}, Tt={Tt}")
    wv, wt, wc = si.block_weights(vs, seed=11), si.block_weights(ts, seed=12), si.connector_weights(vs.hidden, ts.hidden, seed=13)
    xv, _ = si.activations(Tv, vs.hidden, seed=14, std=1.0)
    x_text, dy = si.activations(Tt, ts.hidden, seed=15, std=1.0)

    # oracle chain
    yv_ref, cv = orc.block_fwd(vs, wv, xv, cu_v)
    xt_ref, cc = orc_conn.connector_fwd(wc, yv_ref, n_tiles, grid, eps, x_text, dst)
    yt_ref, ct = orc.block_fwd(ts, wt, xt_ref, cu_t)
    dxt_ref, gt_ref, _ = orc.block_bwd(ts, wt, ct, dy, cu_t)
    dyv_ref, gc_ref = orc_conn.connector_bwd(wc, cc, dxt_ref, n_tiles, grid, eps, dst)
    dxv_ref, gv_ref, _ = orc.block_bwd(vs, wv, cv, dyv_ref, cu_v)

    # HIP chain
    seg_v, seg_t, rows = ob.Segments(cu_v), ob.Segments(cu_t), ob.RowIndex(dst)
    rv, rt = BlockRun(vs, wv, Tv), BlockRun(ts, wt, Tt)
    cdesc = ob.make_connector_desc(vs.hidden, ts.hidden, grid, eps)
    cw = {n: to_dev(a) for n, a in wc.items()}
    cg = {n: torch.zeros_like(t) for n, t in cw.items()}
    csaved = bytes_buf(ob.ob_connector_saved_bytes(cdesc, n_tiles))
    cws = bytes_buf(ob.ob_connector_workspace_bytes(cdesc, n_tiles))
    x_v, x_t, dy_t = to_dev(xv), to_dev(x_text), to_dev(dy)
    y_v = rv.fwd(x_v, seg_v)
    ob.ob_connector_fwd(cdesc, cw, y_v, n_tiles, rows, x_t, Tt, csaved, cws)
    y_t = rt.fwd(x_t, seg_t)
    dx_t = rt.bwd(x_t, dy_t, seg_t)
    dy_v = torch.empty_like(y_v)
    ob.ob_connector_bwd(cdesc, cw, cg, 0, y_v, dx_t, dy_v, n_tiles, rows, Tt, csaved, cws)
    dx_v = rv.bwd(x_v, dy_v, seg_v)
    torch.cuda.synchronize()

    errs = {"y_llm": rel_err(to_np(y_t), yt_ref), "dx_llm": rel_err(to_np(dx_t), dxt_ref),
            "dy_vit": rel_err(to_np(dy_v), dyv_ref), "dx_vit": rel_err(to_np(dx_v), dxv_ref)}
    errs.update({"vit.d" + n: rel_err(to_np(rv.g[n]), gv_ref[n]) for n in gv_ref})
    errs.update({"conn.d" + n: rel_err(to_np(cg[n]), gc_ref[n]) for n in gc_ref})
    errs.update({"llm.d" + n: rel_err(to_np(rt.g[n]), gt_ref[n]) for n in gt_ref})
    _say("  " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, bad
