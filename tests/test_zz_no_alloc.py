"""The attention backward for callers that cannot allocate (ob_varlen_attn_bwd_static): through the C
ABI, against ob_varlen_attn_bwd with a caller-provided workspace, on two calls in a row, the second
with a smaller input (the static scratch keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import paper_2407_20761_amd as ob
import synth_inputs as si
from oracle import block as orc

pytestmark = pytest.mark.gpu
TOL = 2e-2


def _run_both(lens, nq, nkv, d, mask, seed):
    from conftest import rel_err
    from gpu_util import bytes_buf, to_dev, to_np
    cu = si.lengths_to_cu(lens)
    T = int(cu[-1])
    print(f"no-alloc attention bwd: lens={lens} nq={nq} nkv={nkv} d={d} mask={mask}", flush=True)
    q, k, v, d_o = si.qkv_tensors(T, nq, nkv, d, seed=seed)
    scale = 1.0 / np.sqrt(d)
    qd, kd, vd, dod = (to_dev(a.reshape(T, -1)) for a in (q, k, v, d_o))
    seg = ob.Segments(cu)
    o = torch.empty((T, nq * d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((nq, T), dtype=torch.float32, device="cuda")
    ob.ob_varlen_attn_fwd(qd, kd, vd, o, lse, nq * d, nkv * d, nq * d, seg, nq, nkv, d, scale, mask)
    ref = [torch.full_like(t, float("nan")) for t in (qd, kd, vd)]
    ws = bytes_buf(ob.ob_varlen_attn_bwd_workspace_bytes(T, nq, nkv, d))
    ob.ob_varlen_attn_bwd(dod, qd, kd, vd, o, lse, *ref, nq * d, nkv * d, nq * d, seg, nq, nkv, d, scale, mask, ws)
    got = [torch.full_like(t, float("nan")) for t in (qd, kd, vd)]
    before = torch.cuda.memory_allocated()
    ob.ob_varlen_attn_bwd_static(dod, qd, kd, vd, o, lse, *got, nq * d, nkv * d, nq * d, seg, nq, nkv, d, scale, mask)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for name, a, b in zip(("dq", "dk", "dv"), got, ref):
        assert torch.isfinite(a.float()).all(), name
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), name       # same kernels, same bits
    # and against the oracle, to the bar of every other parity test
    dq_ref, dk_ref, dv_ref = orc.attention_bwd(*(a.astype(np.float64) for a in (d_o, q, k, v)), cu, mask, scale)
    assert rel_err(to_np(got[0]).reshape(T, nq, d), dq_ref) < TOL
    assert rel_err(to_np(got[1]).reshape(T, nkv, d), dk_ref) < TOL
    assert rel_err(to_np(got[2]).reshape(T, nkv, d), dv_ref) < TOL


def test_static_scratch_attention_backward_two_calls_second_smaller():
    _run_both([300, 129, 1, 517], 8, 2, 128, orc.MASK_CAUSAL, seed=1)
    _run_both([65, 200], 4, 4, 64, orc.MASK_BIDIR, seed=2)          # smaller: fewer rows, fewer heads
    _run_both([65, 200], 4, 2, 64, orc.MASK_CAUSAL, seed=3)


def test_static_scratch_rejects_sizes_beyond_the_array():
    import ctypes as C
    T, nq = 1 << 20, 8                                               # 8 Mi rows x 8 bytes = 64 MiB > 32 MiB
    cu = np.array([0, T], dtype=np.int32)
    seg = ob.Segments(cu)
    p = C.c_void_p(0x1000)                                           # never dereferenced: refused on the host
    st = ob.lib.ob_varlen_attn_bwd_static(p, p, p, p, p, p, p, p, p, nq * 64, nq * 64, nq * 64, C.byref(seg.c),
                                          nq, nq, 64, 0.125, 1, 0, None)
    assert st == ob.OB_EWORKSPACE and "static" in ob.ob_last_error()
