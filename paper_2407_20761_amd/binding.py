"""ctypes binding of include/omnibal.h: same names, argument marshalling only.

Device tensors are torch tensors (PyTorch is used for device memory and streams only); their
data_ptr() is handed to the C ABI.  Host arrays are numpy.  No step of the method is computed
here, and there is no fallback path: a missing library is an ImportError.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
# PyTorch must be loaded BEFORE the library: the torch wheel ships its own HIP/HSA runtime
# (soname libamdhip64.so.7) and libomnibal.so binds to whichever libamdhip64.so.7 is already in
# the process.  Loading the library first would pull in a second runtime from /opt/rocm, and two
# HSA runtimes in one process cannot both own the device.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libomnibal.so")

OB_OK, OB_EINVAL, OB_ESEGMENTS, OB_EUNSUPPORTED, OB_EWORKSPACE, OB_EHIP = range(6)
OB_BF16, OB_FP32 = 0, 1
OB_BWD_ACCUMULATE, OB_BWD_RECOMPUTE = 1, 2
OB_MASK_SEG_BIDIR, OB_MASK_SEG_CAUSAL = 0, 1
OB_LAYERNORM, OB_RMSNORM = 0, 1
OB_GELU, OB_SWIGLU = 0, 1
GEMM_NT, GEMM_NN, GEMM_TN = 0, 1, 2

WEIGHT_FIELDS = ("n1_g", "n1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                 "n2_g", "n2_b", "w_up", "b_up", "w_down", "b_down")


class ob_block_desc(C.Structure):
    _fields_ = [("hidden", C.c_int), ("n_q_heads", C.c_int), ("n_kv_heads", C.c_int),
                ("head_dim", C.c_int), ("mlp_dim", C.c_int), ("norm", C.c_int), ("mlp", C.c_int),
                ("mask", C.c_int), ("dtype", C.c_int), ("use_rotary", C.c_int),
                ("rotary_base", C.c_float), ("norm_eps", C.c_float), ("has_bias", C.c_int)]


class ob_block_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class ob_block_grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class ob_segments(C.Structure):
    _fields_ = [("cu_host", C.POINTER(C.c_int32)), ("cu_dev", C.c_void_p), ("n_seg", C.c_int),
                ("total_tokens", C.c_int), ("max_seqlen", C.c_int)]


CONNECTOR_FIELDS = ("n_g", "n_b", "w1", "b1", "w2", "b2")


class ob_connector_desc(C.Structure):
    _fields_ = [("vit_hidden", C.c_int), ("llm_hidden", C.c_int), ("grid", C.c_int), ("dtype", C.c_int),
                ("norm_eps", C.c_float)]


class ob_connector_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in CONNECTOR_FIELDS]


class ob_connector_grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in CONNECTOR_FIELDS]


class OmnibalError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"omnibal status {status}: {text}")
        self.status = status


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2407_20761_amd.build` "
                      "(there is no fallback path)")
lib = C.CDLL(LIB_PATH)

_P, _I, _F, _Z = C.c_void_p, C.c_int, C.c_float, C.c_size_t
_SEG = C.POINTER(ob_segments)
_DESC = C.POINTER(ob_block_desc)
_i32p, _i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)

_SIGNATURES = {
    "ob_last_error": (C.c_char_p, []),
    "ob_has_device_code": (_I, []),
    "ob_prof_num_classes": (_I, []),
    "ob_prof_class_name": (C.c_char_p, [_I]),
    "ob_prof_begin": (_I, [_I]),
    "ob_prof_end": (_I, [C.POINTER(C.c_double), _i64p, C.POINTER(C.c_double), _I]),
    "ob_varlen_attn_fwd": (_I, [_P, _P, _P, _P, _P, _I, _I, _I, _SEG, _I, _I, _I, _F, _I, _I, _P]),
    "ob_varlen_attn_bwd_workspace_bytes": (_Z, [_I, _I, _I, _I]),
    "ob_varlen_attn_bwd": (_I, [_P] * 9 + [_I, _I, _I, _SEG, _I, _I, _I, _F, _I, _I, _P, _Z, _P]),
    "ob_varlen_attn_bwd_static": (_I, [_P] * 9 + [_I, _I, _I, _SEG, _I, _I, _I, _F, _I, _I, _P]),
    "ob_block_saved_bytes": (_Z, [_DESC, _I]),
    "ob_block_workspace_bytes": (_Z, [_DESC, _I]),
    "ob_block_saved_offset": (_Z, [_DESC, _I, C.c_char_p]),
    "ob_block_fwd": (_I, [_DESC, C.POINTER(ob_block_weights), _P, _P, _P, _Z, _SEG, _P, _Z, _P]),
    "ob_block_bwd": (_I, [_DESC, C.POINTER(ob_block_weights), C.POINTER(ob_block_grads), _I, _P, _P,
                          _P, _P, _Z, _SEG, _P, _Z, _P]),
    "ob_gemm_workspace_bytes": (_Z, [_I, _I, _I, _I]),
    "ob_gemm_bf16": (_I, [_I, _I, _I, _I, _P, _P, _P, _P, _P, _P, _Z, _P]),
    "ob_debug_materialize_mask": (_I, [_SEG, _I, _P, _P]),
    "ob_connector_saved_bytes": (_Z, [C.POINTER(ob_connector_desc), _I]),
    "ob_connector_workspace_bytes": (_Z, [C.POINTER(ob_connector_desc), _I]),
    "ob_connector_fwd": (_I, [C.POINTER(ob_connector_desc), C.POINTER(ob_connector_weights), _P, _I, _i32p, _P,
                              _P, _I, _P, _Z, _P, _Z, _P]),
    "ob_connector_bwd": (_I, [C.POINTER(ob_connector_desc), C.POINTER(ob_connector_weights),
                              C.POINTER(ob_connector_grads), _I, _P, _P, _P, _I, _i32p, _P, _I, _P, _Z, _P, _Z,
                              _P]),
    "ob_pack_isf": (_I, [_i32p, _i32p, C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_int64, _I,
                         C.c_uint64, _i64p, _i64p, _i64p, _i64p, _i64p, _i64p]),
    "ob_pack_random": (_I, [C.c_int64, C.c_int64, C.c_uint64, _i64p, _i64p, _i64p, _i64p, _i64p]),
    "ob_build_cu_seqlens_llm": (_I, [_i64p, C.c_int64, _i32p, _i32p, _i32p]),
    "ob_build_cu_seqlens_vit": (_I, [C.c_int64, C.c_int32, _i32p]),
    "ob_pack_length_group": (_I, [_i32p, C.c_int64, C.c_int64, C.c_uint64, _i64p, _i64p, _i64p, _i64p, _i64p]),
    "ob_pack_device_group": (_I, [_i32p, C.c_int64, C.c_int64, C.c_uint64, _i64p, _i64p, _i64p, _i64p, _i64p]),
    "ob_recompute_plan": (_I, [C.c_int64, _I, C.c_int64, C.c_double, _I, C.c_int64, C.c_double, _I,
                               C.POINTER(C.c_int), C.POINTER(C.c_int)]),
    "ob_bmp_anchor": (_I, [C.POINTER(C.c_double), _I, _I, C.POINTER(C.c_int)]),
    "ob_bmp_search": (_I, [C.POINTER(C.c_double), C.POINTER(C.c_double), _I, _I, _I, C.c_double, _I,
                           C.POINTER(C.c_int), C.POINTER(C.c_double), _i64p, C.POINTER(C.c_int)]),
    "ob_pad_ratio": (C.c_double, [_i64p, C.c_int64]),
    "ob_dist_ratio": (C.c_double, [_i64p, C.c_int64]),
}
EXPORTED = tuple(_SIGNATURES)
for _name, (_res, _args) in _SIGNATURES.items():
    _fn = getattr(lib, _name)
    _fn.restype, _fn.argtypes = _res, _args


def ob_last_error() -> str:
    return lib.ob_last_error().decode()


def _check(status: int):
    if status != OB_OK:
        raise OmnibalError(status, ob_last_error())


def _ptr(t):
    """device pointer of a torch tensor (None -> NULL)"""
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def ob_prof_begin(max_launches=65536):
    _check(lib.ob_prof_begin(int(max_launches)))


def ob_prof_end() -> dict:
    """{class name: (ms, launches, work)} for the classes that were launched"""
    n = lib.ob_prof_num_classes()
    ms, cnt, work = (C.c_double * n)(), (C.c_int64 * n)(), (C.c_double * n)()
    _check(lib.ob_prof_end(ms, cnt, work, n))
    return {lib.ob_prof_class_name(i).decode(): (ms[i], cnt[i], work[i]) for i in range(n) if cnt[i]}


class Segments:
    """Holds the host and device copies of cu_seqlens alive and exposes the C struct."""

    def __init__(self, cu_host, device="cuda", max_seqlen=None, cu_dev=None):
        self.cu_host = np.ascontiguousarray(cu_host, dtype=np.int32)
        self.cu_dev = (torch.from_numpy(self.cu_host).to(device) if cu_dev is None and device
                       else cu_dev)
        n = len(self.cu_host) - 1
        if max_seqlen is None:
            max_seqlen = int(np.diff(self.cu_host).max()) if n >= 1 else 0
        self.c = ob_segments(self.cu_host.ctypes.data_as(_i32p),
                             None if self.cu_dev is None else self.cu_dev.data_ptr(),
                             n, int(self.cu_host[-1]) if n >= 0 and len(self.cu_host) else 0,
                             int(max_seqlen))

    @property
    def total_tokens(self):
        return self.c.total_tokens


def make_desc(shape, dtype=OB_BF16) -> ob_block_desc:
    """ob_block_desc from any object with the BlockShape fields."""
    return ob_block_desc(shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                         shape.mlp_dim, int(shape.norm), int(shape.mlp), int(shape.mask), dtype,
                         int(bool(shape.use_rotary)), float(shape.rotary_base),
                         float(shape.norm_eps), int(bool(shape.has_bias)))


def _weights_struct(cls, tensors: dict):
    return cls(*[None if tensors.get(n) is None else tensors[n].data_ptr() for n in WEIGHT_FIELDS])


# ---- device entry points -------------------------------------------------------------------

def ob_varlen_attn_fwd(q, k, v, o, lse, ldq, ldkv, ldo, seg: Segments, nq, nkv, d, scale,
                       mask, dtype=OB_BF16, stream=None):
    _check(lib.ob_varlen_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), ldq, ldkv, ldo,
                                  C.byref(seg.c), nq, nkv, d, scale, mask, dtype, _stream(stream)))


def ob_varlen_attn_bwd_workspace_bytes(total_tokens, nq, nkv, d) -> int:
    return lib.ob_varlen_attn_bwd_workspace_bytes(total_tokens, nq, nkv, d)


def ob_varlen_attn_bwd(d_o, q, k, v, o, lse, dq, dk, dv, ldq, ldkv, ldo, seg: Segments, nq, nkv,
                       d, scale, mask, ws, dtype=OB_BF16, stream=None):
    _check(lib.ob_varlen_attn_bwd(_ptr(d_o), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                                  _ptr(dq), _ptr(dk), _ptr(dv), ldq, ldkv, ldo, C.byref(seg.c),
                                  nq, nkv, d, scale, mask, dtype, _ptr(ws),
                                  0 if ws is None else ws.numel() * ws.element_size(),
                                  _stream(stream)))


def ob_varlen_attn_bwd_static(d_o, q, k, v, o, lse, dq, dk, dv, ldq, ldkv, ldo, seg: Segments, nq, nkv,
                              d, scale, mask, dtype=OB_BF16, stream=None):
    _check(lib.ob_varlen_attn_bwd_static(_ptr(d_o), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                                         _ptr(dq), _ptr(dk), _ptr(dv), ldq, ldkv, ldo, C.byref(seg.c),
                                         nq, nkv, d, scale, mask, dtype, _stream(stream)))


def ob_block_saved_bytes(desc, total_tokens) -> int:
    return lib.ob_block_saved_bytes(C.byref(desc), total_tokens)


def ob_block_workspace_bytes(desc, total_tokens) -> int:
    return lib.ob_block_workspace_bytes(C.byref(desc), total_tokens)


def ob_block_saved_offset(desc, total_tokens, name: str) -> int:
    return lib.ob_block_saved_offset(C.byref(desc), total_tokens, name.encode())


def ob_block_fwd(desc, weights: dict, x, y, saved, seg: Segments, ws, stream=None):
    w = _weights_struct(ob_block_weights, weights)
    _check(lib.ob_block_fwd(C.byref(desc), C.byref(w), _ptr(x), _ptr(y), _ptr(saved),
                            saved.numel() * saved.element_size(), C.byref(seg.c), _ptr(ws),
                            ws.numel() * ws.element_size(), _stream(stream)))


def ob_block_bwd(desc, weights: dict, grads: dict, flags, x, dy, dx, saved,
                 seg: Segments, ws, stream=None):
    """flags: bit set of OB_BWD_ACCUMULATE / OB_BWD_RECOMPUTE (False / True = 0 / accumulate)"""
    w = _weights_struct(ob_block_weights, weights)
    g = _weights_struct(ob_block_grads, grads)
    _check(lib.ob_block_bwd(C.byref(desc), C.byref(w), C.byref(g), int(flags), _ptr(x),
                            _ptr(dy), _ptr(dx), _ptr(saved), saved.numel() * saved.element_size(),
                            C.byref(seg.c), _ptr(ws), ws.numel() * ws.element_size(),
                            _stream(stream)))


def ob_gemm_workspace_bytes(layout, M, N, K) -> int:
    return lib.ob_gemm_workspace_bytes(layout, M, N, K)


def ob_gemm_bf16(layout, M, N, K, A, B, Cout, bias=None, R=None, ws=None, stream=None):
    _check(lib.ob_gemm_bf16(layout, M, N, K, _ptr(A), _ptr(B), _ptr(Cout), _ptr(bias), _ptr(R),
                            _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                            _stream(stream)))


class RowIndex:
    """Host and device copies of an int32 row list (the visual rows of a packed LLM batch)."""

    def __init__(self, rows_host, device="cuda"):
        self.host = np.ascontiguousarray(rows_host, dtype=np.int32)
        self.dev = torch.from_numpy(self.host).to(device) if device else None

    @property
    def host_ptr(self):
        return self.host.ctypes.data_as(_i32p)


def make_connector_desc(vit_hidden, llm_hidden, grid=32, norm_eps=1e-5, dtype=OB_BF16) -> ob_connector_desc:
    return ob_connector_desc(int(vit_hidden), int(llm_hidden), int(grid), dtype, float(norm_eps))


def _connector_struct(cls, tensors: dict):
    return cls(*[None if tensors.get(n) is None else tensors[n].data_ptr() for n in CONNECTOR_FIELDS])


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def ob_connector_saved_bytes(desc, n_tiles) -> int:
    return lib.ob_connector_saved_bytes(C.byref(desc), n_tiles)


def ob_connector_workspace_bytes(desc, n_tiles) -> int:
    return lib.ob_connector_workspace_bytes(C.byref(desc), n_tiles)


def ob_connector_fwd(desc, weights: dict, v, n_tiles, dst_rows: RowIndex, x_llm, llm_tokens, saved, ws,
                     stream=None):
    w = _connector_struct(ob_connector_weights, weights)
    _check(lib.ob_connector_fwd(C.byref(desc), C.byref(w), _ptr(v), n_tiles, dst_rows.host_ptr,
                                _ptr(dst_rows.dev), _ptr(x_llm), llm_tokens, _ptr(saved), _nbytes(saved),
                                _ptr(ws), _nbytes(ws), _stream(stream)))


def ob_connector_bwd(desc, weights: dict, grads: dict, flags, v, dx_llm, dv, n_tiles, dst_rows: RowIndex,
                     llm_tokens, saved, ws, stream=None):
    w = _connector_struct(ob_connector_weights, weights)
    g = _connector_struct(ob_connector_grads, grads)
    _check(lib.ob_connector_bwd(C.byref(desc), C.byref(w), C.byref(g), int(flags), _ptr(v), _ptr(dx_llm),
                                _ptr(dv), n_tiles, dst_rows.host_ptr, _ptr(dst_rows.dev), llm_tokens,
                                _ptr(saved), _nbytes(saved), _ptr(ws), _nbytes(ws), _stream(stream)))


def ob_debug_materialize_mask(seg: Segments, mask, out, stream=None):
    _check(lib.ob_debug_materialize_mask(C.byref(seg.c), mask, _ptr(out), _stream(stream)))


# ---- host entry points ---------------------------------------------------------------------

def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def ob_pack_isf(n_img, n_tok, Qv, Qt, Qv_min, Qt_min, iters=10, seed=0):
    """returns (groups: list of int64 arrays, leftover ids, groups accepted per iteration)"""
    n_img = np.ascontiguousarray(n_img, dtype=np.int32)
    n_tok = np.ascontiguousarray(n_tok, dtype=np.int32)
    n = len(n_img)
    offs, ids, left = np.zeros(n + 1, np.int64), np.zeros(max(n, 1), np.int64), np.zeros(max(n, 1), np.int64)
    per_iter = np.zeros(max(iters, 1), np.int64)
    ng, nl = C.c_int64(0), C.c_int64(0)
    _check(lib.ob_pack_isf(n_img.ctypes.data_as(_i32p), n_tok.ctypes.data_as(_i32p), n, int(Qv),
                           int(Qt), int(Qv_min), int(Qt_min), int(iters), int(seed),
                           offs.ctypes.data_as(_i64p), C.byref(ng), ids.ctypes.data_as(_i64p),
                           left.ctypes.data_as(_i64p), C.byref(nl), per_iter.ctypes.data_as(_i64p)))
    groups = [ids[offs[g]:offs[g + 1]].copy() for g in range(ng.value)]
    return groups, left[:nl.value].copy(), per_iter[:iters].copy()


def ob_pack_random(n_samples, B, seed=0):
    n = int(n_samples)
    offs, ids, left = np.zeros(n + 1, np.int64), np.zeros(max(n, 1), np.int64), np.zeros(max(n, 1), np.int64)
    ng, nl = C.c_int64(0), C.c_int64(0)
    _check(lib.ob_pack_random(n, int(B), int(seed), offs.ctypes.data_as(_i64p), C.byref(ng),
                              ids.ctypes.data_as(_i64p), left.ctypes.data_as(_i64p), C.byref(nl)))
    groups = [ids[offs[g]:offs[g + 1]].copy() for g in range(ng.value)]
    return groups, left[:nl.value].copy()


def _pack_by_size(fn, n_tok, B, seed):
    n_tok = np.ascontiguousarray(n_tok, dtype=np.int32)
    n = len(n_tok)
    offs, ids, left = np.zeros(n + 1, np.int64), np.zeros(max(n, 1), np.int64), np.zeros(max(n, 1), np.int64)
    ng, nl = C.c_int64(0), C.c_int64(0)
    _check(fn(n_tok.ctypes.data_as(_i32p), n, int(B), int(seed), offs.ctypes.data_as(_i64p), C.byref(ng),
              ids.ctypes.data_as(_i64p), left.ctypes.data_as(_i64p), C.byref(nl)))
    return [ids[offs[g]:offs[g + 1]].copy() for g in range(ng.value)], left[:nl.value].copy()


def ob_pack_length_group(n_tok, B, seed=0):
    return _pack_by_size(lib.ob_pack_length_group, n_tok, B, seed)


def ob_pack_device_group(n_tok, B, seed=0):
    return _pack_by_size(lib.ob_pack_device_group, n_tok, B, seed)


def ob_recompute_plan(free_bytes, n_vit, bytes_vit, ms_vit, n_llm, bytes_llm, ms_llm, extra_recompute=0):
    kv, kt = C.c_int(0), C.c_int(0)
    _check(lib.ob_recompute_plan(int(free_bytes), int(n_vit), int(bytes_vit), float(ms_vit), int(n_llm),
                                 int(bytes_llm), float(ms_llm), int(extra_recompute), C.byref(kv), C.byref(kt)))
    return kv.value, kt.value


def _dbl(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def ob_bmp_anchor(fwd_ms, N):
    f = _dbl(fwd_ms)
    P = (C.c_int * max(int(N) - 1, 1))()
    _check(lib.ob_bmp_anchor(f.ctypes.data_as(C.POINTER(C.c_double)), len(f), int(N), P))
    return tuple(P[:int(N) - 1])


def ob_bmp_search(fwd_ms, activ, N, r, comm_weight=1.0, top_k=10):
    """([(score, P)] ascending, number of valid candidates)"""
    f, a = _dbl(fwd_ms), _dbl(activ)
    assert len(f) == len(a)
    c = int(N) - 1
    cand = (C.c_int * max(top_k * c, 1))()
    score = (C.c_double * top_k)()
    n_c, n_r = C.c_int64(0), C.c_int(0)
    _check(lib.ob_bmp_search(f.ctypes.data_as(C.POINTER(C.c_double)), a.ctypes.data_as(C.POINTER(C.c_double)),
                             len(f), int(N), int(r), float(comm_weight), int(top_k), cand, score,
                             C.byref(n_c), C.byref(n_r)))
    return [(score[k], tuple(cand[k * c:(k + 1) * c])) for k in range(n_r.value)], n_c.value


def ob_build_cu_seqlens_llm(group_ids, n_tok):
    group_ids = _i64(group_ids)
    n_tok = np.ascontiguousarray(n_tok, dtype=np.int32)
    cu = np.zeros(len(group_ids) + 1, np.int32)
    mx = C.c_int32(0)
    _check(lib.ob_build_cu_seqlens_llm(group_ids.ctypes.data_as(_i64p), len(group_ids),
                                       n_tok.ctypes.data_as(_i32p), cu.ctypes.data_as(_i32p),
                                       C.byref(mx)))
    return cu, mx.value


def ob_build_cu_seqlens_vit(n_tiles, tile_len):
    cu = np.zeros(int(n_tiles) + 1, np.int32)
    _check(lib.ob_build_cu_seqlens_vit(int(n_tiles), int(tile_len), cu.ctypes.data_as(_i32p)))
    return cu


def ob_pad_ratio(tokens_per_sample) -> float:
    a = _i64(tokens_per_sample)
    return lib.ob_pad_ratio(a.ctypes.data_as(_i64p), len(a))


def ob_dist_ratio(tokens_per_minibatch) -> float:
    a = _i64(tokens_per_minibatch)
    return lib.ob_dist_ratio(a.ctypes.data_as(_i64p), len(a))
