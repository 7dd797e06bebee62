"""ctypes binding of libdualkv.so: argument marshalling only.

Every function has the name and argument order of its C entry point
(include/dualkv.h).  Tensors are torch CUDA tensors used purely as device
buffers: the binding reads ``data_ptr()`` and strides and passes the current
torch stream.  Nothing is computed here; if the library is missing, importing
this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdualkv.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libdualkv.so not found at %s -- build it first: python -m paper_2605_15422_amd.build" % LIB_PATH)

lib = C.CDLL(LIB_PATH)

OK, E_INVALID, E_UNSUPPORTED, E_WORKSPACE, E_ALIGN, E_HIP, E_SCRATCH = 0, -1, -2, -3, -4, -5, -6
STATIC_SCRATCH_BYTES = 32 << 20
OP_CTX_FWD, OP_CTX_BWD, OP_FWD, OP_BWD = 0, 1, 2, 3
FLAG_ACCUM_CTX_F32 = 1
FLAG_SKIP_DQ = 2
FLAG_SKIP_DKDV = 4
FLAG_SKIP_PRE = 8

EXPORTS = ["dualkv_workspace_bytes", "dualkv_ctx_fwd", "dualkv_ctx_bwd", "dualkv_fwd", "dualkv_bwd",
           "dualkv_bwd_noalloc", "dualkv_zero_ctx_grads", "dualkv_groups_workspace_bytes", "dualkv_ctx_fwd_groups",
           "dualkv_fwd_groups", "dualkv_ctx_bwd_groups", "dualkv_bwd_groups",
           "dualkv_finalize_ctx_grads", "dualkv_repack", "dualkv_replicate", "dualkv_label_map",
           "dualkv_strerror", "dualkv_version"]


class Shape(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("ctx_len", C.c_int32), ("total_resp", C.c_int32),
                ("max_resp", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("window", C.c_int32), ("softmax_scale", C.c_float),
                ("flags", C.c_uint32)]


class TIn(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("tok_stride", C.c_int64), ("head_stride", C.c_int64)]


class TOut(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("tok_stride", C.c_int64), ("head_stride", C.c_int64)]


class Group(C.Structure):
    _fields_ = [("ctx_offset", C.c_int32), ("ctx_len", C.c_int32), ("seq_begin", C.c_int32), ("seq_end", C.c_int32)]


_PS = C.POINTER(Shape)
lib.dualkv_version.restype = C.c_int
lib.dualkv_strerror.restype = C.c_char_p
lib.dualkv_strerror.argtypes = [C.c_int]
lib.dualkv_workspace_bytes.argtypes = [_PS, C.c_int, C.POINTER(C.c_size_t)]
lib.dualkv_ctx_fwd.argtypes = [_PS, TIn, TIn, TIn, TOut, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
lib.dualkv_ctx_bwd.argtypes = [_PS, TIn, TIn, C.c_void_p, TIn, TIn, TIn, TOut, TOut, TOut,
                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
lib.dualkv_fwd.argtypes = [_PS, TIn, TIn, TIn, TIn, TIn, C.c_void_p, C.c_void_p, TOut, C.c_void_p,
                           C.c_void_p, C.c_size_t, C.c_void_p]
lib.dualkv_bwd.argtypes = [_PS, TIn, TIn, C.c_void_p, TIn, TIn, TIn, TIn, TIn, C.c_void_p, C.c_void_p,
                           TOut, TOut, TOut, TOut, TOut, C.c_void_p, C.c_void_p,
                           C.c_void_p, C.c_size_t, C.c_void_p]
lib.dualkv_bwd_noalloc.argtypes = [_PS, TIn, TIn, C.c_void_p, TIn, TIn, TIn, TIn, TIn, C.c_void_p, C.c_void_p,
                                   TOut, TOut, TOut, TOut, TOut, C.c_void_p, C.c_void_p, C.c_void_p]
_GRP = [_PS, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32]
lib.dualkv_groups_workspace_bytes.argtypes = [_PS, C.c_int32, C.c_int32, C.c_int, C.POINTER(C.c_size_t)]
lib.dualkv_ctx_fwd_groups.argtypes = _GRP + lib.dualkv_ctx_fwd.argtypes[1:]
lib.dualkv_fwd_groups.argtypes = _GRP + lib.dualkv_fwd.argtypes[1:]
lib.dualkv_ctx_bwd_groups.argtypes = _GRP + lib.dualkv_ctx_bwd.argtypes[1:]
lib.dualkv_bwd_groups.argtypes = _GRP + lib.dualkv_bwd.argtypes[1:]
lib.dualkv_zero_ctx_grads.argtypes = [_PS, C.c_void_p, C.c_void_p, C.c_void_p]
lib.dualkv_finalize_ctx_grads.argtypes = [_PS, C.c_void_p, C.c_void_p, TOut, TOut, C.c_void_p]
for _f in (lib.dualkv_repack, lib.dualkv_replicate):
    _f.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                   C.c_void_p, C.c_void_p]
lib.dualkv_label_map.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
for _n in EXPORTS:
    if _n not in ("dualkv_strerror",):
        getattr(lib, _n).restype = C.c_int


class DualKVError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %d (%s)" % (where, code, lib.dualkv_strerror(code).decode()))


def _check(rc: int, where: str) -> None:
    if rc != OK:
        raise DualKVError(rc, where)


def make_shape(n_seqs, ctx_len, total_resp, max_resp, n_q_heads, n_kv_heads, head_dim, window=0,
               softmax_scale=0.0, flags=0) -> Shape:
    return Shape(int(n_seqs), int(ctx_len), int(total_resp), int(max_resp), int(n_q_heads), int(n_kv_heads),
                 int(head_dim), int(window), float(softmax_scale), int(flags))


def _tin(t) -> TIn:
    """(rows, heads, d) bf16 tensor view -> pointer + element strides (None -> NULL)."""
    if t is None:
        return TIn(None, 0, 0)
    assert t.dtype == torch.bfloat16 and t.dim() == 3
    if t.numel() == 0:   # empty region (e.g. P = 0): NULL with the strides of a contiguous tensor
        return TIn(None, t.shape[1] * t.shape[2], t.shape[2])
    assert t.stride(2) == 1
    return TIn(t.data_ptr(), t.stride(0), t.stride(1))


def _tout(t) -> TOut:
    if t is None:
        return TOut(None, 0, 0)
    assert t.dtype == torch.bfloat16 and t.dim() == 3
    if t.numel() == 0:
        return TOut(None, t.shape[1] * t.shape[2], t.shape[2])
    assert t.stride(2) == 1
    return TOut(t.data_ptr(), t.stride(0), t.stride(1))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _host_i32(a):
    if a is None:
        return None
    import numpy as np
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a.ctypes.data_as(C.c_void_p), a


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(ws):
    if ws is None:
        return None, 0
    return C.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def dualkv_version() -> int:
    return lib.dualkv_version()


def dualkv_strerror(code: int) -> str:
    return lib.dualkv_strerror(code).decode()


def dualkv_workspace_bytes(shape: Shape, op: int) -> int:
    out = C.c_size_t(0)
    _check(lib.dualkv_workspace_bytes(C.byref(shape), op, C.byref(out)), "dualkv_workspace_bytes")
    return out.value


def dualkv_ctx_fwd(shape, q_c, k_c, v_c, o_c, lse_c, workspace=None):
    wp, wb = _ws(workspace)
    _check(lib.dualkv_ctx_fwd(C.byref(shape), _tin(q_c), _tin(k_c), _tin(v_c), _tout(o_c), _ptr(lse_c),
                              wp, wb, _stream()), "dualkv_ctx_fwd")


def dualkv_ctx_bwd(shape, do_c, o_c, lse_c, q_c, k_c, v_c, dq_c, dk_c, dv_c, dk_c_acc32=None,
                   dv_c_acc32=None, workspace=None):
    wp, wb = _ws(workspace)
    _check(lib.dualkv_ctx_bwd(C.byref(shape), _tin(do_c), _tin(o_c), _ptr(lse_c), _tin(q_c), _tin(k_c),
                              _tin(v_c), _tout(dq_c), _tout(dk_c), _tout(dv_c), _ptr(dk_c_acc32),
                              _ptr(dv_c_acc32), wp, wb, _stream()), "dualkv_ctx_bwd")


def dualkv_fwd(shape, q_d, k_c, v_c, k_d, v_d, cu_seqlens_dev, cu_seqlens_host, o_d, lse_d, workspace=None):
    wp, wb = _ws(workspace)
    h = _host_i32(cu_seqlens_host)
    _check(lib.dualkv_fwd(C.byref(shape), _tin(q_d), _tin(k_c), _tin(v_c), _tin(k_d), _tin(v_d),
                          _ptr(cu_seqlens_dev), h[0] if h else None, _tout(o_d), _ptr(lse_d), wp, wb,
                          _stream()), "dualkv_fwd")


def dualkv_bwd(shape, do_d, o_d, lse_d, q_d, k_c, v_c, k_d, v_d, cu_seqlens_dev, cu_seqlens_host,
               dq_d, dk_c, dv_c, dk_d, dv_d, dk_c_acc32=None, dv_c_acc32=None, workspace=None):
    wp, wb = _ws(workspace)
    h = _host_i32(cu_seqlens_host)
    _check(lib.dualkv_bwd(C.byref(shape), _tin(do_d), _tin(o_d), _ptr(lse_d), _tin(q_d), _tin(k_c), _tin(v_c),
                          _tin(k_d), _tin(v_d), _ptr(cu_seqlens_dev), h[0] if h else None,
                          _tout(dq_d), _tout(dk_c), _tout(dv_c), _tout(dk_d), _tout(dv_d),
                          _ptr(dk_c_acc32), _ptr(dv_c_acc32), wp, wb, _stream()), "dualkv_bwd")


def dualkv_bwd_noalloc(shape, do_d, o_d, lse_d, q_d, k_c, v_c, k_d, v_d, cu_seqlens_dev, cu_seqlens_host,
                       dq_d, dk_c, dv_c, dk_d, dv_d, dk_c_acc32=None, dv_c_acc32=None):
    h = _host_i32(cu_seqlens_host)
    _check(lib.dualkv_bwd_noalloc(C.byref(shape), _tin(do_d), _tin(o_d), _ptr(lse_d), _tin(q_d), _tin(k_c), _tin(v_c),
                                  _tin(k_d), _tin(v_d), _ptr(cu_seqlens_dev), h[0] if h else None,
                                  _tout(dq_d), _tout(dk_c), _tout(dv_c), _tout(dk_d), _tout(dv_d),
                                  _ptr(dk_c_acc32), _ptr(dv_c_acc32), _stream()), "dualkv_bwd_noalloc")


def _grp(groups_dev, groups_host):
    """(device int32 tensor (n, 4), optional host int32 array (n, 4)) -> the four leading group arguments."""
    import numpy as np
    n = int(groups_dev.shape[0])
    h = None
    if groups_host is not None:
        h = np.ascontiguousarray(groups_host, dtype=np.int32)
        assert h.shape == (n, 4)
    return n, _ptr(groups_dev), (h.ctypes.data_as(C.c_void_p) if h is not None else None), h


def dualkv_groups_workspace_bytes(shape: Shape, n_groups: int, total_ctx: int, op: int) -> int:
    out = C.c_size_t(0)
    _check(lib.dualkv_groups_workspace_bytes(C.byref(shape), n_groups, total_ctx, op, C.byref(out)),
           "dualkv_groups_workspace_bytes")
    return out.value


def dualkv_ctx_fwd_groups(shape, groups_dev, groups_host, total_ctx, q_c, k_c, v_c, o_c, lse_c, workspace=None):
    wp, wb = _ws(workspace)
    n, gd, gh, _keep = _grp(groups_dev, groups_host)
    _check(lib.dualkv_ctx_fwd_groups(C.byref(shape), n, gd, gh, total_ctx, _tin(q_c), _tin(k_c), _tin(v_c), _tout(o_c),
                                     _ptr(lse_c), wp, wb, _stream()), "dualkv_ctx_fwd_groups")


def dualkv_fwd_groups(shape, groups_dev, groups_host, total_ctx, q_d, k_c, v_c, k_d, v_d, cu_seqlens_dev,
                      cu_seqlens_host, o_d, lse_d, workspace=None):
    wp, wb = _ws(workspace)
    h = _host_i32(cu_seqlens_host)
    n, gd, gh, _keep = _grp(groups_dev, groups_host)
    _check(lib.dualkv_fwd_groups(C.byref(shape), n, gd, gh, total_ctx, _tin(q_d), _tin(k_c), _tin(v_c), _tin(k_d),
                                 _tin(v_d), _ptr(cu_seqlens_dev), h[0] if h else None, _tout(o_d), _ptr(lse_d), wp, wb,
                                 _stream()), "dualkv_fwd_groups")


def dualkv_ctx_bwd_groups(shape, groups_dev, groups_host, total_ctx, do_c, o_c, lse_c, q_c, k_c, v_c, dq_c, dk_c, dv_c,
                          dk_c_acc32=None, dv_c_acc32=None, workspace=None):
    wp, wb = _ws(workspace)
    n, gd, gh, _keep = _grp(groups_dev, groups_host)
    _check(lib.dualkv_ctx_bwd_groups(C.byref(shape), n, gd, gh, total_ctx, _tin(do_c), _tin(o_c), _ptr(lse_c),
                                     _tin(q_c), _tin(k_c), _tin(v_c), _tout(dq_c), _tout(dk_c), _tout(dv_c),
                                     _ptr(dk_c_acc32), _ptr(dv_c_acc32), wp, wb, _stream()), "dualkv_ctx_bwd_groups")


def dualkv_bwd_groups(shape, groups_dev, groups_host, total_ctx, do_d, o_d, lse_d, q_d, k_c, v_c, k_d, v_d,
                      cu_seqlens_dev, cu_seqlens_host, dq_d, dk_c, dv_c, dk_d, dv_d, dk_c_acc32=None, dv_c_acc32=None,
                      workspace=None):
    wp, wb = _ws(workspace)
    h = _host_i32(cu_seqlens_host)
    n, gd, gh, _keep = _grp(groups_dev, groups_host)
    _check(lib.dualkv_bwd_groups(C.byref(shape), n, gd, gh, total_ctx, _tin(do_d), _tin(o_d), _ptr(lse_d), _tin(q_d),
                                 _tin(k_c), _tin(v_c), _tin(k_d), _tin(v_d), _ptr(cu_seqlens_dev),
                                 h[0] if h else None, _tout(dq_d), _tout(dk_c), _tout(dv_c), _tout(dk_d), _tout(dv_d),
                                 _ptr(dk_c_acc32), _ptr(dv_c_acc32), wp, wb, _stream()), "dualkv_bwd_groups")


def dualkv_zero_ctx_grads(shape, dk_c_acc32, dv_c_acc32):
    _check(lib.dualkv_zero_ctx_grads(C.byref(shape), _ptr(dk_c_acc32), _ptr(dv_c_acc32), _stream()),
           "dualkv_zero_ctx_grads")


def dualkv_finalize_ctx_grads(shape, dk_c_acc32, dv_c_acc32, dk_c, dv_c):
    _check(lib.dualkv_finalize_ctx_grads(C.byref(shape), _ptr(dk_c_acc32), _ptr(dv_c_acc32), _tout(dk_c),
                                         _tout(dv_c), _stream()), "dualkv_finalize_ctx_grads")


def dualkv_repack(n_seqs, ctx_len, total_resp, cu_seqlens_dev, row_bytes, standard, packed, position_ids=None):
    _check(lib.dualkv_repack(n_seqs, ctx_len, total_resp, _ptr(cu_seqlens_dev), row_bytes, _ptr(standard),
                             _ptr(packed), _ptr(position_ids), _stream()), "dualkv_repack")


def dualkv_replicate(n_seqs, ctx_len, total_resp, cu_seqlens_dev, row_bytes, packed, standard, position_ids=None):
    _check(lib.dualkv_replicate(n_seqs, ctx_len, total_resp, _ptr(cu_seqlens_dev), row_bytes, _ptr(packed),
                                _ptr(standard), _ptr(position_ids), _stream()), "dualkv_replicate")


def dualkv_label_map(n_seqs, ctx_len, total_resp, cu_seqlens_dev, next_index=None, first_token_index=None):
    _check(lib.dualkv_label_map(n_seqs, ctx_len, total_resp, _ptr(cu_seqlens_dev), _ptr(next_index),
                                _ptr(first_token_index), _stream()), "dualkv_label_map")


# --------------------------------------------------------------------------
# buffer plumbing shared by tests / bench / smoke (allocation only, no math)
# --------------------------------------------------------------------------
def bf16_from_bits(bits, device="cuda"):
    """numpy uint16 bit patterns -> torch bf16 tensor on device (bit-exact)."""
    import numpy as np
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def bits_from_bf16(t):
    """torch bf16 tensor -> numpy uint16 bit patterns."""
    import numpy as np
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@dataclass
class DeviceGroup:
    """Device copies of one workload plus output buffers for all four entry points."""
    shape_c: Shape
    q_c: torch.Tensor
    k_c: torch.Tensor
    v_c: torch.Tensor
    q_d: torch.Tensor
    k_d: torch.Tensor
    v_d: torch.Tensor
    do_c: torch.Tensor
    do_d: torch.Tensor
    cu_dev: torch.Tensor
    cu_host: object


def upload(wl, flags=0, device="cuda") -> DeviceGroup:
    s = wl.shape
    shp = make_shape(s.n_seqs, s.ctx_len, wl.total_resp, wl.max_resp, s.n_q_heads, s.n_kv_heads, s.head_dim,
                     s.window, wl.scale, flags)
    return DeviceGroup(shp, *(bf16_from_bits(x, device) for x in
                              (wl.q_c, wl.k_c, wl.v_c, wl.q_d, wl.k_d, wl.v_d, wl.do_c, wl.do_d)),
                       torch.from_numpy(wl.cu_seqlens.copy()).to(device), wl.cu_seqlens.copy())


def workspace(shape: Shape, op: int, device="cuda"):
    n = dualkv_workspace_bytes(shape, op)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)
