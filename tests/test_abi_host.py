"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and rejects bad
arguments with the documented codes before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2605_15422_amd", "libdualkv.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libdualkv.so not built")


def _declared():
    src = open(os.path.join(ROOT, "include", "dualkv.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dualkv_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    lib = C.CDLL(LIB)
    names = _declared()
    assert {"dualkv_ctx_fwd", "dualkv_ctx_bwd", "dualkv_fwd", "dualkv_bwd"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    from paper_2605_15422_amd import binding
    assert sorted(binding.EXPORTS) == names
    assert binding.dualkv_version() >= 100
    assert binding.dualkv_strerror(0) == "ok"


def test_argument_validation_before_launch():
    from paper_2605_15422_amd import binding as B
    ok = dict(n_seqs=2, ctx_len=8, total_resp=6, max_resp=4, n_q_heads=4, n_kv_heads=2, head_dim=64)

    def ws(**kw):
        out = C.c_size_t(0)
        s = B.make_shape(**{**ok, **kw})
        return B.lib.dualkv_workspace_bytes(C.byref(s), B.OP_BWD, C.byref(out)), out.value

    assert ws()[0] == B.OK and ws()[1] >= 6 * 4 * 4
    assert ws(n_q_heads=5)[0] == B.E_INVALID            # H % H_k != 0
    assert ws(head_dim=80)[0] == B.E_UNSUPPORTED
    assert ws(head_dim=512, window=16)[0] == B.E_UNSUPPORTED
    assert ws(n_seqs=0)[0] == B.E_INVALID
    assert ws(ctx_len=-1)[0] == B.E_INVALID
    assert ws(max_resp=7)[0] == B.E_INVALID
    # head dims 64 / 128: the two (H, rows) fp32 statistics arrays of the backward must lie within 4 GB
    big = dict(total_resp=1 << 25, max_resp=1 << 25, n_q_heads=32, n_kv_heads=8)
    assert ws(**big)[0] == B.E_UNSUPPORTED
    assert ws(**big, head_dim=256)[0] == B.OK
    assert ws(**{**big, "total_resp": (1 << 25) - 64, "max_resp": 1 << 20})[0] == B.OK
    s = B.make_shape(**ok)
    assert B.lib.dualkv_workspace_bytes(C.byref(s), 9, C.byref(C.c_size_t())) == B.E_INVALID
    assert B.lib.dualkv_workspace_bytes(None, B.OP_BWD, C.byref(C.c_size_t())) == B.E_INVALID

    # entry points: NULL tensors, misalignment, bad host cu_seqlens -- all rejected on the host
    null = B.TIn(None, 0, 0)
    nullo = B.TOut(None, 0, 0)
    rc = B.lib.dualkv_fwd(C.byref(s), null, null, null, null, null, None, None, nullo, None, None, 0, None)
    assert rc == B.E_INVALID
    import numpy as np
    bad_cu = np.array([0, 5, 3], dtype=np.int32)        # not monotone
    rc = B.lib.dualkv_fwd(C.byref(s), null, null, null, null, null, None, bad_cu.ctypes.data_as(C.c_void_p), nullo,
                          None, None, 0, None)
    assert rc == B.E_INVALID
    bad_cu = np.array([0, 1, 5], dtype=np.int32)        # last != total_resp
    rc = B.lib.dualkv_fwd(C.byref(s), null, null, null, null, null, None, bad_cu.ctypes.data_as(C.c_void_p), nullo,
                          None, None, 0, None)
    assert rc == B.E_INVALID
    fake = B.TIn(0x1008, 256, 64)                        # 8-byte aligned only
    rc = B.lib.dualkv_ctx_fwd(C.byref(s), fake, fake, fake, B.TOut(0x1000, 256, 64), None, None, 0, None)
    assert rc == B.E_ALIGN
    fake = B.TIn(0x1000, 252, 64)                        # stride not a multiple of 8
    rc = B.lib.dualkv_ctx_fwd(C.byref(s), fake, fake, fake, B.TOut(0x1000, 256, 64), None, None, 0, None)
    assert rc == B.E_ALIGN
    fake = B.TIn(0x1000, (1 << 22) + 8, 64)              # token stride beyond the 32-bit row offsets of the kernels
    rc = B.lib.dualkv_ctx_fwd(C.byref(s), fake, fake, fake, B.TOut(0x1000, 256, 64), None, None, 0, None)
    assert rc == B.E_UNSUPPORTED
    good = B.TIn(0x1000, 256, 64)
    goodo = B.TOut(0x1000, 256, 64)
    rc = B.lib.dualkv_ctx_bwd(C.byref(s), good, good, C.c_void_p(0x1000), good, good, good, goodo, goodo, goodo,
                              None, None, None, 0, None)
    assert rc == B.E_WORKSPACE                           # workspace missing
    assert B.lib.dualkv_repack(1, 4, 4, None, 6, None, None, None, None) == B.E_ALIGN
    assert B.lib.dualkv_repack(0, 4, 4, None, 8, None, None, None, None) == B.E_INVALID
    assert "workspace" in B.dualkv_strerror(B.E_WORKSPACE)
    # the allocation-free backward rejects shapes beyond its static scratch before it touches the device
    big = B.make_shape(1, 0, 200000, 200000, 32, 8, 128)
    assert B.dualkv_workspace_bytes(big, B.OP_BWD) > B.STATIC_SCRATCH_BYTES
    rc = B.lib.dualkv_bwd_noalloc(C.byref(big), null, null, None, null, null, null, null, null, None, None,
                                  nullo, nullo, nullo, nullo, nullo, None, None, None)
    assert rc == B.E_SCRATCH and "static scratch" in B.dualkv_strerror(B.E_SCRATCH)
    hdr = open(os.path.join(ROOT, "include", "dualkv.h")).read()
    assert "#define DUALKV_STATIC_SCRATCH_BYTES (32u << 20)" in hdr and B.STATIC_SCRATCH_BYTES == 32 << 20
