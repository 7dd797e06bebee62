"""dualkv_bwd_noalloc (static scratch inside the library, no workspace argument, no allocation) against dualkv_bwd
on the same inputs, through the C ABI: two calls in a row, the second on a smaller group, so that what the first
call left in the shared scratch must not leak into the second.  Outputs that involve no atomics must be bit-equal;
the shared-prompt gradients of these small groups go through fp32 atomics (order-dependent sum) and are held to
the parity tolerance of the other GPU tests."""
import ctypes as C

import numpy as np
import pytest

from paper_2605_15422_amd import workloads as W

pytestmark = pytest.mark.gpu


def _layer(wl, flags=0):
    import torch
    from paper_2605_15422_amd import binding as B, runner
    dg = B.upload(wl, flags)
    b = runner.alloc(dg)
    runner.forward(dg, b)
    torch.cuda.synchronize()
    return dg, b


def _bwd(dg, b, flags, noalloc):
    """One Call-2 backward on the forward results in `b`: dualkv_bwd with a (poisoned) caller workspace, or
    dualkv_bwd_noalloc.  Not synchronised."""
    import torch
    from paper_2605_15422_amd import binding as B
    s = dg.shape_c
    acc = bool(flags & B.FLAG_ACCUM_CTX_F32)

    def like(t):
        x = torch.empty_like(t)
        x.view(torch.int16).fill_(0x7FC0)
        return x

    dq, dkd, dvd = like(dg.q_d), like(dg.k_d), like(dg.v_d)
    dkc, dvc = (None, None) if acc else (like(dg.k_c), like(dg.v_c))
    a_k = torch.zeros(dg.k_c.shape, dtype=torch.float32, device="cuda") if acc else None
    a_v = torch.zeros(dg.v_c.shape, dtype=torch.float32, device="cuda") if acc else None
    if noalloc:
        B.dualkv_bwd_noalloc(s, dg.do_d, b.o_d, b.lse_d, dg.q_d, dg.k_c, dg.v_c, dg.k_d, dg.v_d, dg.cu_dev,
                             dg.cu_host, dq, dkc, dvc, dkd, dvd, a_k, a_v)
    else:
        ws = B.workspace(s, B.OP_BWD)
        ws.fill_(0xFF)
        B.dualkv_bwd(s, dg.do_d, b.o_d, b.lse_d, dg.q_d, dg.k_c, dg.v_c, dg.k_d, dg.v_d, dg.cu_dev, dg.cu_host,
                     dq, dkc, dvc, dkd, dvd, a_k, a_v, ws)
    return dict(dq=dq, dkd=dkd, dvd=dvd, dkc=a_k if acc else dkc, dvc=a_v if acc else dvc)


def _check(name, ref, got):
    import torch
    for k in ("dq", "dkd", "dvd"):
        a, c = ref[k], got[k]
        assert torch.equal(a.view(torch.int16), c.view(torch.int16)), (name, k)
    for k in ("dkc", "dvc"):
        a, c = ref[k].float(), got[k].float()
        assert torch.isfinite(c).all(), (name, k)
        if a.numel() == 0:
            continue
        err = (a - c).abs()
        assert bool((err <= 2e-2 + 2.0 ** -8 * a.abs()).all()), (name, k, float(err.max()))
        assert float((a - c).norm()) <= 1e-2 * float(a.norm()) + 1e-6, (name, k)


@pytest.mark.parametrize("flags", [0, 1])
def test_noalloc_matches_workspace_call_twice_second_smaller(flags):
    cases = [
        ("first", W.Shape("na_first", 4, 517, 0, 0, 8, 2, 128, 0, seed=3301), [131, 70, 0, 200]),
        ("second_smaller", W.Shape("na_second", 2, 129, 0, 0, 4, 2, 128, 0, seed=3302), [33, 64]),
        ("third_d256_window", W.Shape("na_third", 3, 300, 0, 0, 4, 2, 256, 90, seed=3303), [100, 31, 65]),
    ]
    prepared = []
    for name, shape, lens in cases:
        print("case noalloc", name, flags, flush=True)
        wl = W.make_workload(shape, resp_lens=np.asarray(lens))
        prepared.append((name,) + _layer(wl, flags))
    import torch
    # reference results first (dualkv_bwd does not touch the static scratch) ...
    refs = [_bwd(dg, b, flags, noalloc=False) for _, dg, b in prepared]
    torch.cuda.synchronize()
    # ... then the allocation-free calls back to back on one stream: the larger group first, the smaller second
    for rnd in range(2):
        gots = [_bwd(dg, b, flags, noalloc=True) for _, dg, b in prepared]
        torch.cuda.synchronize()
        for (name, _, _), r, g in zip(prepared, refs, gots):
            _check("%s round %d" % (name, rnd), r, g)


def test_noalloc_inside_a_captured_graph():
    """The callers this entry point is for: the call is captured once in a HIP graph (after a first eager call has
    resolved the scratch address) and replayed; every replay, with eager work and new inputs in between, must equal
    the eager dualkv_bwd result on the same inputs."""
    import torch
    from paper_2605_15422_amd import binding as B
    print("case noalloc graph", flush=True)
    shape = W.Shape("na_graph", 3, 300, 0, 0, 8, 2, 128, 0, seed=3310)
    wl = W.make_workload(shape, resp_lens=np.asarray([90, 200, 33]))
    dg, b = _layer(wl, 0)
    s = dg.shape_c
    outs = {n: torch.empty_like(t) for n, t in (("dq", dg.q_d), ("dkc", dg.k_c), ("dvc", dg.v_c), ("dkd", dg.k_d),
                                                ("dvd", dg.v_d))}

    def call():
        B.dualkv_bwd_noalloc(s, dg.do_d, b.o_d, b.lse_d, dg.q_d, dg.k_c, dg.v_c, dg.k_d, dg.v_d, dg.cu_dev, None,
                             outs["dq"], outs["dkc"], outs["dvc"], outs["dkd"], outs["dvd"])

    call()                       # first use on this device: looks the scratch address up, outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(3):
        if rep:                  # new inputs in the same buffers
            dg.do_d.copy_(torch.roll(dg.do_d, rep, 0))
            dg.k_c.copy_(torch.roll(dg.k_c, rep, 0))
            from paper_2605_15422_amd import runner
            runner.forward(dg, b)
        ref = _bwd(dg, b, 0, noalloc=False)
        for t in outs.values():
            t.view(torch.int16).fill_(0x7FC0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _check("graph replay %d" % rep, ref, outs)


def test_noalloc_rejects_shapes_beyond_the_static_scratch():
    from paper_2605_15422_amd import binding as B
    # 2 x (rows x H x 4 B) > 32 MiB
    s = B.make_shape(1, 0, 200000, 200000, 32, 8, 128)
    assert B.dualkv_workspace_bytes(s, B.OP_BWD) > B.STATIC_SCRATCH_BYTES
    null, nullo = B.TIn(None, 0, 0), B.TOut(None, 0, 0)
    rc = B.lib.dualkv_bwd_noalloc(C.byref(s), null, null, None, null, null, null, null, null, None, None,
                                  nullo, nullo, nullo, nullo, nullo, None, None, None)
    assert rc == B.E_SCRATCH
    assert "static scratch" in B.dualkv_strerror(B.E_SCRATCH)
