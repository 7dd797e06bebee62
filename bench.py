#!/usr/bin/env python3
"""Benchmark of the shared-prompt attention hot path on one MI355X.

A step = one pass of the whole path over one synthetic group: Call 1 forward, Call 2 forward, clearing the fp32
accumulators of the shared-prompt gradients, Call 2 backward (D preprocess, dK/dV, dQ), Call 1 backward, both adding
their dK_c / dV_c terms into the fp32 accumulators, and the single cast of the Call-1 + Call-2 sum (Eq. 6, Alg. 2).
Inputs are resident in HBM before timing starts.  Prints ONE JSON line (metric, value = algorithmic TFLOP/s of the
whole layer, ms_per_step = ms/layer, the roofline of the dominant kernel, the other benchmark configs, the N-copy
reference point and the CPU-oracle baseline).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg2_qwen8b] [--no-ncopy] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16
HBM_PEAK_GBS = 8000.0
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.txt")


def measured_traffic(config, stage):
    """HBM bytes per launch (read + written) of one stage's kernel, from the tracked table of rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE results (already scaled by the copy-kernel calibration stated in that file); None if the
    table has no line for it."""
    try:
        with open(TRAFFIC_TABLE) as f:
            for ln in f:
                w = ln.split()
                if len(w) >= 3 and not ln.startswith("#") and w[0] == config and w[1] == stage:
                    return int(w[2])
    except OSError:
        pass
    return None


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


STAGES = ["ctx_fwd", "fwd", "zero_acc", "bwd_pre", "bwd_dkdv", "bwd_dq", "ctx_bwd_pre", "ctx_bwd_dkdv", "ctx_bwd_dq",
          "finalize"]


def time_layer(dg, bufs, steps, warmup):
    """Times `steps` layer passes; returns (ms_per_step, wall ms per step, per-stage average ms).

    The Call-2 / Call-1 backward is issued stage by stage (same kernels, same order as the plain call) so
    that HIP events on the launch stream bracket every kernel of the path.  With DUALKV_FLAG_ACCUM_CTX_F32 in the
    group's flags (the default of this benchmark) both backward calls add into the fp32 accumulators, which are
    cleared before and cast once after (Eq. 6); without it each call writes its own bf16 term and the two extra
    stages are empty.
    """
    import torch
    from paper_2605_15422_amd import binding as B

    s = dg.shape_c
    base = s.flags
    accum = bool(base & B.FLAG_ACCUM_CTX_F32)

    def shape_with(flags):
        c = type(s).from_buffer_copy(bytes(s))
        c.flags = base | flags
        return c

    s_pre = shape_with(B.FLAG_SKIP_DQ | B.FLAG_SKIP_DKDV)
    s_dkdv = shape_with(B.FLAG_SKIP_PRE | B.FLAG_SKIP_DQ)
    s_dq = shape_with(B.FLAG_SKIP_PRE | B.FLAG_SKIP_DKDV)
    dk2, dv2, dk1, dv1 = (None, None, None, None) if accum else (bufs.dk_c2, bufs.dv_c2, bufs.dk_c1, bufs.dv_c1)

    def bwd2(sh):
        B.dualkv_bwd(sh, dg.do_d, bufs.o_d, bufs.lse_d, dg.q_d, dg.k_c, dg.v_c, dg.k_d, dg.v_d, dg.cu_dev, None,
                     bufs.dq_d, dk2, dv2, bufs.dk_d, bufs.dv_d, bufs.dk_c_acc, bufs.dv_c_acc, bufs.ws_bwd)

    def bwd1(sh):
        B.dualkv_ctx_bwd(sh, dg.do_c, bufs.o_c, bufs.lse_c, dg.q_c, dg.k_c, dg.v_c, bufs.dq_c, dk1, dv1,
                         bufs.dk_c_acc, bufs.dv_c_acc, bufs.ws_ctx_bwd)

    def one_step(ev):
        k = 0
        ev[k].record(); k += 1
        if s.ctx_len > 0:
            B.dualkv_ctx_fwd(s, dg.q_c, dg.k_c, dg.v_c, bufs.o_c, bufs.lse_c)
        ev[k].record(); k += 1
        B.dualkv_fwd(s, dg.q_d, dg.k_c, dg.v_c, dg.k_d, dg.v_d, dg.cu_dev, None, bufs.o_d, bufs.lse_d)
        ev[k].record(); k += 1
        if accum:
            B.dualkv_zero_ctx_grads(s, bufs.dk_c_acc, bufs.dv_c_acc)
        ev[k].record(); k += 1
        for sh in (s_pre, s_dkdv, s_dq):
            bwd2(sh)
            ev[k].record(); k += 1
        for sh in (s_pre, s_dkdv, s_dq):
            if s.ctx_len > 0:
                bwd1(sh)
            ev[k].record(); k += 1
        if accum:
            B.dualkv_finalize_ctx_grads(s, bufs.dk_c_acc, bufs.dv_c_acc, bufs.dk_c, bufs.dv_c)
        ev[k].record(); k += 1

    nev = len(STAGES) + 1
    dummy = _events(nev)
    for _ in range(warmup):
        one_step(dummy)
    torch.cuda.synchronize()
    evs = [_events(nev) for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        one_step(evs[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = evs[0][0].elapsed_time(evs[-1][-1])
    stage = {n: 0.0 for n in STAGES}
    for ev in evs:
        for j, n in enumerate(STAGES):
            stage[n] += ev[j].elapsed_time(ev[j + 1]) / steps
    return max(gpu_ms, 0.0) / steps, wall_ms / steps, stage


def random_device_group(shape, flags):
    """A group of `shape` whose tensors are drawn on the device (torch.randn, seeded): for timing the other
    configs without minutes of host-side number generation.  Lengths come from the same seeded recipe as the parity
    workloads."""
    import torch
    from paper_2605_15422_amd import binding as B
    from paper_2605_15422_amd import workloads as W
    wl = W.make_workload(shape, tensors=False)
    g = torch.Generator(device="cuda")
    g.manual_seed(shape.seed)
    P, T, H, Hk, d = shape.ctx_len, wl.total_resp, shape.n_q_heads, shape.n_kv_heads, shape.head_dim

    def rnd(rows, heads):
        return torch.randn((rows, heads, d), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)

    shp = B.make_shape(shape.n_seqs, P, T, wl.max_resp, H, Hk, d, shape.window, wl.scale, flags)
    dg = B.DeviceGroup(shp, rnd(P, H), rnd(P, Hk), rnd(P, Hk), rnd(T, H), rnd(T, Hk), rnd(T, Hk), rnd(P, H), rnd(T, H),
                       torch.from_numpy(wl.cu_seqlens.copy()).cuda(), wl.cu_seqlens.copy())
    return wl, dg


def time_other_configs(names, flags, steps=2, warmup=1):
    """ms/layer, algorithmic TFLOP/s and fraction of the MFMA peak of the other benchmark configs (same step)."""
    import torch
    from paper_2605_15422_amd import accounting as acc
    from paper_2605_15422_amd import runner
    from paper_2605_15422_amd import workloads as W
    out = {}
    for name in names:
        shape = W.CONFIGS[name]
        wl, dg = random_device_group(shape, flags)
        bufs = runner.alloc(dg, poison=False)
        n = 20 if name == "cfg1_tiny" else steps
        ms, _, stage = time_layer(dg, bufs, n, warmup)
        fl = acc.layer_flops(shape, wl.resp_lens)
        tf = fl["layer"] / (ms * 1e-3) / 1e12
        out[name] = {"ms_per_layer": round(ms, 4), "tflops": round(tf, 2), "frac_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                     "layer_tflop": round(fl["layer"] / 1e12, 3), "steps": n,
                     "fwd_ms": round(stage["ctx_fwd"] + stage["fwd"], 4),
                     "bwd_ms": round(sum(v for k, v in stage.items() if k not in ("ctx_fwd", "fwd")), 4)}
        del bufs, dg
        torch.cuda.empty_cache()
    return out


def time_fused_calls(dg, steps, warmup):
    """Call 1 and Call 2 in ONE launch per stage: the prompt enters the *_groups entry points as a group of its own
    (a plain causal sequence without a shared prefix, P_g = 0) next to the group of the N responses, with prompt and
    response rows in one packed buffer.  Two-term mode: total dK_c = Call-1 rows of dK_d + Call-2 dK_c."""
    import numpy as np
    import torch
    from paper_2605_15422_amd import binding as B
    s = dg.shape_c
    P, T, N, H, Hk, d = s.ctx_len, s.total_resp, s.n_seqs, s.n_q_heads, s.n_kv_heads, s.head_dim
    cat = lambda a, b: torch.cat([a, b], dim=0)
    q, k, v, do = cat(dg.q_c, dg.q_d), cat(dg.k_c, dg.k_d), cat(dg.v_c, dg.v_d), cat(dg.do_c, dg.do_d)
    cu = np.concatenate([[0], P + np.asarray(dg.cu_host, dtype=np.int64)]).astype(np.int32)
    table = np.asarray([(0, 0, 0, 1), (0, P, 1, N + 1)], dtype=np.int32)
    shp = B.make_shape(N + 1, P, P + T, int(np.diff(cu).max()), H, Hk, d, s.window, s.softmax_scale, 0)
    g_dev, cu_dev = torch.from_numpy(table).cuda(), torch.from_numpy(cu).cuda()
    ws_f = torch.empty(max(16, B.dualkv_groups_workspace_bytes(shp, 2, P, B.OP_FWD)), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(max(16, B.dualkv_groups_workspace_bytes(shp, 2, P, B.OP_BWD)), dtype=torch.uint8, device="cuda")
    o, dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    dk_c, dv_c = torch.empty_like(dg.k_c), torch.empty_like(dg.v_c)
    lse = torch.empty((H, P + T), dtype=torch.float32, device="cuda")

    def step():
        B.dualkv_fwd_groups(shp, g_dev, None, P, q, k[:P], v[:P], k, v, cu_dev, None, o, lse, ws_f)
        B.dualkv_bwd_groups(shp, g_dev, None, P, do, o, lse, q, k[:P], v[:P], k, v, cu_dev, None, dq, dk_c, dv_c, dk, dv,
                            None, None, ws_b)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(2)
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_ncopy(wl, steps, warmup):
    """The same kernels on the explicitly replicated N x (P + R_i) layout (ctx_len = 0)."""
    import numpy as np
    import torch
    from paper_2605_15422_amd import binding as B, runner

    s = wl.shape
    N, P, T = s.n_seqs, s.ctx_len, wl.total_resp
    cu_dev = torch.from_numpy(wl.cu_seqlens.copy()).cuda()
    cu_rep = np.zeros(N + 1, dtype=np.int32)
    cu_rep[1:] = np.cumsum(P + wl.resp_lens)
    rows = int(cu_rep[-1])

    def rep(x_c, x_d):
        packed = torch.cat([B.bf16_from_bits(x_c), B.bf16_from_bits(x_d)], dim=0)
        out = torch.empty((rows,) + tuple(packed.shape[1:]), dtype=torch.bfloat16, device="cuda")
        B.dualkv_replicate(N, P, T, cu_dev, packed.shape[1] * packed.shape[2] * 2, packed, out)
        return out

    q, k, v, do = rep(wl.q_c, wl.q_d), rep(wl.k_c, wl.k_d), rep(wl.v_c, wl.v_d), rep(wl.do_c, wl.do_d)
    H, Hk, d = s.n_q_heads, s.n_kv_heads, s.head_dim
    shp = B.make_shape(N, 0, rows, int((P + wl.resp_lens).max()), H, Hk, d, s.window, wl.scale, 0)
    empty_q = torch.empty((0, H, d), dtype=torch.bfloat16, device="cuda")
    empty_k = torch.empty((0, Hk, d), dtype=torch.bfloat16, device="cuda")
    dg = B.DeviceGroup(shp, empty_q, empty_k, empty_k, q, k, v, empty_q, do, torch.from_numpy(cu_rep).cuda(), cu_rep)
    bufs = runner.alloc(dg, poison=False)

    def step():
        runner.forward(dg, bufs, call1=False)
        runner.backward(dg, bufs, call1=False)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(2)
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def cpu_baseline(wl, max_tokens=9216):
    """The fp64 oracle timed on this host: replica 0, KV head 0 with its query heads, fwd + bwd."""
    import numpy as np
    from oracle import attention_oracle as orc
    from paper_2605_15422_amd import workloads as W

    s = wl.shape
    P, G = s.ctx_len, s.group
    R0 = int(wl.resp_lens[0])
    f = W.bf16_bits_to_f64
    q = np.concatenate([f(wl.q_c[:, :G]), f(wl.q_d[:R0, :G])])[:max_tokens]
    k = np.concatenate([f(wl.k_c[:, :1]), f(wl.k_d[:R0, :1])])[:max_tokens]
    v = np.concatenate([f(wl.v_c[:, :1]), f(wl.v_d[:R0, :1])])[:max_tokens]
    do = np.concatenate([f(wl.do_c[:, :G]), f(wl.do_d[:R0, :G])])[:max_tokens]
    S = q.shape[0]
    t0 = time.perf_counter()
    orc.attn_fwd_seq(q, k, v, wl.scale, s.window)
    orc.attn_bwd_seq(q, k, v, do, wl.scale, s.window)
    dt = time.perf_counter() - t0
    pairs = orc.visible_pairs_call1(S, s.window)
    flops = 14 * s.head_dim * pairs * G
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": "numpy fp64 dense fwd+bwd of the first %d tokens of replica 0 (prompt + response 0), "
                      "KV head 0 with its %d query heads; algorithmic flops = 14*d*visible pairs" % (S, G)}


def time_repack(wl, reps=5):
    """Layout kernels on one (rows, H, d) bf16 tensor: single-prompt packing -> N replicated sequences and back."""
    import numpy as np
    import torch
    from paper_2605_15422_amd import binding as B
    s = wl.shape
    N, P, T = s.n_seqs, s.ctx_len, wl.total_resp
    cu_dev = torch.from_numpy(wl.cu_seqlens.copy()).cuda()
    packed = torch.cat([B.bf16_from_bits(wl.q_c), B.bf16_from_bits(wl.q_d)], dim=0)
    row_bytes = packed.shape[1] * packed.shape[2] * 2
    rows_rep = N * P + T
    standard = torch.empty((rows_rep,) + tuple(packed.shape[1:]), dtype=torch.bfloat16, device="cuda")
    back = torch.empty_like(packed)
    pos = torch.empty(P + T, dtype=torch.int32, device="cuda")
    res = {}
    for name, fn, nbytes in (
            ("replicate", lambda: B.dualkv_replicate(N, P, T, cu_dev, row_bytes, packed, standard), 2 * rows_rep * row_bytes),
            ("repack", lambda: B.dualkv_repack(N, P, T, cu_dev, row_bytes, standard, back, pos), 2 * (P + T) * row_bytes)):
        fn()
        ev = _events(2)
        ev[0].record()
        for _ in range(reps):
            fn()
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / reps
        res[name] = {"ms": round(ms, 4), "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1)}
    assert torch.equal(back, packed)
    if P > 0:
        # fp32 -> bf16 cast of the shared-prompt gradients (Alg. 2): 2 tensors x (4 B read + 2 B written) per element
        Hk, d = s.n_kv_heads, s.head_dim
        shp = B.make_shape(N, P, T, wl.max_resp, s.n_q_heads, Hk, d, s.window, wl.scale, 0)
        acc = [torch.randn((P, Hk, d), dtype=torch.float32, device="cuda") for _ in range(2)]
        outb = [torch.empty((P, Hk, d), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
        B.dualkv_finalize_ctx_grads(shp, acc[0], acc[1], outb[0], outb[1])
        ev = _events(2)
        ev[0].record()
        for _ in range(reps):
            B.dualkv_finalize_ctx_grads(shp, acc[0], acc[1], outb[0], outb[1])
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / reps
        res["finalize_ctx_grads"] = {"ms": round(ms, 4), "gbs": round(2 * P * Hk * d * 6 / (ms * 1e-3) / 1e9, 1)}
    res["what"] = ("one (rows, H, d) bf16 tensor, %d B per row: %d packed rows <-> %d replicated rows; GB/s counts bytes "
                   "read + written by the gather" % (row_bytes, P + T, rows_rep))
    return res


def groups_one_call(shape, dgs):
    """Packs the groups (device copies) into the multi-group layout and returns a function that runs one layer pass
    over all of them through the *_groups entry points."""
    import numpy as np
    import torch
    from paper_2605_15422_amd import binding as B
    cat = lambda name: torch.cat([getattr(dg, name) for dg in dgs], dim=0)
    t = {n: cat(n) for n in ("q_c", "k_c", "v_c", "do_c", "q_d", "k_d", "v_d", "do_d")}
    table, cu = [], [0]
    c_off = seq = 0
    for dg in dgs:
        n, P = dg.shape_c.n_seqs, dg.shape_c.ctx_len
        table.append((c_off, P, seq, seq + n))
        c_off += P
        seq += n
        cu.extend(int(cu[-1] + x) for x in np.diff(dg.cu_host))
    table = np.asarray(table, dtype=np.int32)
    cu = np.asarray(cu, dtype=np.int32)
    total_ctx, T = c_off, int(cu[-1])
    H, Hk, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    flags = B.FLAG_ACCUM_CTX_F32
    shp = B.make_shape(seq, max(dg.shape_c.ctx_len for dg in dgs), T, int(np.diff(cu).max()), H, Hk, d, shape.window,
                       0.0, flags)
    shp_all = B.make_shape(1, total_ctx, 0, 0, H, Hk, d, shape.window, 0.0, flags)
    g_dev, cu_dev = torch.from_numpy(table).cuda(), torch.from_numpy(cu).cuda()
    ws = {op: torch.empty(max(16, B.dualkv_groups_workspace_bytes(shp, len(dgs), total_ctx, op)), dtype=torch.uint8,
                          device="cuda") for op in (B.OP_CTX_FWD, B.OP_FWD, B.OP_CTX_BWD, B.OP_BWD)}
    o_c, o_d = torch.empty_like(t["q_c"]), torch.empty_like(t["q_d"])
    dq_c, dq_d = torch.empty_like(t["q_c"]), torch.empty_like(t["q_d"])
    dk_d, dv_d = torch.empty_like(t["k_d"]), torch.empty_like(t["v_d"])
    dk_c, dv_c = torch.empty_like(t["k_c"]), torch.empty_like(t["v_c"])
    a_k = torch.empty(t["k_c"].shape, dtype=torch.float32, device="cuda")
    a_v = torch.empty(t["v_c"].shape, dtype=torch.float32, device="cuda")
    lse_c = torch.empty((H, total_ctx), dtype=torch.float32, device="cuda")
    lse_d = torch.empty((H, T), dtype=torch.float32, device="cuda")

    def run():
        B.dualkv_ctx_fwd_groups(shp, g_dev, None, total_ctx, t["q_c"], t["k_c"], t["v_c"], o_c, lse_c, ws[B.OP_CTX_FWD])
        B.dualkv_fwd_groups(shp, g_dev, None, total_ctx, t["q_d"], t["k_c"], t["v_c"], t["k_d"], t["v_d"], cu_dev, None,
                            o_d, lse_d, ws[B.OP_FWD])
        B.dualkv_zero_ctx_grads(shp_all, a_k, a_v)
        B.dualkv_bwd_groups(shp, g_dev, None, total_ctx, t["do_d"], o_d, lse_d, t["q_d"], t["k_c"], t["v_c"], t["k_d"],
                            t["v_d"], cu_dev, None, dq_d, None, None, dk_d, dv_d, a_k, a_v, ws[B.OP_BWD])
        B.dualkv_ctx_bwd_groups(shp, g_dev, None, total_ctx, t["do_c"], o_c, lse_c, t["q_c"], t["k_c"], t["v_c"], dq_c,
                                None, None, a_k, a_v, ws[B.OP_CTX_BWD])
        B.dualkv_finalize_ctx_grads(shp_all, a_k, a_v, dk_c, dv_c)

    return run


def time_groups(shape, n_groups, steps):
    """`n_groups` prompt groups of `shape` (different seeds), one layer pass each: the per-group calls issued
    eagerly, and the same calls captured once in a HIP graph and replayed (one launch for all groups)."""
    import torch
    from paper_2605_15422_amd import binding as B, runner
    from paper_2605_15422_amd import workloads as W
    groups = []
    for g in range(n_groups):
        sh = W.Shape("%s_g%d" % (shape.name, g), shape.n_seqs, shape.ctx_len, shape.resp_lo, shape.resp_hi,
                     shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.window, shape.seed + 100 * (g + 1))
        dg = B.upload(W.make_workload(sh), B.FLAG_ACCUM_CTX_F32)
        groups.append((dg, runner.alloc(dg, poison=False)))

    def all_groups():
        for dg, b in groups:
            runner.layer_step(dg, b)

    # independent groups on a few streams (default priority): branches of the captured graph that may overlap
    side = [torch.cuda.Stream() for _ in range(min(4, n_groups))]

    def all_groups_forked():
        cur = torch.cuda.current_stream()
        for st in side:
            st.wait_stream(cur)
        for i, (dg, b) in enumerate(groups):
            with torch.cuda.stream(side[i % len(side)]):
                runner.layer_step(dg, b)
        for st in side:
            cur.wait_stream(st)

    all_groups()
    all_groups_forked()
    torch.cuda.synchronize()
    graph, graph_forked = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        all_groups()
    with torch.cuda.graph(graph_forked):
        all_groups_forked()
    one_call = groups_one_call(shape, [dg for dg, _ in groups])
    one_call()
    torch.cuda.synchronize()
    graph_one = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph_one):
        one_call()
    res = {}
    for name, fn in (("eager", all_groups), ("eager_streams", all_groups_forked), ("graph", graph.replay),
                     ("graph_branches", graph_forked.replay), ("one_call", one_call),
                     ("one_call_graph", graph_one.replay)):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        res[name] = round((time.perf_counter() - t0) * 1e3 / steps, 4)
    return {"groups": n_groups, **{k + "_ms": v for k, v in res.items()},
            "what": "wall time per pass over all groups: per-group calls issued one by one on one stream / on %d "
                    "streams, one replay of a HIP graph that captured them as a chain / as %d branches, and the "
                    "*_groups entry points (every kernel launched once for all groups), eagerly / as a graph"
                    % (len(side), len(side))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg2_qwen8b")
    ap.add_argument("--no-ncopy", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the other benchmark configs")
    ap.add_argument("--no-alt", action="store_true", help="skip the short run in the other gradient mode")
    ap.add_argument("--two-terms", action="store_true",
                    help="time the mode that returns the Call-1 and Call-2 terms of dK_c / dV_c as two bf16 tensors "
                         "(the paper's interface) instead of the fp32 joint accumulation with one cast")
    ap.add_argument("--ncopy-steps", type=int, default=2)
    ap.add_argument("--graph-groups", type=int, default=0,
                    help="also time this many prompt groups of the config, eagerly and as one captured graph")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (one GPU per box; no collectives are built); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_15422_amd import accounting as acc
    from paper_2605_15422_amd import binding as B, runner
    from paper_2605_15422_amd import workloads as W

    torch.cuda.set_device(0)
    shape = W.CONFIGS[args.config]
    wl = W.make_workload(shape)
    fl = acc.layer_flops(shape, wl.resp_lens)
    flags = 0 if args.two_terms else B.FLAG_ACCUM_CTX_F32
    dg = B.upload(wl, flags)
    bufs = runner.alloc(dg, poison=False)
    torch.cuda.synchronize()

    ms, wall_ms, stage = time_layer(dg, bufs, args.steps, args.warmup)
    # the other mode, for reference (fewer steps)
    ms_alt = ms_fused = None
    if not args.no_alt:
        ms_fused = time_fused_calls(dg, max(3, args.steps // 2), 2)
        dg_alt = B.upload(wl, B.FLAG_ACCUM_CTX_F32 if args.two_terms else 0)
        bufs_alt = runner.alloc(dg_alt, poison=False)
        ms_alt, _, _ = time_layer(dg_alt, bufs_alt, max(3, args.steps // 3), 1)
        del dg_alt, bufs_alt

    # dominant kernel and its roofline (MFMA bound: algorithmic flops of that kernel / its duration)
    d, H = shape.head_dim, shape.n_q_heads
    kern_flops = {
        "ctx_fwd": 4 * d * H * fl["pairs_call1"], "fwd": 4 * d * H * fl["pairs_call2"],
        "bwd_dkdv": 8 * d * H * fl["pairs_call2"], "bwd_dq": 2 * d * H * fl["pairs_call2"],
        "ctx_bwd_dkdv": 8 * d * H * fl["pairs_call1"], "ctx_bwd_dq": 2 * d * H * fl["pairs_call1"],
    }
    dom = max(kern_flops, key=lambda n: stage[n])
    achieved = kern_flops[dom] / (stage[dom] * 1e-3) / 1e12 if stage[dom] > 0 else 0.0
    # the kernel symbols that serve this head dim (as the rocprofv3 kernel trace names them)
    fam = {64: ("fwd2_kernel", "dq2_kernel", "dkdv4_kernel"), 128: ("fwd2_kernel", "dq2_kernel", "dkdv4_kernel"),
           256: ("fwd256_kernel", "dq256_kernel", "dkdv256_kernel"),
           512: ("fwd512_kernel", "dq512_kernel", "dkdv512_kernel")}.get(d, ("fwd_kernel", "dq_kernel", "dkdv_kernel"))
    kernel_names = {"ctx_fwd": fam[0] + " (Call 1)", "fwd": fam[0] + " (Call 2)",
                    "bwd_dkdv": fam[2] + " (Call 2)", "bwd_dq": fam[1] + " (Call 2)",
                    "ctx_bwd_dkdv": fam[2] + " (Call 1)", "ctx_bwd_dq": fam[1] + " (Call 1)"}
    roofline = {"bound": "mfma", "kernel": kernel_names[dom], "achieved": round(achieved, 2),
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                "traffic": measured_traffic(args.config, dom), "kernel_ms": round(stage[dom], 4),
                "algorithmic_flops_per_launch": kern_flops[dom]}

    tflops = fl["layer"] / (ms * 1e-3) / 1e12
    out = {
        "metric": "DualKV attn fwd+bwd ms/layer & TFLOP/s (MFMA util) vs N-copy attention",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: N=%d P=%d R=[%d,%d] (sum %d) H=%d Hk=%d d=%d window=%d, Q/K/V/dO ~ N(0,1) seed %d" % (
            shape.name, shape.n_seqs, shape.ctx_len, int(wl.resp_lens.min()), int(wl.resp_lens.max()),
            wl.total_resp, shape.n_q_heads, shape.n_kv_heads, d, shape.window, shape.seed),
            "packed_tokens": shape.ctx_len + wl.total_resp},
        "frac_mfma_peak": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "layer_tflop": round(fl["layer"] / 1e12, 3),
        "wall_ms_per_step": round(wall_ms, 4),
        "stage_ms": {k: round(v, 4) for k, v in stage.items()},
        "stage_tflops": {k: round(kern_flops[k] / (stage[k] * 1e-3) / 1e12, 1) for k in kern_flops if stage[k] > 0},
        "fwd_ms": round(stage["ctx_fwd"] + stage["fwd"], 4),
        "bwd_ms": round(sum(v for k, v in stage.items() if k not in ("ctx_fwd", "fwd")), 4),
        "ctx_grad_mode": ("two bf16 terms (Call 1, Call 2), summed by the caller" if args.two_terms else
                          "fp32 joint accumulation of Call 1 + Call 2, one cast (Eq. 6 inside the timed step)"),
        ("ms_per_step_joint_fp32" if args.two_terms else "ms_per_step_two_terms"): (round(ms_alt, 4) if ms_alt else None),
        "ms_per_step_fused_calls": (round(ms_fused, 4) if ms_fused else None),
        "roofline": roofline,
        "ncopy_flop_ratio": round(fl["ncopy"] / fl["layer"], 3),   # FLOPs of N-copy attention over this layer's
    }
    pre_bytes = 2 * wl.total_resp * H * d * 2 + wl.total_resp * H * 4
    if stage["bwd_pre"] > 0:
        out["preprocess_gbs"] = round(pre_bytes / (stage["bwd_pre"] * 1e-3) / 1e9, 1)

    if not args.no_ncopy:
        del bufs
        torch.cuda.empty_cache()
        nms = time_ncopy(wl, args.ncopy_steps, 1)
        out["ncopy"] = {"ms_per_step": round(nms, 3), "tflop": round(fl["ncopy"] / 1e12, 3),
                        "tflops": round(fl["ncopy"] / (nms * 1e-3) / 1e12, 2), "speedup_dualkv": round(nms / ms, 3),
                        "flop_ratio": round(fl["ncopy"] / fl["layer"], 3),
                        "what": "same kernels on the replicated N x (P+R_i) layout (ctx_len=0), fwd+bwd"}
    if not args.no_ncopy:
        out["layout_kernels"] = time_repack(wl)
    if not args.no_others and args.config == "cfg2_qwen8b":
        del dg
        torch.cuda.empty_cache()
        out["other_configs"] = time_other_configs(["cfg1_tiny", "cfg3_ragged", "cfg4_30b", "cfg5b_swa", "cfg5a_global"], flags)
    if args.graph_groups > 0:
        out["multi_group"] = time_groups(shape, args.graph_groups, max(args.steps, 20))
    elif not args.no_others and args.config == "cfg2_qwen8b":
        # several prompt groups in one call (Sec. 2.2): eight groups of config 1
        out["multi_group"] = time_groups(W.CONFIGS["cfg1_tiny"], 8, 20)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
