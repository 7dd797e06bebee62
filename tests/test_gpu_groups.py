"""Several prompt groups in ONE call of the *_groups entry points (Sec. 2.2, "multiple groups") against the fp64
oracle evaluated group by group: heterogeneous prompt lengths (including P_g = 0), a group without sequences,
empty responses, both gradient modes, every kernel family (d = 64/128, 256, 512, 96), with and without a window."""
import numpy as np
import pytest

from oracle import attention_oracle as orc
from paper_2605_15422_amd import workloads as W

import parity_util as PU

pytestmark = pytest.mark.gpu


def _build(specs, H, Hk, d, window, seed):
    """specs: list of (P_g, response lengths).  Returns per-group workloads and the packed arrays / tables."""
    wls = []
    for g, (P, lens) in enumerate(specs):
        shape = W.Shape("grp%d" % g, max(len(lens), 1), P, 0, 0, H, Hk, d, window, seed=seed + 17 * g)
        # a group without sequences is given one empty response on the oracle side: its prompt pass is unchanged
        wls.append(W.make_workload(shape, resp_lens=np.asarray(lens if len(lens) else [0])))
    cat = lambda name: np.concatenate([getattr(w, name) for w in wls], axis=0)
    packed = {n: cat(n) for n in ("q_c", "k_c", "v_c", "do_c", "q_d", "k_d", "v_d", "do_d")}
    table, cu = [], [0]
    ctx_off = seq = 0
    for (P, lens) in specs:
        table.append((ctx_off, P, seq, seq + len(lens)))
        ctx_off += P
        seq += len(lens)
        for r in lens:
            cu.append(cu[-1] + int(r))
    return wls, packed, np.asarray(table, dtype=np.int32).reshape(-1, 4), np.asarray(cu, dtype=np.int32)


def _oracle(wls, window):
    refs = []
    for w in wls:
        x = PU.oracle_inputs(w)
        refs.append(orc.dualkv_reference(x["q_c"], x["k_c"], x["v_c"], x["q_d"], x["k_d"], x["v_d"], w.cu_seqlens, w.scale,
                                         x["do_c"], x["do_d"], window))
    return refs


def _run_groups(specs, packed, table, cu, H, Hk, d, window, flags):
    import torch
    from paper_2605_15422_amd import binding as B
    dev = {k: B.bf16_from_bits(v) for k, v in packed.items()}
    n_seqs = len(cu) - 1
    total_ctx, T = int(packed["q_c"].shape[0]), int(cu[-1])
    lens = np.diff(cu)
    max_p = max(P for P, _ in specs)
    shp = B.make_shape(max(n_seqs, 1), max_p, T, int(lens.max()) if n_seqs else 0, H, Hk, d, window, 0.0, flags)
    g_dev = torch.from_numpy(table.copy()).cuda()
    cu_dev = torch.from_numpy(cu.copy()).cuda()

    def ws(op):
        n = B.dualkv_groups_workspace_bytes(shp, len(specs), total_ctx, op)
        return torch.full((max(n, 16),), 0xFF, dtype=torch.uint8, device="cuda")

    def nan_like(t):
        x = torch.empty_like(t)
        x.view(torch.int16).fill_(0x7FC0)
        return x

    out = dict(o_c=nan_like(dev["q_c"]), o_d=nan_like(dev["q_d"]), dq_c=nan_like(dev["q_c"]), dq_d=nan_like(dev["q_d"]),
               dk_d=nan_like(dev["k_d"]), dv_d=nan_like(dev["v_d"]),
               lse_c=torch.full((H, total_ctx), float("nan"), device="cuda"),
               lse_d=torch.full((H, T), float("nan"), device="cuda"))
    acc = bool(flags & B.FLAG_ACCUM_CTX_F32)
    if acc:
        out["dk_c_acc"] = torch.full(dev["k_c"].shape, float("nan"), dtype=torch.float32, device="cuda")
        out["dv_c_acc"] = torch.full(dev["v_c"].shape, float("nan"), dtype=torch.float32, device="cuda")
        out["dk_c"], out["dv_c"] = nan_like(dev["k_c"]), nan_like(dev["v_c"])
        shp_all = B.make_shape(1, total_ctx, 0, 0, H, Hk, d, window, 0.0, flags)
        B.dualkv_zero_ctx_grads(shp_all, out["dk_c_acc"], out["dv_c_acc"])
    else:
        for n in ("dk_c1", "dv_c1", "dk_c2", "dv_c2"):
            out[n] = nan_like(dev["k_c"])
    B.dualkv_ctx_fwd_groups(shp, g_dev, table, total_ctx, dev["q_c"], dev["k_c"], dev["v_c"], out["o_c"], out["lse_c"],
                            ws(B.OP_CTX_FWD))
    B.dualkv_fwd_groups(shp, g_dev, table, total_ctx, dev["q_d"], dev["k_c"], dev["v_c"], dev["k_d"], dev["v_d"], cu_dev,
                        cu, out["o_d"], out["lse_d"], ws(B.OP_FWD))
    B.dualkv_bwd_groups(shp, g_dev, table, total_ctx, dev["do_d"], out["o_d"], out["lse_d"], dev["q_d"], dev["k_c"],
                        dev["v_c"], dev["k_d"], dev["v_d"], cu_dev, cu, out["dq_d"],
                        None if acc else out["dk_c2"], None if acc else out["dv_c2"], out["dk_d"], out["dv_d"],
                        out.get("dk_c_acc"), out.get("dv_c_acc"), ws(B.OP_BWD))
    B.dualkv_ctx_bwd_groups(shp, g_dev, table, total_ctx, dev["do_c"], out["o_c"], out["lse_c"], dev["q_c"], dev["k_c"],
                            dev["v_c"], out["dq_c"], None if acc else out["dk_c1"], None if acc else out["dv_c1"],
                            out.get("dk_c_acc"), out.get("dv_c_acc"), ws(B.OP_CTX_BWD))
    if acc:
        B.dualkv_finalize_ctx_grads(shp_all, out["dk_c_acc"], out["dv_c_acc"], out["dk_c"], out["dv_c"])
    torch.cuda.synchronize()
    return dev, out


CASES = [
    # name, H, Hk, d, window, specs
    ("d128_mixed", 8, 2, 128, 0, [(100, [40, 17, 64]), (0, [33, 5]), (257, []), (64, [1, 0, 130])]),
    ("d64_window", 4, 2, 64, 37, [(150, [120, 0]), (31, [200]), (0, [70])]),
    ("d128_many_small", 4, 4, 128, 0, [(33, [5, 9]), (1, [1]), (129, [64, 64, 64]), (200, [3]), (7, [0, 0]), (90, [31, 33])]),
    ("d256_roles", 4, 2, 256, 0, [(130, [64, 31]), (0, [20]), (65, [])]),
    ("d512_roles", 2, 1, 512, 0, [(65, [33, 70]), (40, [9])]),
    ("d96_window", 2, 2, 96, 40, [(130, [90, 33]), (50, [64])]),
    ("d256_window", 4, 1, 256, 48, [(90, [100, 17]), (0, [70]), (200, [33, 0, 64])]),
    ("d512_many", 4, 2, 512, 0, [(17, [16, 15]), (0, [40]), (64, []), (33, [1, 31, 17])]),
]


@pytest.mark.parametrize("flags", [0, 1], ids=["two_terms", "joint_fp32"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_groups_in_one_call_match_the_oracle_group_by_group(case, flags):
    name, H, Hk, d, window, specs = case
    print("case groups", name, flags, flush=True)
    wls, packed, table, cu = _build(specs, H, Hk, d, window, seed=5100 + len(name))
    refs = _oracle(wls, window)
    dev, out = _run_groups(specs, packed, table, cu, H, Hk, d, window, flags)
    rep = []
    try:
        seq = 0
        for g, ((P, lens), ref) in enumerate(zip(specs, refs)):
            c0 = int(table[g, 0])
            r0, r1 = int(cu[seq]), int(cu[seq + len(lens)])
            seq += len(lens)
            tag = "g%d " % g
            cs, rs = slice(c0, c0 + P), slice(r0, r1)
            PU.compare(tag + "O_c", PU.to_f64(out["o_c"][cs]), ref["o_c"], rep)
            PU.compare_lse(tag + "LSE_c", PU.to_f64(out["lse_c"][:, cs]), ref["lse_c"], rep)
            PU.compare(tag + "dQ_c", PU.to_f64(out["dq_c"][cs]), ref["call1"]["dq_c"], rep)
            if len(lens):
                PU.compare(tag + "O_d", PU.to_f64(out["o_d"][rs]), ref["o_d"], rep)
                PU.compare_lse(tag + "LSE_d", PU.to_f64(out["lse_d"][:, rs]), ref["lse_d"], rep)
                for n in ("dq_d", "dk_d", "dv_d"):
                    PU.compare(tag + n, PU.to_f64(out[n][rs]), ref["call2"][n], rep)
            if flags & 1:
                for n in ("dk_c", "dv_c"):
                    PU.compare(tag + n + "32", PU.to_f64(out[n + "_acc"][cs]), ref["total"][n], rep)
                    PU.compare(tag + n, PU.to_f64(out[n][cs]), ref["total"][n], rep)
            else:
                for n in ("dk_c", "dv_c"):
                    PU.compare(tag + n + "(2)", PU.to_f64(out[n + "2"][cs]), ref["call2"][n], rep)
                    PU.compare(tag + n + "(1)", PU.to_f64(out[n + "1"][cs]), ref["call1"][n], rep)
    finally:
        print("\n[groups %s flags=%d]\n  " % (name, flags) + "\n  ".join(rep), flush=True)


def test_groups_call_equals_the_per_group_calls_bit_for_bit():
    """Outputs that involve no atomics are the same bits whether the groups go through one *_groups call or through one
    single-group call each (same kernels, same tiles, same summation order)."""
    import torch
    from paper_2605_15422_amd import binding as B, runner
    H, Hk, d, window = 8, 2, 128, 0
    specs = [(300, [90, 260]), (64, [128]), (517, [131, 70, 1])]
    wls, packed, table, cu = _build(specs, H, Hk, d, window, seed=6200)
    dev, out = _run_groups(specs, packed, table, cu, H, Hk, d, window, 0)
    seq = 0
    for g, ((P, lens), wl) in enumerate(zip(specs, wls)):
        dg = B.upload(wl)
        b = runner.alloc(dg)
        runner.layer_step(dg, b)
        torch.cuda.synchronize()
        c0 = int(table[g, 0])
        cs, rs = slice(c0, c0 + P), slice(int(cu[seq]), int(cu[seq + len(lens)]))
        seq += len(lens)
        for n, sl in (("o_c", cs), ("dq_c", cs), ("o_d", rs), ("dq_d", rs), ("dk_d", rs), ("dv_d", rs)):
            assert torch.equal(out[n][sl].view(torch.int16), getattr(b, n).view(torch.int16)), (g, n)
        assert torch.equal(out["lse_c"][:, cs], b.lse_c) and torch.equal(out["lse_d"][:, rs], b.lse_d), g


def test_group_table_validation_on_the_host():
    import ctypes as C
    from paper_2605_15422_amd import binding as B
    shp = B.make_shape(3, 100, 50, 30, 4, 2, 128)
    null, nullo = B.TIn(None, 0, 0), B.TOut(None, 0, 0)

    def rc(table, total_ctx=150):
        t = np.asarray(table, dtype=np.int32).reshape(-1, 4)
        fake_dev = C.c_void_p(0x1000)
        return B.lib.dualkv_fwd_groups(C.byref(shp), len(t), fake_dev, t.ctypes.data_as(C.c_void_p), total_ctx, null, null,
                                       null, null, null, None, None, nullo, None, None, 0, None)

    assert rc([(0, 100, 0, 2), (100, 50, 2, 3)]) == B.E_INVALID      # passes the table, then NULL tensors
    assert rc([(0, 100, 0, 2), (100, 50, 1, 3)]) == B.E_INVALID      # sequence ranges overlap
    assert rc([(0, 100, 0, 2)]) == B.E_INVALID                        # sequences 2.. not covered
    assert rc([(0, 101, 0, 3)]) == B.E_INVALID                        # P_g above shape.ctx_len
    assert rc([(100, 60, 0, 3)]) == B.E_INVALID                       # prompt beyond total_ctx
    assert B.lib.dualkv_fwd_groups(C.byref(shp), 0, None, None, 0, null, null, null, null, null, None, None, nullo, None,
                                   None, 0, None) == B.E_INVALID
    assert B.dualkv_groups_workspace_bytes(shp, 2, 150, B.OP_FWD) >= 3 * 8


def test_large_groups_take_the_unsplit_prompt_tile_path():
    """Groups of realistic size (hundreds of prompt tiles: every prompt tile is owned by ONE workgroup that sums all the
    sequences and heads of its group in registers and writes bf16 directly, no atomics): the *_groups call must then
    reproduce the per-group calls bit for bit on EVERY output, including the shared-prompt gradients, with prompt
    lengths that differ by 4x, a group without sequences and ragged responses."""
    import torch
    from paper_2605_15422_amd import binding as B, runner
    H, Hk, d, window = 16, 8, 128, 0
    specs = [(8192, [700, 1024, 333]), (2048, [1500]), (4100, []), (16384, [64, 2000, 1, 900])]
    print("case large groups", flush=True)
    wls, packed, table, cu = _build(specs, H, Hk, d, window, seed=7300)
    dev, out = _run_groups(specs, packed, table, cu, H, Hk, d, window, 0)
    seq = 0
    for g, ((P, lens), wl) in enumerate(zip(specs, wls)):
        dg = B.upload(wl)
        b = runner.alloc(dg)
        runner.layer_step(dg, b)
        torch.cuda.synchronize()
        c0 = int(table[g, 0])
        cs, rs = slice(c0, c0 + P), slice(int(cu[seq]), int(cu[seq + len(lens)]))
        seq += len(lens)
        names = [("o_c", cs), ("dq_c", cs), ("dk_c1", cs), ("dv_c1", cs)]
        if len(lens):
            names += [("o_d", rs), ("dq_d", rs), ("dk_d", rs), ("dv_d", rs)]
        for n, sl in names:
            assert torch.equal(out[n][sl].view(torch.int16), getattr(b, n).view(torch.int16)), (g, n)
        # a per-group call of a short prompt (fewer than 512 prompt-tile workgroups) cuts its sequence loop and sums
        # with fp32 atomics; the long prompts are summed in registers in both routes: same bits
        unsplit_alone = (P + 127) // 128 * Hk >= 512
        for n in ("dk_c2", "dv_c2") if len(lens) else ():
            a, c = out[n][cs].float(), getattr(b, n).float()
            if unsplit_alone:
                assert torch.equal(a, c), (g, n)
            else:
                assert float((a - c).norm()) <= 1e-2 * float(c.norm()), (g, n)
        assert torch.equal(out["lse_c"][:, cs], b.lse_c), g
        if len(lens):
            assert torch.equal(out["lse_d"][:, rs], b.lse_d), g
        else:   # no sequence attends to this prompt: its Call-2 gradients are exact zeros
            assert float(out["dk_c2"][cs].float().abs().max()) == 0.0 and float(out["dv_c2"][cs].float().abs().max()) == 0.0
    # sampled rows of the largest group against the oracle's one-row evaluation (Eq. 4)
    rng = np.random.default_rng(5)
    g, (P, lens), wl = 3, specs[3], wls[3]
    c0, r0 = int(table[g, 0]), int(cu[4])
    f = W.bf16_bits_to_f64
    k_c, v_c, k_d, v_d = f(wl.k_c[:, :1]), f(wl.v_c[:, :1]), f(wl.k_d[:, :1]), f(wl.v_d[:, :1])
    q_d, do_d = f(wl.q_d[:, :2]), f(wl.do_d[:, :2])
    got_o, ref_o, got_l, ref_l, got_q, ref_q = [], [], [], [], [], []
    for _ in range(12):
        i = int(rng.choice([0, 1, 3]))
        r = int(rng.integers(0, lens[i]))
        hh = int(rng.integers(0, 2))
        row = int(wl.cu_seqlens[i]) + r
        o, lse, dq = orc.response_row(q_d, k_c, v_c, k_d, v_d, wl.cu_seqlens, wl.scale, i, r, hh, 0, do_row=do_d[row, hh])
        ref_o.append(o); ref_l.append(lse); ref_q.append(dq)
        got_o.append(PU.to_f64(out["o_d"][r0 + row, hh])); got_l.append(float(out["lse_d"][hh, r0 + row]))
        got_q.append(PU.to_f64(out["dq_d"][r0 + row, hh]))
    rep = []
    PU.compare("O_d", np.array(got_o), np.array(ref_o), rep)
    PU.compare_lse("LSE_d", np.array(got_l), np.array(ref_l), rep)
    PU.compare("dQ_d", np.array(got_q), np.array(ref_q), rep)
    print("\n  " + "\n  ".join(rep), flush=True)


@pytest.mark.parametrize("d,window", [(128, 0), (64, 50), (256, 0)])
def test_call1_and_call2_in_one_launch(d, window):
    """The prompt itself as a group of its own (a plain causal sequence, P_g = 0) next to the group of its N responses,
    prompt and response rows in one packed buffer: one forward launch and one backward call then cover Call 1 and
    Call 2 (Eq. 3 and Eq. 4 together).  Every output equals that of the four separate entry points: bit for bit where
    no atomics are involved, the Call-2 shared-prompt term (fp32 atomics on these small shapes) within the parity
    tolerance; total dK_c = Call-1 rows of dK_d + Call-2 dK_c (Eq. 6)."""
    import torch
    from paper_2605_15422_amd import binding as B, runner
    print("case fused calls", d, window, flush=True)
    H, Hk, P, lens = 8, 2, 333, [190, 0, 77, 260]
    shape = W.Shape("fused", len(lens), P, 0, 0, H, Hk, d, window, seed=8800 + d)
    wl = W.make_workload(shape, resp_lens=np.asarray(lens))
    dg = B.upload(wl)
    ref = runner.alloc(dg)
    runner.layer_step(dg, ref)
    N, T = len(lens), wl.total_resp
    cat = lambda a, b: torch.cat([a, b], dim=0)
    q, k, v, do = cat(dg.q_c, dg.q_d), cat(dg.k_c, dg.k_d), cat(dg.v_c, dg.v_d), cat(dg.do_c, dg.do_d)
    cu = np.concatenate([[0], P + wl.cu_seqlens.astype(np.int64)]).astype(np.int32)
    table = np.asarray([(0, 0, 0, 1), (0, P, 1, N + 1)], dtype=np.int32)
    shp = B.make_shape(N + 1, P, P + T, int(np.diff(cu).max()), H, Hk, d, window, wl.scale, 0)
    g_dev, cu_dev = torch.from_numpy(table).cuda(), torch.from_numpy(cu).cuda()
    ws = lambda op: torch.full((max(16, B.dualkv_groups_workspace_bytes(shp, 2, P, op)),), 0xFF, dtype=torch.uint8, device="cuda")

    def nan_like(t):
        x = torch.empty_like(t)
        x.view(torch.int16).fill_(0x7FC0)
        return x

    o, dq, dk, dv = nan_like(q), nan_like(q), nan_like(k), nan_like(v)
    dk_c, dv_c = nan_like(dg.k_c), nan_like(dg.v_c)
    lse = torch.full((H, P + T), float("nan"), device="cuda")
    B.dualkv_fwd_groups(shp, g_dev, table, P, q, k[:P], v[:P], k, v, cu_dev, cu, o, lse, ws(B.OP_FWD))
    B.dualkv_bwd_groups(shp, g_dev, table, P, do, o, lse, q, k[:P], v[:P], k, v, cu_dev, cu, dq, dk_c, dv_c, dk, dv,
                        None, None, ws(B.OP_BWD))
    torch.cuda.synchronize()
    bits = lambda t: t.contiguous().view(torch.int16)
    for got, want, name in ((o[:P], ref.o_c, "O_c"), (o[P:], ref.o_d, "O_d"), (dq[:P], ref.dq_c, "dQ_c"),
                            (dq[P:], ref.dq_d, "dQ_d"), (dk[P:], ref.dk_d, "dK_d"), (dv[P:], ref.dv_d, "dV_d"),
                            (dk[:P], ref.dk_c1, "dK_c(1)"), (dv[:P], ref.dv_c1, "dV_c(1)")):
        assert torch.equal(bits(got), bits(want)), name
    assert torch.equal(lse[:, :P], ref.lse_c) and torch.equal(lse[:, P:], ref.lse_d)
    for got, want, name in ((dk_c, ref.dk_c2, "dK_c(2)"), (dv_c, ref.dv_c2, "dV_c(2)")):
        a, c = got.float(), want.float()
        assert bool(((a - c).abs() <= 2e-2 + 2.0 ** -8 * c.abs()).all()), name
        assert float((a - c).norm()) <= 1e-2 * float(c.norm()), name
