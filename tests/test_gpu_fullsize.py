"""GPU parity at the FULL benchmark sizes, in the launch configuration bench.py times.

The dense fp64 oracle is too slow at these sizes, so each config is checked three ways:
  1. seeded samples of query rows (O, LSE, dQ of both calls) against the oracle's one-row evaluation of
     Eq. 3 / Eq. 4, including first / last rows and rows next to tile edges;
  2. the shared accumulation itself (Sec. 3.2, Alg. 1 + Alg. 2, App. A.5), configs 2 and 3: with the DENSE upstream
     gradient, dK_c / dV_c of a seeded sample of >= 256 prompt keys of one seeded KV head -- each the fp32 sum of
     the contributions of every response row of all N sequences and the G heads of the group -- and dK_d / dV_d of
     sampled response keys, element by element against the oracle's column evaluation over ALL rows of that head
     group (one fp64 pass over its (row, key) pairs);
     configs 4 and 5, where that pass takes many minutes: a second backward with an upstream gradient that is
     non-zero only on a seeded set of rows: dK / dV of sampled prompt keys and response keys of one KV head then
     depend on those rows only, and are compared with the oracle's column evaluation (all sequences contribute
     to the shared prompt keys);
  3. identities that hold for the full dense-gradient outputs at any size: sum_j dV_j = sum_rows dO
     (softmax rows sum to one), sum_j dK_j = 0 (rows of dS sum to zero), <q,dq> = <k,dk> (scale symmetry),
     per KV head, over prompt + response keys of Call 2 and over the prompt keys of Call 1.
"""
import numpy as np
import pytest

from oracle import attention_oracle as orc
from paper_2605_15422_amd import workloads as W

import parity_util as PU

pytestmark = pytest.mark.gpu

N_ROW_SAMPLES = 48
N_SPARSE_ROWS = 24
N_KEY_SAMPLES = 40
N_DENSE_CTX_KEYS = 256          # prompt keys checked against the dense-gradient column evaluation (configs 2, 3)
N_DENSE_DEC_KEYS = 64
DENSE_COLUMN_CONFIGS = ("cfg2_qwen8b", "cfg3_ragged")


def _say(*a):
    print(*a, flush=True)


def _f32(bits):
    return W.bf16_bits_to_f32(bits)


def _sample_rows(rng, wl, n):
    """(i, r) pairs: first / last rows, rows next to 32- and 64-row tile edges, and random ones."""
    lens = wl.resp_lens
    out = set()
    for i in (0, len(lens) - 1, int(np.argmax(lens)), int(np.argmin(lens))):
        R = int(lens[i])
        if R == 0:
            continue
        for r in (0, R - 1, min(R - 1, 31), min(R - 1, 32), min(R - 1, 63), min(R - 1, 64), R // 2):
            out.add((i, int(r)))
    while len(out) < n:
        i = int(rng.integers(0, len(lens)))
        if lens[i] > 0:
            out.add((i, int(rng.integers(0, lens[i]))))
    return sorted(out)[:max(n, 1)] if len(out) > n else sorted(out)


# the five benchmark configs, plus two shapes of the paper-shape sweeps: a Tab. 1 point with N = 28 sequences and the
# longest prompt of the prompt-length grid (P = 131072, where 32-bit offset arithmetic is most at risk)
@pytest.mark.parametrize("name", ["cfg2_qwen8b", "cfg3_ragged", "cfg4_30b", "cfg5b_swa", "cfg5a_global",
                                  "tab1_n28_p16k", "grid_p131072_mb4"])
def test_full_size(name):
    import torch
    from paper_2605_15422_amd import binding as B, runner

    shape = W.CONFIGS[name]
    _say("case", name, "generating inputs")
    wl = W.make_workload(shape)
    rng = np.random.default_rng(shape.seed + 7)
    P, cu, G, d, Wn = shape.ctx_len, wl.cu_seqlens, shape.group, shape.head_dim, shape.window
    T, H, Hk = wl.total_resp, shape.n_q_heads, shape.n_kv_heads
    kv = int(rng.integers(0, Hk))
    hs = slice(kv * G, (kv + 1) * G)

    _say("  uploading / running the layer (dense dO)")
    dg = B.upload(wl)
    bufs = runner.alloc(dg)
    runner.layer_step(dg, bufs)
    torch.cuda.synchronize()

    # ---- oracle-side views of the selected KV head group (bf16 -> fp32 is exact; products run in fp64)
    k_c = W.bf16_bits_to_f64(wl.k_c[:, kv:kv + 1])
    v_c = W.bf16_bits_to_f64(wl.v_c[:, kv:kv + 1])
    k_d = W.bf16_bits_to_f64(wl.k_d[:, kv:kv + 1])
    v_d = W.bf16_bits_to_f64(wl.v_d[:, kv:kv + 1])
    q_c, do_c = _f32(wl.q_c[:, hs]), _f32(wl.do_c[:, hs])
    q_d, do_d = _f32(wl.q_d[:, hs]), _f32(wl.do_d[:, hs])

    rep = []
    try:
        # ---- 1. sampled query rows
        _say("  sampled rows")
        rows = _sample_rows(rng, wl, N_ROW_SAMPLES)
        got_o, ref_o, got_l, ref_l, got_dq, ref_dq = [], [], [], [], [], []
        o_d, lse_d, dq_d = bufs.o_d, bufs.lse_d, bufs.dq_d
        for (i, r) in rows:
            g = int(rng.integers(0, G))
            h = kv * G + g
            row = int(cu[i]) + r
            o, lse, dq = orc.response_row(q_d, k_c, v_c, k_d, v_d, cu, wl.scale, i, r, g, Wn, do_row=do_d[row, g].astype(np.float64))
            ref_o.append(o); ref_l.append(lse); ref_dq.append(dq)
            got_o.append(PU.to_f64(o_d[row, h])); got_l.append(float(lse_d[h, row])); got_dq.append(PU.to_f64(dq_d[row, h]))
        PU.compare("O_d", np.array(got_o), np.array(ref_o), rep)
        PU.compare_lse("LSE_d", np.array(got_l), np.array(ref_l), rep)
        PU.compare("dQ_d", np.array(got_dq), np.array(ref_dq), rep)
        got_o, ref_o, got_l, ref_l, got_dq, ref_dq = [], [], [], [], [], []
        prow = sorted(set([0, 1, 31, 32, 63, 64, P // 2, P - 1] + [int(x) for x in rng.integers(0, P, size=16)]))
        for t in prow:
            g = int(rng.integers(0, G))
            h = kv * G + g
            o, lse, dq = orc.prompt_row(q_c, k_c, v_c, wl.scale, t, g, Wn, do_row=do_c[t, g].astype(np.float64))
            ref_o.append(o); ref_l.append(lse); ref_dq.append(dq)
            got_o.append(PU.to_f64(bufs.o_c[t, h])); got_l.append(float(bufs.lse_c[h, t]))
            got_dq.append(PU.to_f64(bufs.dq_c[t, h]))
        PU.compare("O_c", np.array(got_o), np.array(ref_o), rep)
        PU.compare_lse("LSE_c", np.array(got_l), np.array(ref_l), rep)
        PU.compare("dQ_c", np.array(got_dq), np.array(ref_dq), rep)

        # ---- 3. identities on the dense-gradient outputs (fp64 reductions of the device tensors)
        _say("  identities")
        f64 = torch.float64
        for k in range(Hk):
            g0, g1 = k * G, (k + 1) * G
            sum_do = dg.do_d[:, g0:g1].to(f64).sum(dim=(0, 1))
            sum_dv = bufs.dv_c2[:, k].to(f64).sum(0) + bufs.dv_d[:, k].to(f64).sum(0)
            sum_dk = bufs.dk_c2[:, k].to(f64).sum(0) + bufs.dk_d[:, k].to(f64).sum(0)
            abs_dk = bufs.dk_c2[:, k].to(f64).abs().sum(0) + bufs.dk_d[:, k].to(f64).abs().sum(0)
            qdq = (dg.q_d[:, g0:g1].to(f64) * bufs.dq_d[:, g0:g1].to(f64)).sum()
            kdk = (dg.k_c[:, k].to(f64) * bufs.dk_c2[:, k].to(f64)).sum() + \
                  (dg.k_d[:, k].to(f64) * bufs.dk_d[:, k].to(f64)).sum()
            scale_ref = sum_do.abs().max().item() + 1e-30
            e_dv = (sum_dv - sum_do).abs().max().item() / scale_ref
            e_dk = (sum_dk.abs() / (abs_dk + 1e-30)).max().item()
            qabs = (dg.q_d[:, g0:g1].to(f64) * bufs.dq_d[:, g0:g1].to(f64)).abs().sum().item() + 1e-30
            e_sym = abs(qdq.item() - kdk.item()) / qabs
            # Call 1
            sum_do1 = dg.do_c[:, g0:g1].to(f64).sum(dim=(0, 1))
            e_dv1 = (bufs.dv_c1[:, k].to(f64).sum(0) - sum_do1).abs().max().item() / (sum_do1.abs().max().item() + 1e-30)
            e_dk1 = (bufs.dk_c1[:, k].to(f64).sum(0).abs() / (bufs.dk_c1[:, k].to(f64).abs().sum(0) + 1e-30)).max().item()
            rep.append("kv %d: |sum dV - sum dO|/max=%.2e  |sum dK|/sum|dK|=%.2e  |<q,dq>-<k,dk>|/sum|q dq|=%.2e  "
                       "call1: %.2e %.2e" % (k, e_dv, e_dk, e_sym, e_dv1, e_dk1))
            # every term is a bf16 value (2^-9 relative rounding, unbiased) -> the sums agree far inside 1e-2
            assert e_dv < 1e-2 and e_dk < 1e-2 and e_sym < 1e-2 and e_dv1 < 1e-2 and e_dk1 < 1e-2, rep[-1]

        # ---- 2a. dense upstream gradient: the N x G x R_i-way fp32 sum into each shared prompt key
        if name in DENSE_COLUMN_CONFIGS:
            _say("  dense-gradient key columns (all %d response rows x %d heads of KV head %d)" % (T, G, kv))
            edge = [0, 1, 31, 32, 63, 64, 127, 128, 129, P // 2, P - 129, P - 128, P - 2, P - 1]
            ctx_keys = sorted(set(edge + [int(x) for x in rng.choice(P, size=N_DENSE_CTX_KEYS, replace=False)]))
            dec_keys = set()
            for i in sorted(set([0, shape.n_seqs - 1, int(np.argmax(wl.resp_lens)), int(np.argmin(wl.resp_lens))])):
                R = int(wl.resp_lens[i])
                for j in (0, 1, 31, 32, 127, 128, R // 2, R - 2, R - 1):
                    if 0 <= j < R:
                        dec_keys.add((i, int(j)))
            while len(dec_keys) < N_DENSE_DEC_KEYS:
                i = int(rng.integers(0, shape.n_seqs))
                if wl.resp_lens[i] > 0:
                    dec_keys.add((i, int(rng.integers(0, wl.resp_lens[i]))))
            dec_keys = sorted(dec_keys)
            dk_c, dv_c, dk_dd, dv_dd = orc.key_columns_call2(
                q_d, k_c, v_c, k_d, v_d, cu, wl.scale, do_d, 0, ctx_keys, dec_keys, Wn,
                progress=lambda i: _say("    sequence %d / %d" % (i + 1, shape.n_seqs)) if i % 8 == 7 else None)
            rep.append("dense dO: %d prompt keys and %d response keys of KV head %d, every one of the %d x %d "
                       "(row, head) contributions summed" % (len(ctx_keys), len(dec_keys), kv, T, G))
            PU.compare("dK_c(2)*", PU.to_f64(bufs.dk_c2[ctx_keys, kv]), dk_c, rep)
            PU.compare("dV_c(2)*", PU.to_f64(bufs.dv_c2[ctx_keys, kv]), dv_c, rep)
            didx = [int(cu[i]) + j for (i, j) in dec_keys]
            PU.compare("dK_d*", PU.to_f64(bufs.dk_d[didx, kv]), dk_dd, rep)
            PU.compare("dV_d*", PU.to_f64(bufs.dv_d[didx, kv]), dv_dd, rep)

        # ---- 2b. sparse upstream gradient -> key columns of one KV head
        _say("  sparse-gradient backward")
        srows = _sample_rows(rng, wl, N_SPARSE_ROWS)
        do_sp = torch.zeros_like(dg.do_d)
        idx = torch.tensor([int(cu[i]) + r for (i, r) in srows], device="cuda")
        do_sp[idx] = dg.do_d[idx]
        sprow = sorted(set([0, P - 1] + [int(x) for x in rng.integers(0, P, size=10)]))
        do_spc = torch.zeros_like(dg.do_c)
        pidx = torch.tensor(sprow, device="cuda")
        do_spc[pidx] = dg.do_c[pidx]
        dg2 = B.DeviceGroup(dg.shape_c, dg.q_c, dg.k_c, dg.v_c, dg.q_d, dg.k_d, dg.v_d, do_spc, do_sp, dg.cu_dev,
                            dg.cu_host)
        runner.backward(dg2, bufs)
        torch.cuda.synchronize()
        ctx_keys = sorted(set([0, 1, 63, 64, 127, 128, P - 1, max(0, P - max(Wn, 1))] +
                              [int(x) for x in rng.integers(0, P, size=N_KEY_SAMPLES)]))
        if Wn > 0:   # keys near the end of the prompt are the ones a window can still see
            ctx_keys = sorted(set(ctx_keys + [int(x) for x in rng.integers(max(0, P - Wn), P, size=N_KEY_SAMPLES)]))
        dec_keys = []
        for (i, r) in srows:
            for j in sorted(set([0, r, r // 2, max(0, r - 1), max(0, r - Wn + 1) if Wn else 0])):
                dec_keys.append((i, int(j)))
        dec_keys = sorted(set(dec_keys))
        do_d_sp = np.zeros_like(do_d)
        for (i, r) in srows:
            do_d_sp[int(cu[i]) + r] = do_d[int(cu[i]) + r]
        dk_c, dv_c, dk_dd, dv_dd = orc.key_columns_call2(q_d, k_c, v_c, k_d, v_d, cu, wl.scale, do_d_sp, 0, ctx_keys,
                                                       dec_keys, Wn, rows=srows)
        PU.compare("dK_c(2)", PU.to_f64(bufs.dk_c2[ctx_keys, kv]), dk_c, rep)
        PU.compare("dV_c(2)", PU.to_f64(bufs.dv_c2[ctx_keys, kv]), dv_c, rep)
        didx = [int(cu[i]) + j for (i, j) in dec_keys]
        PU.compare("dK_d", PU.to_f64(bufs.dk_d[didx, kv]), dk_dd, rep)
        PU.compare("dV_d", PU.to_f64(bufs.dv_d[didx, kv]), dv_dd, rep)
        # Call 1: the prompt as a single sequence without a shared prefix
        cu1 = np.array([0, P], dtype=np.int32)
        e = np.zeros((0, 1, d))
        do_c_sp = np.zeros_like(do_c)
        do_c_sp[sprow] = do_c[sprow]
        keys1 = [(0, j) for j in ctx_keys]
        _, _, dk1, dv1 = orc.key_columns_call2(q_c, e, e, k_c, v_c, cu1, wl.scale, do_c_sp, 0, [], keys1, Wn,
                                              rows=[(0, t) for t in sprow])
        PU.compare("dK_c(1)", PU.to_f64(bufs.dk_c1[ctx_keys, kv]), dk1, rep)
        PU.compare("dV_c(1)", PU.to_f64(bufs.dv_c1[ctx_keys, kv]), dv1, rep)
        # keys no sampled row can see must be exactly zero (rows of other sequences carry dO = 0)
        touched = sorted(set(i for (i, _) in srows))
        for i in range(shape.n_seqs):
            if i not in touched and wl.resp_lens[i] > 0:
                assert float(bufs.dk_d[int(cu[i]):int(cu[i + 1])].float().abs().max()) == 0.0
                assert float(bufs.dv_d[int(cu[i]):int(cu[i + 1])].float().abs().max()) == 0.0
                break
    finally:
        _say("[%s full size, kv head %d]\n  " % (name, kv) + "\n  ".join(rep))
