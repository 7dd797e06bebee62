"""Pins of the CPU oracle against things other than itself.

Forward: closed forms and explicit-loop evaluation of the definition.
Backward: central finite differences of L = sum(O * dO) and autograd.
Shared-prompt mapping: finite differences with respect to the single shared
K_c / V_c in the single-prompt layout (so a mistake in the replicate / sum
logic cannot cancel), and the paper's invariants.
"""
import math

import numpy as np
import pytest

from oracle import attention_oracle as orc


def _rand(rng, *shape):
    return rng.standard_normal(shape)


# ---------------------------------------------------------------- forward
def test_zero_keys_give_running_mean_and_log_count():
    # all scores equal -> uniform weights over the visible keys:
    # O_t = mean(V_0..V_t), LSE_t = log(t+1)
    rng = np.random.default_rng(0)
    S, H, Hk, d = 13, 4, 2, 8
    q = _rand(rng, S, H, d)
    k = np.zeros((S, Hk, d))
    v = _rand(rng, S, Hk, d)
    o, lse = orc.attn_fwd_seq(q, k, v, 0.37)
    for t in range(S):
        for h in range(H):
            np.testing.assert_allclose(o[t, h], v[:t + 1, h // 2].mean(axis=0), rtol=1e-13, atol=1e-13)
            assert abs(lse[h, t] - math.log(t + 1)) < 1e-13


def test_zero_keys_window_counts_last_w_keys():
    # window W: exactly min(t+1, W) keys, namely t-W+1..t
    rng = np.random.default_rng(1)
    S, H, Hk, d, W = 17, 2, 1, 4, 5
    q = _rand(rng, S, H, d)
    k = np.zeros((S, Hk, d))
    v = _rand(rng, S, Hk, d)
    o, lse = orc.attn_fwd_seq(q, k, v, 1.0, window=W)
    for t in range(S):
        lo = max(0, t - W + 1)
        np.testing.assert_allclose(o[t, 1], v[lo:t + 1, 0].mean(axis=0), rtol=1e-13, atol=1e-13)
        assert abs(lse[0, t] - math.log(min(t + 1, W))) < 1e-13


def test_two_keys_logistic():
    # row 1 sees two keys: weight on key 1 is the logistic of the score difference
    rng = np.random.default_rng(2)
    d = 6
    q = _rand(rng, 2, 1, d)
    k = _rand(rng, 2, 1, d)
    v = _rand(rng, 2, 1, d)
    scale = 0.8
    o, lse = orc.attn_fwd_seq(q, k, v, scale)
    s0 = scale * float(q[1, 0] @ k[0, 0])
    s1 = scale * float(q[1, 0] @ k[1, 0])
    w1 = 1.0 / (1.0 + math.exp(s0 - s1))
    np.testing.assert_allclose(o[1, 0], (1 - w1) * v[0, 0] + w1 * v[1, 0], rtol=1e-13)
    np.testing.assert_allclose(o[0, 0], v[0, 0], rtol=1e-14)          # row 0 sees only itself
    assert abs(lse[0, 0] - scale * float(q[0, 0] @ k[0, 0])) < 1e-13
    assert abs(lse[0, 1] - (s1 + math.log1p(math.exp(s0 - s1)))) < 1e-13


def test_key_shift_invariance_and_constant_values():
    # adding c to every key adds scale*q.c to every score of a row: O unchanged, LSE shifted
    rng = np.random.default_rng(3)
    S, H, Hk, d = 9, 2, 2, 5
    q, k, v = _rand(rng, S, H, d), _rand(rng, S, Hk, d), _rand(rng, S, Hk, d)
    c = _rand(rng, d)
    o0, l0 = orc.attn_fwd_seq(q, k, v, 0.5)
    o1, l1 = orc.attn_fwd_seq(q, k + c, v, 0.5)
    np.testing.assert_allclose(o1, o0, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(l1 - l0, 0.5 * np.einsum("shd,d->hs", q, c), rtol=1e-11, atol=1e-12)
    vc = np.broadcast_to(_rand(rng, 1, Hk, d), (S, Hk, d)).copy()
    oc, _ = orc.attn_fwd_seq(q, k, vc, 0.5)
    np.testing.assert_allclose(oc, np.broadcast_to(vc[:1], oc.shape), rtol=1e-12, atol=1e-13)


def _loops_fwd(q, k, v, scale, window, G):
    """Definition with explicit Python sums (no matrix products, no masks)."""
    S, H, d = q.shape
    o = np.zeros_like(q)
    lse = np.zeros((H, S))
    for h in range(H):
        kv = h // G
        for t in range(S):
            lo = 0 if not window else max(0, t - window + 1)
            sc = [scale * sum(q[t, h, e] * k[j, kv, e] for e in range(d)) for j in range(lo, t + 1)]
            z = sum(math.exp(x) for x in sc)
            lse[h, t] = math.log(z)
            for e in range(d):
                o[t, h, e] = sum(math.exp(x) / z * v[j, kv, e] for x, j in zip(sc, range(lo, t + 1)))
    return o, lse


@pytest.mark.parametrize("window", [0, 3])
def test_forward_matches_explicit_loops(window):
    rng = np.random.default_rng(4)
    S, H, Hk, d = 7, 4, 2, 3
    q, k, v = _rand(rng, S, H, d), _rand(rng, S, Hk, d), _rand(rng, S, Hk, d)
    o, lse = orc.attn_fwd_seq(q, k, v, 0.6, window)
    o2, lse2 = _loops_fwd(q, k, v, 0.6, window, 2)
    np.testing.assert_allclose(o, o2, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, lse2, rtol=1e-12, atol=1e-13)


def test_gqa_head_map_is_integer_division():
    # make KV head 1 distinguishable: only query heads 2,3 (G=2) may read it
    rng = np.random.default_rng(5)
    S, d = 5, 4
    q = _rand(rng, S, 4, d)
    k = np.zeros((S, 2, d))
    v = np.zeros((S, 2, d))
    v[:, 1, :] = 1.0
    o, _ = orc.attn_fwd_seq(q, k, v, 1.0)
    assert np.all(o[:, :2] == 0.0) and np.allclose(o[:, 2:], 1.0)


# ---------------------------------------------------------------- backward
def _loss(q, k, v, do, scale, window):
    o, _ = orc.attn_fwd_seq(q, k, v, scale, window)
    return float((o * do).sum())


@pytest.mark.parametrize("window", [0, 4])
def test_backward_matches_finite_differences(window):
    rng = np.random.default_rng(6)
    S, H, Hk, d = 9, 4, 2, 4
    q, k, v, do = _rand(rng, S, H, d), _rand(rng, S, Hk, d), _rand(rng, S, Hk, d), _rand(rng, S, H, d)
    scale = 0.7
    dq, dk, dv = orc.attn_bwd_seq(q, k, v, do, scale, window)
    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + eps
            lp = _loss(q, k, v, do, scale, window)
            x[idx] = old - eps
            lm = _loss(q, k, v, do, scale, window)
            x[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        np.testing.assert_allclose(g, num, rtol=2e-6, atol=2e-8, err_msg=name)


@pytest.mark.parametrize("window", [0, 5])
def test_backward_matches_autograd(window):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(7)
    S, H, Hk, d = 19, 6, 2, 8
    G = H // Hk
    q, k, v, do = _rand(rng, S, H, d), _rand(rng, S, Hk, d), _rand(rng, S, Hk, d), _rand(rng, S, H, d)
    scale = 0.3
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    t = torch.arange(S)[:, None]
    j = torch.arange(S)[None, :]
    vis = j <= t
    if window:
        vis = vis & (j > t - window)
    s = torch.einsum("thd,jhd->htj", tq, tk.repeat_interleave(G, dim=1)) * scale
    a = torch.softmax(s.masked_fill(~vis, float("-inf")), dim=-1)
    o = torch.einsum("htj,jhd->thd", a, tv.repeat_interleave(G, dim=1))
    (o * torch.tensor(do)).sum().backward()
    dq, dk, dv = orc.attn_bwd_seq(q, k, v, do, scale, window)
    o_ref, _ = orc.attn_fwd_seq(q, k, v, scale, window)
    np.testing.assert_allclose(o_ref, o.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_zero_upstream_gives_zero_grads_and_rowsum_identities():
    rng = np.random.default_rng(8)
    S, H, Hk, d = 11, 2, 1, 4
    q, k, v, do = _rand(rng, S, H, d), _rand(rng, S, Hk, d), _rand(rng, S, Hk, d), _rand(rng, S, H, d)
    z = orc.attn_bwd_seq(q, k, v, np.zeros_like(do), 0.5)
    assert all(np.all(x == 0) for x in z)
    dq, dk, dv = orc.attn_bwd_seq(q, k, v, do, 0.5)
    # rows of softmax sum to one -> sum_j dV_j = sum_t,h dO_t ; rows of dS sum to zero -> sum_j dK_j = 0
    np.testing.assert_allclose(dv.sum(axis=0)[0], do.sum(axis=(0, 1)), rtol=1e-12)
    np.testing.assert_allclose(dk.sum(axis=0), 0.0, atol=1e-12)
    # scale symmetry q->cq, k->k/c : <q,dq> = <k,dk>
    assert abs((q * dq).sum() - (k * dk).sum()) < 1e-11


# ---------------------------------------------------------------- shared-prompt layout
def _group(rng, P, lens, H, Hk, d):
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    T = int(cu[-1])
    return dict(q_c=_rand(rng, P, H, d), k_c=_rand(rng, P, Hk, d), v_c=_rand(rng, P, Hk, d),
                q_d=_rand(rng, T, H, d), k_d=_rand(rng, T, Hk, d), v_d=_rand(rng, T, Hk, d),
                do_c=_rand(rng, P, H, d), do_d=_rand(rng, T, H, d), cu=cu)


def _loops_call2(g, scale, window, G):
    """Eq. 4 in the single-prompt layout: keys of row r are [K_c ; K_d^(i)[0..r]] -- explicit sums."""
    P = g["q_c"].shape[0]
    cu = g["cu"]
    T, H, d = g["q_d"].shape
    o = np.zeros((T, H, d))
    lse = np.zeros((H, T))
    for i in range(len(cu) - 1):
        for r in range(cu[i + 1] - cu[i]):
            row = cu[i] + r
            t = P + r
            for h in range(H):
                kv = h // G
                keys = [(g["k_c"][j, kv], g["v_c"][j, kv]) for j in range(P)]
                keys += [(g["k_d"][cu[i] + j, kv], g["v_d"][cu[i] + j, kv]) for j in range(r + 1)]
                if window:
                    keys = keys[max(0, t - window + 1):]
                sc = [scale * float(g["q_d"][row, h] @ kk) for kk, _ in keys]
                z = sum(math.exp(x) for x in sc)
                lse[h, row] = math.log(z)
                o[row, h] = sum(math.exp(x) / z * vv for x, (_, vv) in zip(sc, keys))
    return o, lse


@pytest.mark.parametrize("window", [0, 6])
def test_replicated_oracle_equals_two_region_definition(window):
    rng = np.random.default_rng(9)
    H, Hk, d = 4, 2, 3
    g = _group(rng, 5, [3, 1, 4], H, Hk, d)
    f = orc.dualkv_forward(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], g["cu"], 0.9, window)
    o, lse = _loops_call2(g, 0.9, window, H // Hk)
    np.testing.assert_allclose(f["o_d"], o, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(f["lse_d"], lse, rtol=1e-12, atol=1e-13)
    # prompt rows = plain causal attention on the prompt alone (Eq. 3)
    oc, lc = orc.attn_fwd_seq(g["q_c"], g["k_c"], g["v_c"], 0.9, window)
    np.testing.assert_allclose(f["o_c"], oc, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(f["lse_c"], lc, rtol=1e-12, atol=1e-13)
    # sampled-row helpers agree with the dense pass
    for (i, r, h) in [(0, 2, 3), (1, 0, 0), (2, 3, 1)]:
        orow, lrow, _ = orc.response_row(g["q_d"], g["k_c"], g["v_c"], g["k_d"], g["v_d"], g["cu"], 0.9, i, r, h, window)
        np.testing.assert_allclose(orow, o[g["cu"][i] + r, h], rtol=1e-12, atol=1e-13)
        assert abs(lrow - lse[h, g["cu"][i] + r]) < 1e-12


def _packed_loss(g, scale, window):
    """L = <O_c, dO_c> + <O_d, dO_d> evaluated in the single-prompt layout."""
    f = orc.dualkv_forward(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], g["cu"], scale, window)
    return float((f["o_c"] * g["do_c"]).sum() + (f["o_d"] * g["do_d"]).sum())


@pytest.mark.parametrize("window", [0, 5])
def test_shared_prompt_gradients_by_finite_differences(window):
    # total dK_c/dV_c = sum over replicas (gradient-equivalence theorem) checked by perturbing the
    # single shared K_c / V_c, and all other gradients in the packed layout likewise
    rng = np.random.default_rng(10)
    H, Hk, d = 2, 1, 3
    g = _group(rng, 4, [2, 3], H, Hk, d)
    scale = 0.8
    ref = orc.dualkv_reference(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], g["cu"], scale,
                               g["do_c"], g["do_d"], window)
    full = orc.dualkv_backward(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], g["cu"], scale,
                               g["do_c"], g["do_d"], window)
    eps = 1e-6
    want = {"q_c": full["dq_c"], "k_c": ref["total"]["dk_c"], "v_c": ref["total"]["dv_c"],
            "q_d": full["dq_d"], "k_d": full["dk_d"], "v_d": full["dv_d"]}
    for name, gexp in want.items():
        x = g[name]
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + eps
            lp = _packed_loss(g, scale, window)
            x[idx] = old - eps
            lm = _packed_loss(g, scale, window)
            x[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        np.testing.assert_allclose(gexp, num, rtol=5e-6, atol=5e-8, err_msg=name)
    # per-call split adds up (Eq. "dkc-total") and the call-2 part ignores dO_c
    np.testing.assert_allclose(ref["call1"]["dk_c"] + ref["call2"]["dk_c"], full["dk_c"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ref["call2"]["dq_d"], full["dq_d"], rtol=1e-12, atol=1e-13)
    # call 1 alone = plain causal backward on the prompt
    dq1, dk1, dv1 = orc.attn_bwd_seq(g["q_c"], g["k_c"], g["v_c"], g["do_c"], scale, window)
    np.testing.assert_allclose(ref["call1"]["dq_c"], dq1, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ref["call1"]["dk_c"], dk1, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ref["call1"]["dv_c"], dv1, rtol=1e-12, atol=1e-13)


def test_any_split_of_prompt_upstream_gradient_gives_same_total():
    rng = np.random.default_rng(11)
    g = _group(rng, 6, [2, 5, 1], 4, 2, 4)
    args = (g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], g["cu"], 0.5, g["do_c"], g["do_d"])
    a = orc.dualkv_backward(*args, ctx_grad_owner=0)
    b = orc.dualkv_backward(*args, ctx_grad_owner=2)
    c = orc.dualkv_backward(*args, ctx_grad_owner=np.array([0.2, 0.5, 0.3]))
    for key in a:
        np.testing.assert_allclose(a[key], b[key], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(a[key], c[key], rtol=1e-12, atol=1e-12)


def test_degenerate_shapes():
    rng = np.random.default_rng(12)
    # P = 0: plain varlen causal attention per response; R_i = 0 allowed; N = 1
    g = _group(rng, 0, [3, 0, 2], 2, 2, 4)
    f = orc.dualkv_forward(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], g["cu"], 0.5)
    o0, l0 = orc.attn_fwd_seq(g["q_d"][:3], g["k_d"][:3], g["v_d"][:3], 0.5)
    np.testing.assert_allclose(f["o_d"][:3], o0, rtol=1e-13)
    o2, l2 = orc.attn_fwd_seq(g["q_d"][3:], g["k_d"][3:], g["v_d"][3:], 0.5)
    np.testing.assert_allclose(f["o_d"][3:], o2, rtol=1e-13)
    # window >= longest sequence equals no window
    g = _group(rng, 4, [3], 2, 1, 4)
    a = orc.dualkv_forward(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], g["cu"], 0.5, 0)
    b = orc.dualkv_forward(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], g["cu"], 0.5, 7)
    np.testing.assert_allclose(a["o_d"], b["o_d"], rtol=1e-14)


def test_key_column_sampler_matches_dense_backward():
    rng = np.random.default_rng(13)
    H, Hk, d = 4, 2, 4
    g = _group(rng, 7, [4, 6, 2], H, Hk, d)
    for window in (0, 5):
        ref = orc.dualkv_reference(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], g["cu"], 0.6,
                                   g["do_c"], g["do_d"], window)["call2"]
        ctx_keys = [0, 3, 6]
        dec_keys = [(0, 1), (1, 5), (2, 0)]
        dk_c, dv_c, dk_d, dv_d = orc.key_columns_call2(g["q_d"], g["k_c"], g["v_c"], g["k_d"], g["v_d"], g["cu"],
                                                     0.6, g["do_d"], 1, ctx_keys, dec_keys, window)
        np.testing.assert_allclose(dk_c, ref["dk_c"][ctx_keys, 1], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(dv_c, ref["dv_c"][ctx_keys, 1], rtol=1e-11, atol=1e-13)
        for n, (i, j) in enumerate(dec_keys):
            np.testing.assert_allclose(dk_d[n], ref["dk_d"][g["cu"][i] + j, 1], rtol=1e-11, atol=1e-13)
            np.testing.assert_allclose(dv_d[n], ref["dv_d"][g["cu"][i] + j, 1], rtol=1e-11, atol=1e-13)
        # sparse upstream gradient: restricting to the non-zero rows gives the same columns
        do_sparse = np.zeros_like(g["do_d"])
        rows = [(0, 3), (1, 0), (1, 4)]
        for (i, r) in rows:
            do_sparse[g["cu"][i] + r] = g["do_d"][g["cu"][i] + r]
        a = orc.key_columns_call2(g["q_d"], g["k_c"], g["v_c"], g["k_d"], g["v_d"], g["cu"], 0.6, do_sparse, 1,
                                  ctx_keys, dec_keys, window)
        b = orc.key_columns_call2(g["q_d"], g["k_c"], g["v_c"], g["k_d"], g["v_d"], g["cu"], 0.6, do_sparse, 1,
                                  ctx_keys, dec_keys, window, rows=rows)
        for x, y in zip(a, b):
            np.testing.assert_allclose(x, y, rtol=1e-12, atol=1e-14)


def test_row_samplers_give_o_lse_dq():
    """response_row / prompt_row (one query row straight from Eq. 4 / Eq. 3) against the dense replicated pass:
    O, LSE and dQ of every row and head of a small group, with and without a window."""
    rng = np.random.default_rng(14)
    H, Hk, d = 4, 2, 4
    g = _group(rng, 5, [4, 3], H, Hk, d)
    P, cu = 5, g["cu"]
    for window in (0, 4):
        fwd = orc.dualkv_forward(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], cu, 0.6, window)
        full = orc.dualkv_backward(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], cu, 0.6,
                                   g["do_c"], g["do_d"], window)
        for i in range(2):
            for r in range(int(cu[i + 1] - cu[i])):
                for h in range(H):
                    row = cu[i] + r
                    o, lse, dq = orc.response_row(g["q_d"], g["k_c"], g["v_c"], g["k_d"], g["v_d"], cu, 0.6, i, r, h,
                                                  window, do_row=g["do_d"][row, h])
                    np.testing.assert_allclose(o, fwd["o_d"][row, h], rtol=1e-12, atol=1e-14)
                    assert abs(lse - fwd["lse_d"][h, row]) < 1e-12
                    np.testing.assert_allclose(dq, full["dq_d"][row, h], rtol=1e-11, atol=1e-13)
        # prompt rows: the dense pass of the prompt alone (attn_fwd_seq is pinned by closed forms above) ...
        o_c, lse_c = orc.attn_fwd_seq(g["q_c"], g["k_c"], g["v_c"], 0.6, window)
        for t in range(P):
            for h in range(H):
                o, lse, dqc = orc.prompt_row(g["q_c"], g["k_c"], g["v_c"], 0.6, t, h, window, do_row=g["do_c"][t, h])
                np.testing.assert_allclose(o, o_c[t, h], rtol=1e-12, atol=1e-14)
                assert abs(lse - lse_c[h, t]) < 1e-12
                # ... and the prompt rows of the replicated group pass (Sec. 2.2: identical in every replica)
                np.testing.assert_allclose(o, fwd["o_c"][t, h], rtol=1e-12, atol=1e-14)
                assert abs(lse - fwd["lse_c"][h, t]) < 1e-12
                np.testing.assert_allclose(dqc, full["dq_c"][t, h], rtol=1e-11, atol=1e-13)
    # closed form: zero keys -> LSE_t = log(t + 1) (window: log min(t + 1, W)), O_t = mean of the visible values
    kz = np.zeros_like(g["k_c"])
    for t in range(P):
        o, lse, _ = orc.prompt_row(g["q_c"], kz, g["v_c"], 0.6, t, 3)
        assert abs(lse - math.log(t + 1)) < 1e-13
        np.testing.assert_allclose(o, g["v_c"][:t + 1, 1].mean(axis=0), rtol=1e-13)
        o, lse, _ = orc.prompt_row(g["q_c"], kz, g["v_c"], 0.6, t, 0, window=2)
        assert abs(lse - math.log(min(t + 1, 2))) < 1e-13
        np.testing.assert_allclose(o, g["v_c"][max(0, t - 1):t + 1, 0].mean(axis=0), rtol=1e-13)


def test_packings_hand_example():
    """The two packings (Eq. 1 <-> Eq. 5) and their position ids (App. A.2) on a hand-written example:
    P = 3 prompt records a b c, responses of 2, 0 and 1 records (u v | | w)."""
    cu = np.array([0, 2, 2, 3])
    x_c = np.array([[10], [11], [12]])            # a b c
    x_d = np.array([[20], [21], [30]])            # u v w
    rep, cu_rep = orc.replicated_layout(3, cu, x_c, x_d)
    #           seq 0: a b c u v | seq 1: a b c | seq 2: a b c w
    assert rep[:, 0].tolist() == [10, 11, 12, 20, 21, 10, 11, 12, 10, 11, 12, 30]
    assert cu_rep.tolist() == [0, 5, 8, 12]
    assert orc.position_ids_replicated(3, cu).tolist() == [0, 1, 2, 3, 4, 0, 1, 2, 0, 1, 2, 3]
    # single-prompt packing: a b c | u v | | w, every response restarts at position P
    assert orc.single_prompt_layout(3, cu, rep)[:, 0].tolist() == [10, 11, 12, 20, 21, 30]
    assert orc.position_ids_single_prompt(3, cu).tolist() == [0, 1, 2, 3, 4, 3]
    # no prompt: both packings coincide
    rep0, cu0 = orc.replicated_layout(0, cu, x_c[:0], x_d)
    assert rep0[:, 0].tolist() == [20, 21, 30] and cu0.tolist() == [0, 2, 2, 3]
    assert orc.position_ids_replicated(0, cu).tolist() == [0, 1, 0] == orc.position_ids_single_prompt(0, cu).tolist()
    # the position of a response row in the single-prompt packing is the one it has inside its replica
    rng = np.random.default_rng(3)
    for _ in range(10):
        P = int(rng.integers(0, 6))
        lens = rng.integers(0, 5, size=int(rng.integers(1, 5)))
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        pos_rep = orc.position_ids_replicated(P, cu)
        tags_c = np.arange(P)[:, None]
        tags_d = 1000 + np.arange(int(cu[-1]))[:, None]
        rep, _ = orc.replicated_layout(P, cu, tags_c, tags_d)
        pos_sp = orc.position_ids_single_prompt(P, cu)
        sp = orc.single_prompt_layout(P, cu, rep)[:, 0]
        assert sp.tolist() == list(range(P)) + [1000 + x for x in range(int(cu[-1]))]
        for tag, pos in zip(sp, pos_sp):
            assert set(pos_rep[rep[:, 0] == tag].tolist()) == {int(pos)}


# ---------------------------------------------------------------- counting / analytic helpers
def test_pair_counts_by_enumeration():
    P, lens = 5, [3, 0, 4]
    for W in (0, 3, 100):
        def vis(t, j):
            return j <= t and (not W or j > t - W)
        c1 = sum(vis(t, j) for t in range(P) for j in range(P))
        c2 = sum(vis(P + r, j) for R in lens for r in range(R) for j in range(P + R))
        cr = sum(vis(t, j) for R in lens for t in range(P + R) for j in range(P + R))
        assert orc.visible_pairs_call1(P, W) == c1
        assert orc.visible_pairs_call2(P, lens, W) == c2
        assert orc.visible_pairs_replicated(P, lens, W) == cr
        # N-copy = N prompt passes + the response rows
        assert cr == len(lens) * c1 + c2


def test_next_token_pairs_hand_example_and_coverage():
    """The next-token map of the packed layout (Sec. 2.3): a hand-written example, and the property that
    pins it in general: every packed row except row 0 is predicted exactly once, and only the last prompt row
    predicts more than one row (the first token of every non-empty response)."""
    # P = 3, responses of 2, 0 and 1 tokens: packed rows 0 1 2 | 3 4 | | 5
    cu = np.array([0, 2, 2, 3])
    want = {(0, 1), (1, 2), (2, 3), (3, 4), (2, 5)}
    assert orc.next_token_pairs_replicated(3, cu) == want
    rng = np.random.default_rng(11)
    for _ in range(20):
        P = int(rng.integers(1, 9))
        lens = rng.integers(0, 6, size=int(rng.integers(1, 6)))
        cu = np.concatenate([[0], np.cumsum(lens)])
        pairs = orc.next_token_pairs_replicated(P, cu)
        T = P + int(cu[-1])
        targets = sorted(b for _, b in pairs)
        assert targets == list(range(1, T))                      # each row but the first is predicted once
        fan = {}
        for a, b in pairs:
            fan.setdefault(a, []).append(b)
        for a, bs in fan.items():
            if a == P - 1:
                assert sorted(bs) == [P + int(cu[i]) for i in range(len(lens)) if lens[i] > 0]
            else:
                assert bs == [a + 1]
    # no prompt: plain per-sequence shift, nothing predicts a first token
    assert orc.next_token_pairs_replicated(0, np.array([0, 2, 3])) == {(0, 1)}

