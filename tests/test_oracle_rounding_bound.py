"""Pin of oracle/rounding_bound.py: a numpy emulation of a machine that rounds to bf16 exactly where the FA2 lineage
does (P and dS as matrix operands, the stored O, every stored output; everything else fp64) must stay inside the
bound on every element, and must come within a modest factor of it somewhere, so the bound is neither unsound nor
vacuous.  A dropped term shows: without the D term the dS-fed gradients of rows with large |dO.O| break the
bound; without the scale factor dQ / dK break it (scale > 1 below); without the output term dV breaks it.
"""
import numpy as np
import pytest

from oracle import attention_oracle as orc
from oracle import rounding_bound as rb


def bf16(x):
    """Round fp64 -> bf16 (nearest even) -> fp64."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    u = x32.view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return (((u + r) >> 16) << 16).astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


def machine_seq(q, k, v, do, scale, window=0):
    """Causal attention forward + backward of one sequence with bf16 rounding at the FA2 places."""
    S, H, d = q.shape
    Hk = k.shape[1]
    G = H // Hk
    vis = orc.visibility(S, window)
    o = np.zeros_like(q)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for h in range(H):
        kv = h // G
        s = np.where(vis, scale * (q[:, h] @ k[:, kv].T), -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        l = e.sum(axis=1, keepdims=True)
        # forward: un-normalised P rounded for the product, normalised at the end, O stored as bf16
        o[:, h] = bf16((bf16(e) @ v[:, kv]) / l)
        a = e / l
        dv[:, kv] += bf16(a).T @ do[:, h]
        dp = do[:, h] @ v[:, kv].T
        dd = (do[:, h] * o[:, h]).sum(axis=1, keepdims=True)       # from the stored O
        ds = bf16(a * (dp - dd))
        dq[:, h] = bf16(scale * (ds @ k[:, kv]))
        dk[:, kv] += scale * (ds.T @ q[:, h])
    return o, dq, bf16(dk), bf16(dv)


@pytest.mark.parametrize("window", [0, 5])
@pytest.mark.parametrize("scale", [0.3, 1.7])
def test_bound_holds_and_is_not_vacuous(window, scale):
    rng = np.random.default_rng(100 + window)
    worst = {}
    for trial in range(6):
        S, H, Hk, d = int(rng.integers(3, 40)), 4, 2, 8
        q, k, v, do = (bf16(rng.standard_normal(s)) for s in ((S, H, d), (S, Hk, d), (S, Hk, d), (S, H, d)))
        if trial % 2:      # large |dO . O|: the D term dominates the error of dS
            do = bf16(do + 3.0 * np.sign(v[:, np.arange(H) // 2]))
        o, dq, dk, dv = machine_seq(q, k, v, do, scale, window)
        o_ref, _ = orc.attn_fwd_seq(q, k, v, scale, window)
        dq_ref, dk_ref, dv_ref = orc.attn_bwd_seq(q, k, v, do, scale, window)
        b = rb.bounds_seq(q, k, v, do, scale, window)
        for name, got, ref in (("o", o, o_ref), ("dq", dq, dq_ref), ("dk", dk, dk_ref), ("dv", dv, dv_ref)):
            err = np.abs(got - ref)
            assert (err <= 1.02 * b[name] + 1e-12).all(), (name, trial, float((err - b[name]).max()))
            worst[name] = max(worst.get(name, 0.0), float((err / (b[name] + 1e-300)).max()))
    # somewhere the machine uses at least a fifth of the allowance (worst-case bounds of random rounding errors)
    for name, w in worst.items():
        assert w > 0.2, (name, w)


def test_group_bounds_follow_the_reference_layout():
    """dualkv_bounds: same keys and shapes as dualkv_reference; the shared-prompt bounds are the sums over the
    replicas (errors of the N contributions add at worst), and the fp32 totals carry no output-rounding term."""
    rng = np.random.default_rng(7)
    H, Hk, d, P = 4, 2, 4, 5
    cu = np.array([0, 3, 3, 7])
    T = 7
    g = {n: bf16(rng.standard_normal(s)) for n, s in (("q_c", (P, H, d)), ("k_c", (P, Hk, d)), ("v_c", (P, Hk, d)),
                                                     ("q_d", (T, H, d)), ("k_d", (T, Hk, d)), ("v_d", (T, Hk, d)),
                                                     ("do_c", (P, H, d)), ("do_d", (T, H, d)))}
    b, ref = rb.dualkv_bounds(g["q_c"], g["k_c"], g["v_c"], g["q_d"], g["k_d"], g["v_d"], cu, 0.6, g["do_c"], g["do_d"])
    for call in ("call1", "call2", "total"):
        for n, x in ref[call].items():
            assert b[call][n].shape == x.shape and (b[call][n] >= 0).all()
    # machine on each replica, prompt gradients summed in fp64 then rounded once: inside the `total` bound
    dk_c = np.zeros((P, Hk, d))
    dv_c = np.zeros((P, Hk, d))
    for i in range(3):
        do = np.concatenate([g["do_c"] if i == 0 else np.zeros_like(g["do_c"]), g["do_d"][cu[i]:cu[i + 1]]])
        S = P + cu[i + 1] - cu[i]
        q, k, v = (orc.replicate(P, cu, g[a], g[c], i) for a, c in (("q_c", "q_d"), ("k_c", "k_d"), ("v_c", "v_d")))
        # un-rounded outputs of the machine: recompute dk, dv without the final cast
        vis = orc.visibility(S)
        for h in range(H):
            kv = h // 2
            s = np.where(vis, 0.6 * (q[:, h] @ k[:, kv].T), -np.inf)
            e = np.exp(s - s.max(axis=1, keepdims=True))
            l = e.sum(axis=1, keepdims=True)
            o = bf16((bf16(e) @ v[:, kv]) / l)
            a = e / l
            dp = do[:, h] @ v[:, kv].T
            ds = bf16(a * (dp - (do[:, h] * o).sum(axis=1, keepdims=True)))
            dk_c[:, kv] += (0.6 * (ds.T @ q[:, h]))[:P]
            dv_c[:, kv] += (bf16(a).T @ do[:, h])[:P]
    assert (np.abs(dk_c - ref["total"]["dk_c"]) <= 1.02 * b["total32"]["dk_c"] + 1e-12).all()
    assert (np.abs(dv_c - ref["total"]["dv_c"]) <= 1.02 * b["total32"]["dv_c"] + 1e-12).all()
    assert (np.abs(bf16(dk_c) - ref["total"]["dk_c"]) <= 1.02 * b["total"]["dk_c"] + 1e-12).all()
    assert (b["total"]["dk_c"] >= b["total32"]["dk_c"]).all()
