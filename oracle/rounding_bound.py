"""First-order worst-case bound on what bf16 operand rounding can do to attention outputs.  TEST INFRASTRUCTURE ONLY.

The paper computes "in the FA2 lineage" (Sec. 3): the probabilities P and the score gradients dS enter their
second matrix products as bf16 values, the products accumulate in fp32, D = rowsum(dO * O) is formed from the
stored bf16 O (Alg. 1 "Require"), and every output is stored as bf16.  The dense fp64 oracle ignores all of this.
This module bounds, element by element and from the exact fp64 quantities, how far a machine that rounds at
exactly those places can land from the exact result, with unit roundoff u = 2^-8 (bf16 keeps 8 significant
bits, round to nearest):

  stored O      |dO_c|    <= u * sum_j a_j |V_jc|            (P rounded)        + u |O_c|      (output rounded)
  D             |dD|      <= sum_c |dO_c| |dO_c-bound|
  dV_jc         <= u * sum_r a_rj |dO_rc|                     (P rounded)        + u |dV_jc|
  dS_rj (value fed to the products)
                |ddS_rj|  <= a_rj |dD_r| + u (|dS_rj| + a_rj |dD_r|)             (D error, then dS rounded)
  dQ_rc         <= scale * sum_j |ddS_rj| |K_jc|                                 + u |dQ_rc|
  dK_jc         <= scale * sum_r |ddS_rj| |Q_rc|                                 + u |dK_jc|

(a = softmax probabilities, sums over visible pairs; fp32 accumulation and the fp32 exponential add terms of
relative size 2^-20 and below, covered by the slack factor the tests apply.)  An error above this bound cannot be
explained by operand rounding: it is a defect.  The bound is a sum of absolute values, so it grows with the number
of summed terms times their magnitude, e.g. for a one-token prompt whose dK_c sums thousands of rows.

Pinned in tests/test_oracle_rounding_bound.py by a numpy emulation of such a machine (round P, dS, O and the
outputs to bf16 at those places, everything else fp64): its error must stay inside the bound on every element,
and must reach a fair fraction of it somewhere (the bound is not vacuous).
"""
from __future__ import annotations

import numpy as np

from . import attention_oracle as orc

U_BF16 = 2.0 ** -8


def bounds_seq(q, k, v, do, scale, window=0, u=U_BF16, round_outputs=True):
    """Bounds for one sequence (dense).  q, do: (S, H, d); k, v: (S, H_k, d).

    Returns dict(o, dq: (S, H, d); dk, dv: (S, H_k, d)) of non-negative bounds on |machine - exact|.
    dk / dv sum the bounds of the G query heads of a group (their errors add at worst).
    """
    S, H, d = q.shape
    Hk = k.shape[1]
    G = H // Hk
    bo = np.zeros_like(q)
    bdq = np.zeros_like(q)
    bdk = np.zeros_like(k)
    bdv = np.zeros_like(v)
    if S == 0:
        return dict(o=bo, dq=bdq, dk=bdk, dv=bdv)
    vis = orc.visibility(S, window)
    uo = u if round_outputs else 0.0
    for h in range(H):
        kv = h // G
        s = np.where(vis, scale * (q[:, h, :] @ k[:, kv, :].T), -np.inf)
        a = np.exp(s - s.max(axis=1, keepdims=True))
        a /= a.sum(axis=1, keepdims=True)
        o = a @ v[:, kv, :]
        # the stored O always is a rounded bf16 value, whatever the caller does with the gradients
        bo[:, h, :] = u * (a @ np.abs(v[:, kv, :])) + u * np.abs(o)
        b_d = (np.abs(do[:, h, :]) * bo[:, h, :]).sum(axis=1, keepdims=True)
        dp = do[:, h, :] @ v[:, kv, :].T
        ds = a * (dp - (a * dp).sum(axis=1, keepdims=True))
        b_ds = a * b_d + u * (np.abs(ds) + a * b_d)
        dq = scale * (ds @ k[:, kv, :])
        bdq[:, h, :] = scale * (b_ds @ np.abs(k[:, kv, :])) + uo * np.abs(dq)
        bdk[:, kv, :] += scale * (b_ds.T @ np.abs(q[:, h, :]))
        bdv[:, kv, :] += u * (a.T @ np.abs(do[:, h, :]))
    if round_outputs:
        _, dk, dv = orc.attn_bwd_seq(q, k, v, do, scale, window)
        bdk += u * np.abs(dk)
        bdv += u * np.abs(dv)
    return dict(o=bo, dq=bdq, dk=bdk, dv=bdv)


def dualkv_bounds(q_c, k_c, v_c, q_d, k_d, v_d, cu, scale, do_c, do_d, window=0, u=U_BF16):
    """Bounds for everything the four entry points return, laid out like attention_oracle.dualkv_reference.

    ``call1`` / ``call2``: bf16 outputs of each backward call; ``total32``: the fp32 joint accumulators of dK_c, dV_c
    (no output rounding); ``total``: their single bf16 cast.
    """
    P = q_c.shape[0]
    N = len(cu) - 1
    z_c, z_d = np.zeros_like(do_c), np.zeros_like(do_d)

    def run(doc, dod, round_outputs):
        out = dict(o_c=None, o_d=np.zeros_like(q_d), dq_c=np.zeros_like(q_c), dq_d=np.zeros_like(q_d),
                   dk_c=np.zeros_like(k_c), dv_c=np.zeros_like(v_c), dk_d=np.zeros_like(k_d), dv_d=np.zeros_like(v_d))
        for i in range(N):
            w = 1.0 if i == 0 else 0.0
            do = np.concatenate([w * doc[:P], dod[cu[i]:cu[i + 1]]], axis=0)
            b = bounds_seq(orc.replicate(P, cu, q_c, q_d, i), orc.replicate(P, cu, k_c, k_d, i),
                           orc.replicate(P, cu, v_c, v_d, i), do, scale, window, u, round_outputs=False)
            if out["o_c"] is None:
                out["o_c"] = b["o"][:P].copy()
            out["o_d"][cu[i]:cu[i + 1]] = b["o"][P:]
            out["dq_c"] += b["dq"][:P]
            out["dq_d"][cu[i]:cu[i + 1]] = b["dq"][P:]
            out["dk_c"] += b["dk"][:P]
            out["dv_c"] += b["dv"][:P]
            out["dk_d"][cu[i]:cu[i + 1]] = b["dk"][P:]
            out["dv_d"][cu[i]:cu[i + 1]] = b["dv"][P:]
        return out

    b1 = run(do_c, z_d, False)
    b2 = run(z_c, do_d, False)
    ref = orc.dualkv_reference(q_c, k_c, v_c, q_d, k_d, v_d, cu, scale, do_c, do_d, window)

    def rnd(bound, exact):          # output stored as bf16
        return bound + u * np.abs(exact)

    out = dict(o_c=b1["o_c"] if b1["o_c"] is not None else np.zeros_like(q_c), o_d=b2["o_d"])
    out["call1"] = dict(dq_c=rnd(b1["dq_c"], ref["call1"]["dq_c"]), dk_c=rnd(b1["dk_c"], ref["call1"]["dk_c"]),
                        dv_c=rnd(b1["dv_c"], ref["call1"]["dv_c"]))
    out["call2"] = dict(dq_d=rnd(b2["dq_d"], ref["call2"]["dq_d"]), dk_c=rnd(b2["dk_c"], ref["call2"]["dk_c"]),
                        dv_c=rnd(b2["dv_c"], ref["call2"]["dv_c"]), dk_d=rnd(b2["dk_d"], ref["call2"]["dk_d"]),
                        dv_d=rnd(b2["dv_d"], ref["call2"]["dv_d"]))
    out["total32"] = dict(dk_c=b1["dk_c"] + b2["dk_c"], dv_c=b1["dv_c"] + b2["dv_c"])
    out["total"] = dict(dk_c=rnd(out["total32"]["dk_c"], ref["total"]["dk_c"]),
                        dv_c=rnd(out["total32"]["dv_c"], ref["total"]["dv_c"]))
    return out, ref
