"""FLOP / byte accounting of the hot path (host arithmetic on lengths only).

Algorithmic work per visible (query, key) pair and query head: forward 4 d
(Q K^T and P V), backward 10 d (S recompute, dV, dP, dQ, dK); visible pairs are
counted exactly from the sequence lengths (the paper's approximate speedup
formula, App. C.2, is not used).
"""
from __future__ import annotations


def _causal_pairs(n_rows: int, first_pos: int, window: int) -> int:
    """Sum over rows t = first_pos .. first_pos+n_rows-1 of min(t+1, window or inf)."""
    if n_rows <= 0:
        return 0
    lo, hi = first_pos + 1, first_pos + n_rows           # keys seen by first / last row without window
    if window and window > 0:
        if lo >= window:
            return n_rows * window
        if hi <= window:
            return (lo + hi) * n_rows // 2
        k = window - lo                                   # rows below the window size
        return (lo + window - 1) * k // 2 + (n_rows - k) * window
    return (lo + hi) * n_rows // 2


def pairs_call1(P: int, window: int = 0) -> int:
    return _causal_pairs(P, 0, window)


def pairs_call2(P: int, resp_lens, window: int = 0) -> int:
    return sum(_causal_pairs(int(R), P, window) for R in resp_lens)


def pairs_ncopy(P: int, resp_lens, window: int = 0) -> int:
    return sum(_causal_pairs(P + int(R), 0, window) for R in resp_lens)


def flops_fwd(pairs: int, H: int, d: int) -> int:
    return 4 * d * pairs * H


def flops_bwd(pairs: int, H: int, d: int) -> int:
    return 10 * d * pairs * H


def layer_flops(shape, resp_lens):
    """Dict of algorithmic flops of the four entry points and of the N-copy baseline."""
    P, H, d, W = shape.ctx_len, shape.n_q_heads, shape.head_dim, shape.window
    p1, p2, pn = pairs_call1(P, W), pairs_call2(P, resp_lens, W), pairs_ncopy(P, resp_lens, W)
    return dict(pairs_call1=p1, pairs_call2=p2, pairs_ncopy=pn,
                ctx_fwd=flops_fwd(p1, H, d), ctx_bwd=flops_bwd(p1, H, d),
                fwd=flops_fwd(p2, H, d), bwd=flops_bwd(p2, H, d),
                layer=14 * d * H * (p1 + p2), ncopy=14 * d * H * pn)
