"""Closed-form helpers of the paper's analysis.  TEST INFRASTRUCTURE ONLY.

rho (App. C.3, Eq. "rho"), per-layer kernel-level memory savings (App. C.1,
Table "kernel-mem") and packed token counts (Eq. 1 and Eq. 5).
"""


def tokens_standard(N, P, R):
    """Standard packing, Eq. 1: N (P + R) tokens."""
    return N * (P + R)


def tokens_dualkv(N, P, R):
    """Single-prompt packing, Eq. 5: P + N R tokens."""
    return P + N * R


def rho(N, P, R):
    """Token reduction ratio T_std / T_dk."""
    return tokens_standard(N, P, R) / tokens_dualkv(N, P, R)


def rho_limit_large_n(P, R):
    return 1.0 + P / R


def kernel_memory_savings_bytes(N, P, H, Hk, d, bytes_per_el=2):
    """Per-layer tensors an N-copy call would hold N times and DualKV holds once.

    Returns (kv_bytes, q_prompt_bytes, lse_prompt_bytes).
    """
    kv = 2 * (N - 1) * P * Hk * d * bytes_per_el
    qp = (N - 1) * P * H * d * bytes_per_el
    lse = (N - 1) * P * H * 4
    return kv, qp, lse
