"""Closed-form helpers against the numbers the paper prints."""
import os

from oracle import analytic

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_rho_table():
    for N, P, R, printed in _rows("rho_table.txt"):
        assert abs(analytic.rho(int(N), int(P), int(R)) - float(printed)) <= 0.05 + 1e-9
    # limits stated in App. C.3: N -> inf gives 1 + P/R (9x at P=16K, R=2K); P -> inf gives N
    assert analytic.rho_limit_large_n(16384, 2048) == 9.0
    assert abs(analytic.rho(10 ** 9, 16384, 2048) - 9.0) < 1e-4
    assert abs(analytic.rho(16, 10 ** 12, 2048) - 16.0) < 1e-4


def test_kernel_memory_table():
    want = {k: float(v) for k, v in _rows("kernel_memory.txt")}
    kv, qp, lse = analytic.kernel_memory_savings_bytes(8, 16384, 32, 8, 128)
    assert abs(kv / 1e6 - want["kv"]) < 1.0
    assert abs(qp / 1e6 - want["q_prompt"]) < 1.0
    assert abs(lse / 2 ** 20 - want["lse_prompt"]) < 1e-9
    assert want["kv"] + want["q_prompt"] + want["lse_prompt"] == want["total"]


def test_token_counts():
    for N, P, R, std, dk in _rows("token_counts.txt"):
        assert analytic.tokens_standard(int(N), int(P), int(R)) == int(std)
        assert analytic.tokens_dualkv(int(N), int(P), int(R)) == int(dk)
