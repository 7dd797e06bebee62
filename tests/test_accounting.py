"""Pair / FLOP accounting of the product package against enumeration and the oracle's own counters."""
import numpy as np

from oracle import attention_oracle as orc
from paper_2605_15422_amd import accounting as acc
from paper_2605_15422_amd import workloads as W


def test_pairs_match_enumeration_and_oracle():
    rng = np.random.default_rng(0)
    for _ in range(40):
        P = int(rng.integers(0, 40))
        lens = rng.integers(0, 30, size=int(rng.integers(1, 5)))
        Wn = int(rng.choice([0, 1, 3, 17, 100]))
        assert acc.pairs_call1(P, Wn) == orc.visible_pairs_call1(P, Wn)
        assert acc.pairs_call2(P, lens, Wn) == orc.visible_pairs_call2(P, lens, Wn)
        assert acc.pairs_ncopy(P, lens, Wn) == orc.visible_pairs_replicated(P, lens, Wn)


def test_config2_flops():
    s = W.CONFIGS["cfg2_qwen8b"]
    f = acc.layer_flops(s, W.response_lengths(s))
    # 16 x 1024 rows see 8192 prompt keys plus a causal triangle of 1024
    assert f["pairs_call2"] == 16 * (1024 * 8192 + 1024 * 1025 // 2)
    assert f["pairs_call1"] == 8192 * 8193 // 2
    assert abs(f["layer"] / 1e12 - 10.1) < 0.05 and abs(f["ncopy"] / 1e12 - 39.0) < 0.05
