"""Seeded synthetic workloads for shared-prompt attention.

This module only *generates inputs*: shapes, response lengths, N(0,1) tensors
rounded to bf16 bit patterns.  It holds none of the method's arithmetic and is
the only module used by both the CPU oracle's tests and the HIP path, so both
sides see exactly the same bits.

Layout follows the single-prompt packing (Eq. 5 of the paper): one prompt of
``P`` tokens followed by ``N`` responses of ``R_i`` tokens; ``cu_seqlens`` holds
the (N+1) int32 offsets of the responses inside the packed response tensors.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np


# --------------------------------------------------------------------------
# bf16 bit helpers (storage format only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact up-cast of bf16 bit patterns (uint16) to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


# --------------------------------------------------------------------------
# workload description
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Shape:
    name: str
    n_seqs: int          # N
    ctx_len: int         # P
    resp_lo: int         # R_i drawn uniform in [resp_lo, resp_hi] (inclusive)
    resp_hi: int
    n_q_heads: int       # H
    n_kv_heads: int      # H_k
    head_dim: int        # d
    window: int = 0      # W > 0: sliding window of W keys including self
    seed: int = 0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# The five benchmark shapes (seed 1000+k) and shrunk replicas of configs 2-5 that
# keep H/H_k/d/window/raggedness but divide P and R so a full fp64 oracle pass
# finishes in seconds; odd P and R exercise both partial tiles.
CONFIGS: Dict[str, Shape] = {
    "cfg1_tiny":   Shape("cfg1_tiny", 4, 256, 128, 128, 4, 2, 64, 0, 1001),
    "cfg2_qwen8b": Shape("cfg2_qwen8b", 16, 8192, 1024, 1024, 32, 8, 128, 0, 1002),
    "cfg3_ragged": Shape("cfg3_ragged", 32, 8192, 256, 4096, 32, 8, 128, 0, 1003),
    "cfg4_30b":    Shape("cfg4_30b", 32, 16384, 1024, 8192, 32, 4, 128, 0, 1004),
    "cfg5a_global": Shape("cfg5a_global", 8, 57344, 8192, 8192, 8, 2, 512, 0, 1005),
    "cfg5b_swa":   Shape("cfg5b_swa", 8, 57344, 8192, 8192, 8, 2, 256, 1024, 1006),
    # the (N, P) points of the paper's kernel benchmark (Tab. 1: Qwen3-8B dimensions, R = 2048 throughout);
    # bench-only shapes that place this GPU's numbers beside the paper's
    "tab1_n28_p4k":  Shape("tab1_n28_p4k", 28, 4096, 2048, 2048, 32, 8, 128, 0, 1101),
    "tab1_n28_p16k": Shape("tab1_n28_p16k", 28, 16384, 2048, 2048, 32, 8, 128, 0, 1102),
    "tab1_n16_p32k": Shape("tab1_n16_p32k", 16, 32768, 2048, 2048, 32, 8, 128, 0, 1103),
    "tab1_n16_p64k": Shape("tab1_n16_p64k", 16, 65536, 2048, 2048, 32, 8, 128, 0, 1104),
    # the (P, micro-batch) grid of the paper's single-layer comparison (App. "Comparison with Prefix Grouper":
    # Qwen3-8B dimensions, R ~ U(131, 2048)); bench-only shapes, attention part only
    **{"grid_p%d_mb%d" % (P, mb): Shape("grid_p%d_mb%d" % (P, mb), mb, P, 131, 2048, 32, 8, 128, 0, 1200 + 10 * i + j)
       for i, P in enumerate((5059, 8192, 16384, 32768, 65536, 131072)) for j, mb in enumerate((4, 8, 16, 32))},
    # one mid-size shape per remaining head dim of the supported set (bench-only)
    "dim_d64":  Shape("dim_d64", 8, 16384, 2048, 2048, 32, 8, 64, 0, 1301),
    "dim_d96":  Shape("dim_d96", 8, 16384, 2048, 2048, 16, 4, 96, 0, 1302),
    "dim_d192": Shape("dim_d192", 8, 16384, 2048, 2048, 12, 4, 192, 0, 1303),
    "dim_d256": Shape("dim_d256", 8, 16384, 2048, 2048, 16, 4, 256, 0, 1304),
    # shrunk replicas
    "cfg2_small":  Shape("cfg2_small", 4, 517, 131, 131, 8, 2, 128, 0, 2002),
    "cfg3_small":  Shape("cfg3_small", 6, 509, 17, 260, 8, 2, 128, 0, 2003),
    "cfg4_small":  Shape("cfg4_small", 5, 1021, 60, 500, 8, 1, 128, 0, 2004),
    "cfg5a_small": Shape("cfg5a_small", 3, 701, 257, 257, 4, 2, 512, 0, 2005),
    "cfg5b_small": Shape("cfg5b_small", 3, 701, 300, 300, 4, 2, 256, 96, 2006),
}


@dataclass
class Workload:
    shape: Shape
    resp_lens: np.ndarray            # (N,) int64
    cu_seqlens: np.ndarray           # (N+1,) int32
    scale: float
    # bf16 bit patterns (uint16).  *_c: prompt rows, *_d: packed response rows.
    q_c: np.ndarray
    k_c: np.ndarray
    v_c: np.ndarray
    q_d: np.ndarray
    k_d: np.ndarray
    v_d: np.ndarray
    do_c: np.ndarray
    do_d: np.ndarray
    extra: dict = field(default_factory=dict)

    @property
    def total_resp(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def max_resp(self) -> int:
        return int(self.resp_lens.max()) if len(self.resp_lens) else 0


def response_lengths(shape: Shape) -> np.ndarray:
    rng = np.random.default_rng(shape.seed)
    return rng.integers(shape.resp_lo, shape.resp_hi, endpoint=True,
                        size=shape.n_seqs).astype(np.int64)


def _normal_bf16(seed: int, stream: int, shape) -> np.ndarray:
    """N(0,1) fp32 from an independent substream, rounded to bf16 bits.

    Generated in row chunks so that the fp32 staging copy stays small.
    """
    rng = np.random.default_rng([seed, stream])
    out = np.empty(shape, dtype=np.uint16)
    flat = out.reshape(-1)
    step = 1 << 24
    for s in range(0, flat.size, step):
        e = min(flat.size, s + step)
        flat[s:e] = f32_to_bf16_bits(rng.standard_normal(e - s, dtype=np.float32))
    return out


def make_workload(shape: Shape, resp_lens: Optional[np.ndarray] = None,
                  tensors: bool = True) -> Workload:
    """Build the seeded workload of ``shape``.

    ``tensors=False`` skips the (large) random tensors and returns only the
    length metadata; useful for FLOP accounting.
    """
    if resp_lens is None:
        resp_lens = response_lengths(shape)
    resp_lens = np.asarray(resp_lens, dtype=np.int64)
    cu = np.zeros(shape.n_seqs + 1, dtype=np.int32)
    cu[1:] = np.cumsum(resp_lens)
    P, T = shape.ctx_len, int(cu[-1])
    H, Hk, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    scale = 1.0 / float(np.sqrt(d))
    if not tensors:
        e = np.empty((0,), dtype=np.uint16)
        return Workload(shape, resp_lens, cu, scale, e, e, e, e, e, e, e, e)
    s = shape.seed
    return Workload(
        shape, resp_lens, cu, scale,
        q_c=_normal_bf16(s, 1, (P, H, d)),
        k_c=_normal_bf16(s, 2, (P, Hk, d)),
        v_c=_normal_bf16(s, 3, (P, Hk, d)),
        q_d=_normal_bf16(s, 4, (T, H, d)),
        k_d=_normal_bf16(s, 5, (T, Hk, d)),
        v_d=_normal_bf16(s, 6, (T, Hk, d)),
        do_c=_normal_bf16(s, 7, (P, H, d)),
        do_d=_normal_bf16(s, 8, (T, H, d)),
    )
