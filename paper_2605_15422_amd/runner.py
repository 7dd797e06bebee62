"""Buffer allocation and call sequencing for one shared-prompt attention layer.

Allocates outputs with torch and calls the four C entry points in the order a
training step would (Call 1 fwd, Call 2 fwd, Call 2 bwd, Call 1 bwd).  No
arithmetic happens here.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

from . import binding as B


@dataclass
class LayerBuffers:
    o_c: torch.Tensor
    lse_c: torch.Tensor
    o_d: torch.Tensor
    lse_d: torch.Tensor
    dq_c: torch.Tensor
    dq_d: torch.Tensor
    dk_c1: torch.Tensor      # Call-1 term of dK_c (bf16)
    dv_c1: torch.Tensor
    dk_c2: torch.Tensor      # Call-2 term of dK_c (bf16)
    dv_c2: torch.Tensor
    dk_d: torch.Tensor
    dv_d: torch.Tensor
    ws_ctx_bwd: torch.Tensor
    ws_bwd: torch.Tensor
    dk_c_acc: Optional[torch.Tensor] = None   # fp32 joint accumulators (flag mode)
    dv_c_acc: Optional[torch.Tensor] = None
    dk_c: Optional[torch.Tensor] = None       # bf16 cast of the joint sum
    dv_c: Optional[torch.Tensor] = None


def alloc(dg: B.DeviceGroup, poison: bool = True) -> LayerBuffers:
    dev = dg.q_d.device

    def like(t):
        x = torch.empty_like(t)
        if poison:
            x.view(torch.int16).fill_(0x7FC0)   # bf16 NaN: outputs must be fully overwritten
        return x

    s = dg.shape_c
    P, T, H = s.ctx_len, s.total_resp, s.n_q_heads

    def lse(n):
        return torch.full((H, n), float("nan"), dtype=torch.float32, device=dev)

    def ws(op):
        w = B.workspace(s, op, dev)
        if poison:
            w.fill_(0xFF)                        # scratch must be initialised by the library
        return w

    bufs = LayerBuffers(
        o_c=like(dg.q_c), lse_c=lse(P), o_d=like(dg.q_d), lse_d=lse(T),
        dq_c=like(dg.q_c), dq_d=like(dg.q_d),
        dk_c1=like(dg.k_c), dv_c1=like(dg.v_c), dk_c2=like(dg.k_c), dv_c2=like(dg.v_c),
        dk_d=like(dg.k_d), dv_d=like(dg.v_d),
        ws_ctx_bwd=ws(B.OP_CTX_BWD), ws_bwd=ws(B.OP_BWD))
    if s.flags & B.FLAG_ACCUM_CTX_F32:
        bufs.dk_c_acc = torch.zeros(dg.k_c.shape, dtype=torch.float32, device=dev)
        bufs.dv_c_acc = torch.zeros(dg.v_c.shape, dtype=torch.float32, device=dev)
        bufs.dk_c = like(dg.k_c)
        bufs.dv_c = like(dg.v_c)
    return bufs


def forward(dg: B.DeviceGroup, b: LayerBuffers, call1: bool = True, call2: bool = True) -> None:
    s = dg.shape_c
    if call1:
        B.dualkv_ctx_fwd(s, dg.q_c, dg.k_c, dg.v_c, b.o_c, b.lse_c)
    if call2:
        B.dualkv_fwd(s, dg.q_d, dg.k_c, dg.v_c, dg.k_d, dg.v_d, dg.cu_dev, dg.cu_host, b.o_d, b.lse_d)


def backward(dg: B.DeviceGroup, b: LayerBuffers, call1: bool = True, call2: bool = True) -> None:
    s = dg.shape_c
    acc = bool(s.flags & B.FLAG_ACCUM_CTX_F32)
    if call2:
        B.dualkv_bwd(s, dg.do_d, b.o_d, b.lse_d, dg.q_d, dg.k_c, dg.v_c, dg.k_d, dg.v_d, dg.cu_dev, dg.cu_host,
                     b.dq_d, None if acc else b.dk_c2, None if acc else b.dv_c2, b.dk_d, b.dv_d,
                     b.dk_c_acc, b.dv_c_acc, b.ws_bwd)
    if call1:
        B.dualkv_ctx_bwd(s, dg.do_c, b.o_c, b.lse_c, dg.q_c, dg.k_c, dg.v_c, b.dq_c,
                         None if acc else b.dk_c1, None if acc else b.dv_c1,
                         b.dk_c_acc, b.dv_c_acc, b.ws_ctx_bwd)
    if acc and call1 and call2:
        B.dualkv_finalize_ctx_grads(s, b.dk_c_acc, b.dv_c_acc, b.dk_c, b.dv_c)


def layer_step(dg: B.DeviceGroup, b: LayerBuffers) -> None:
    """One pass of the whole hot path: both forward calls, then both backward calls."""
    forward(dg, b)
    if b.dk_c_acc is not None:
        B.dualkv_zero_ctx_grads(dg.shape_c, b.dk_c_acc, b.dv_c_acc)
    backward(dg, b)
