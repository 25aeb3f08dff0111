"""Operator chains of the three tenant models, as lists of ``lithos_op_t``.

Only plumbing lives here: device buffers (torch), weight layout, and the
order and dtype of every edge.  All arithmetic runs in liblithos kernels.

Edge dtypes (what is stored between two kernels):

* MLP layer        GEMM(+bias+GELU) -> fp32; LayerNorm -> fp32.  The batch is
                   small, so the GEMM is the weight-streaming kind, which
                   reads fp32 activations against bf16 weights.
* encoder layer    QKV GEMM -> bf16; attention -> bf16; out-proj(+bias+residual) -> fp32;
                   LayerNorm -> fp32 + bf16 copy; FFN1(+bias+GELU) -> bf16;
                   FFN2(+bias+residual) -> fp32; LayerNorm -> fp32 + bf16 copy
* decoder layer    every edge fp32 (weight-streaming GEMMs), except the
                   key/value cache, which is bf16: the current token's rotated
                   key and its value are rounded when appended.
"""
from __future__ import annotations

import math
from typing import List

import numpy as np
import torch

from . import binding as B
from .inputs import bits_to_torch


def _dev(bits: np.ndarray, device) -> torch.Tensor:
    return bits_to_torch(bits, device).contiguous()


def _f32(a: np.ndarray, device) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def _wt(bits: np.ndarray, device) -> torch.Tensor:
    """[K,N] weight bits -> device tensor stored [N,K] (TRANS_B layout)."""
    return bits_to_torch(np.ascontiguousarray(bits.T), device).contiguous()


class MlpChain:
    """h <- LayerNorm(GELU(h W + b)), n_layers times, batch rows.

    Weights are kept [N,K] so that small batches use the weight-streaming
    GEMM; ``tile`` forces an MFMA tile variant (then weights stay [K,N] and
    the LayerNorm output feeding the next GEMM is bf16)."""

    def __init__(self, layers, batch: int, device="cuda", tile: int = B.TILE_AUTO):
        self.batch = batch
        self.hidden = layers[0]["w"].shape[0]
        self.n_layers = len(layers)
        H, Bn = self.hidden, batch
        self.skinny = tile in (B.TILE_AUTO, B.TILE_SKINNY) and batch <= 32
        self.tile = tile
        self.w = [(_wt(L["w"], device) if self.skinny else _dev(L["w"], device)) for L in layers]
        self.b = [_f32(L["b"], device) for L in layers]
        self.gamma = [_f32(L["gamma"], device) for L in layers]
        self.beta = [_f32(L["beta"], device) for L in layers]
        self.x = torch.zeros((Bn, H), dtype=torch.bfloat16, device=device)
        self.act = torch.zeros((Bn, H), dtype=torch.float32, device=device)
        hdt = torch.float32 if self.skinny else torch.bfloat16
        self.h = [torch.zeros((Bn, H), dtype=hdt, device=device) for _ in range(2)]
        self.out = torch.zeros((Bn, H), dtype=torch.float32, device=device)

    def ops(self, x: torch.Tensor = None) -> List[B.Op]:
        """Operator list reading ``x`` (default: the chain's own input buffer)."""
        H, Bn = self.hidden, self.batch
        src = self.x if x is None else x
        ops = []
        for i in range(self.n_layers):
            ops.append(B.gemm_op(src, self.w[i], self.act, Bn, H, H, tb=self.skinny, bias=self.b[i], gelu=True,
                                 tile=self.tile, op_id=2 * i))
            last = i + 1 == self.n_layers
            dst = self.out if last else self.h[i % 2]
            ops.append(B.layernorm_op(self.act, self.gamma[i], self.beta[i], dst, Bn, H, op_id=2 * i + 1))
            src = dst
        return ops

    def set_input(self, x_bits: np.ndarray):
        self.x.copy_(bits_to_torch(x_bits))


def run_ops(ctx, ops, part=None, atom_blocks=0):
    """Launch a chain's operators in order on one partition and wait.

    torch's own work (fills, copies) runs on torch's stream, the library's on
    its CU-masked queues: torch is drained first so the two cannot race."""
    torch.cuda.synchronize()
    for op in ops:
        B.lithos_launch_atomized(ctx, op, (0, 0, 0), atom_blocks, part, None)
    B.lithos_partition_sync(ctx, part)
