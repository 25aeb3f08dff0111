"""Operator chains of the three tenant models, as lists of ``lithos_op_t``.

Only plumbing lives here: device buffers (torch), weight layout, and the
order and dtype of every edge.  All arithmetic runs in liblithos kernels.

Edge dtypes (what is stored between two kernels):

* MLP layer        GEMM(+bias+GELU) -> fp32; LayerNorm -> fp32.  The batch is
                   small, so the GEMM is the weight-streaming kind, which
                   reads fp32 activations against bf16 weights.
* encoder layer    QKV GEMM -> bf16; attention -> split bf16; out-proj(+bias+residual) -> fp32;
                   LayerNorm -> fp32 + split bf16; FFN1(+bias+GELU) -> split bf16;
                   FFN2(+bias+residual) -> fp32; LayerNorm -> fp32 + split bf16.
                   "Split bf16" = two bf16 planes hi + lo (~16 significant bits): the
                   MFMA GEMMs multiply both planes with the same weights, so the GEMM
                   inputs carry no coarse rounding that another implementation could
                   round the other way.
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


def norm_colsums(ctx, gamma: torch.Tensor, beta: torch.Tensor, w: torch.Tensor) -> torch.Tensor:
    """[2, N] fp32: the rows gamma and beta multiplied with the [N, K] weight matrix ``w`` by the
    weight-streaming GEMM itself; what a GEMM that layer-normalises its rows on load needs of
    gamma and beta.  Made once per weight matrix (``ctx`` None: in a context of its own)."""
    n, k = w.shape
    gb = torch.stack([gamma, beta]).contiguous()
    out = torch.zeros((2, n), dtype=torch.float32, device=w.device)
    torch.cuda.synchronize()
    own = ctx is None
    if own:
        ctx = B.lithos_init(w.device.index or 0, None)
    try:
        B.lithos_launch_atomized(ctx, B.gemm_op(gb, w, out, 2, n, k, tb=True), (0, 0, 0), 0, None, None)
        B.lithos_partition_sync(ctx, None)
    finally:
        if own:
            B.lithos_shutdown(ctx)
    return out


class MlpChain:
    """h <- LayerNorm(GELU(h W + b)), n_layers times, batch rows.

    Weights are kept [N,K] so that small batches use the weight-streaming
    GEMM; ``tile`` forces an MFMA tile variant (then weights stay [K,N] and
    the LayerNorm output feeding the next GEMM is bf16).  With ``fused``
    (at most 16 rows) a layer's LayerNorm is applied by the
    next layer's GEMM while it loads its rows, so a request is one launch per
    layer plus the last LayerNorm instead of two per layer."""

    def __init__(self, layers, batch: int, device="cuda", tile: int = B.TILE_AUTO, fused: bool = False, ctx=None):
        self.batch = batch
        self.hidden = layers[0]["w"].shape[0]
        self.n_layers = len(layers)
        H, Bn = self.hidden, batch
        self.skinny = tile in (B.TILE_AUTO, B.TILE_SKINNY) and batch <= 32
        self.tile = tile
        self.fused = bool(fused)
        if self.fused and not (self.skinny and batch <= 16):
            raise ValueError("the fused chain is built on the weight-streaming GEMM (at most 16 rows)")
        self.w = [(_wt(L["w"], device) if self.skinny else _dev(L["w"], device)) for L in layers]
        self.b = [_f32(L["b"], device) for L in layers]
        self.gamma = [_f32(L["gamma"], device) for L in layers]
        self.beta = [_f32(L["beta"], device) for L in layers]
        self.x = torch.zeros((Bn, H), dtype=torch.bfloat16, device=device)
        self.act = torch.zeros((Bn, H), dtype=torch.float32, device=device)
        self.act2 = torch.zeros((Bn, H), dtype=torch.float32, device=device) if self.fused else None
        # layer i + 1 normalises with layer i's gamma and beta: their products with layer i + 1's weights
        self.colsums = [norm_colsums(ctx, self.gamma[i], self.beta[i], self.w[i + 1]) for i in range(self.n_layers - 1)] if self.fused else []
        hdt = torch.float32 if self.skinny else torch.bfloat16
        self.h = [torch.zeros((Bn, H), dtype=hdt, device=device) for _ in range(2)]
        self.out = torch.zeros((Bn, H), dtype=torch.float32, device=device)

    def ops(self, x: torch.Tensor = None) -> List[B.Op]:
        """Operator list reading ``x`` (default: the chain's own input buffer)."""
        H, Bn = self.hidden, self.batch
        src = self.x if x is None else x
        ops = []
        if self.fused:
            acts = (self.act, self.act2)
            for i in range(self.n_layers):
                norm = dict(norm_gamma=self.gamma[i - 1], norm_colsums=self.colsums[i - 1]) if i else {}
                ops.append(B.gemm_op(src, self.w[i], acts[i % 2], Bn, H, H, tb=True, bias=self.b[i], gelu=True,
                                     tile=self.tile, op_id=i, **norm))
                src = acts[i % 2]
            ops.append(B.layernorm_op(src, self.gamma[-1], self.beta[-1], self.out, Bn, H, op_id=self.n_layers))
            return ops
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


class EncoderChain:
    """Post-LayerNorm encoder stack (QKV GEMM, full attention, out-proj + residual,
    LayerNorm, FFN with GELU + residual, LayerNorm) on [batch*seq, hidden] tokens.
    The residual stream is fp32; GEMM inputs are split-bf16 pairs (hi + lo planes) of it, the
    packed qkv tensor that attention reads is plain bf16."""

    def __init__(self, layers, batch: int, seq: int = 128, heads: int = 12, device="cuda", tile: int = B.TILE_AUTO):
        self.batch, self.seq, self.heads = batch, seq, heads
        H = layers[0]["w_qkv"].shape[0]
        F = layers[0]["w_1"].shape[1]
        T = batch * seq
        self.H, self.F, self.T, self.tile = H, F, T, tile
        self.d = H // heads
        self.p = []
        for L in layers:
            self.p.append({k: (_dev(v, device) if v.dtype == np.uint16 else _f32(v, device)) for k, v in L.items()})
        bf, f32 = torch.bfloat16, torch.float32
        self.x = torch.zeros((T, H), dtype=f32, device=device)          # input copy
        self.h32 = torch.zeros((T, H), dtype=f32, device=device)        # residual stream
        self.hb = torch.zeros((2, T, H), dtype=bf, device=device)       # hi, lo planes
        self.qkv = torch.zeros((T, 3 * H), dtype=bf, device=device)
        self.att = torch.zeros((2, T, H), dtype=bf, device=device)
        self.r = torch.zeros((T, H), dtype=f32, device=device)
        self.f = torch.zeros((2, T, F), dtype=bf, device=device)
        self.one = torch.ones((H,), dtype=f32, device=device)
        self.zero = torch.zeros((H,), dtype=f32, device=device)
        self.out = self.h32

    def ops(self) -> List[B.Op]:
        T, H, F, t = self.T, self.H, self.F, self.tile
        ops = [
            B.bias_act_op(self.x, self.h32, T, H, None, gelu=False),     # working copy of the input
        ]
        first = True
        for P in self.p:
            if first:      # hi/lo planes of the input hidden states for the first GEMM
                first = False
                ops.append(B.split_op(self.x, self.hb, T, H))
            ops += [
                B.gemm_op(self.hb, P["w_qkv"], self.qkv, T, 3 * H, H, bias=P["b_qkv"], tile=t, a_split=True),
                B.attn_enc_op(self.qkv, self.att, self.batch, self.heads, self.seq, self.d, 1.0 / math.sqrt(self.d), split=True),
                B.gemm_op(self.att, P["w_o"], self.r, T, H, H, bias=P["b_o"], residual=self.h32, tile=t, a_split=True),
                B.layernorm_op(self.r, P["ln1_g"], P["ln1_b"], self.h32, T, H, y_bf16=self.hb, split=True),
                B.gemm_op(self.hb, P["w_1"], self.f, T, F, H, bias=P["b_1"], gelu=True, tile=t, a_split=True, c_split=True),
                B.gemm_op(self.f, P["w_2"], self.r, T, H, F, bias=P["b_2"], residual=self.h32, tile=t, a_split=True),
                B.layernorm_op(self.r, P["ln2_g"], P["ln2_b"], self.h32, T, H, y_bf16=self.hb, split=True),
            ]
        for i, o in enumerate(ops):
            o.op_id = i
        return ops

    def set_input(self, x32: np.ndarray):
        self.x.copy_(torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)))


class DecoderChain:
    """One decode step of a pre-norm grouped-query decoder stack against a bf16
    key/value cache.  All GEMMs are the weight-streaming kind (weights [N,K],
    fp32 activations); the cache slot ``pos`` is rewritten on every step.  With
    ``fused`` (the default for at most 16 sequences) the two RMSNorms run inside
    the GEMMs that consume them and SiLU(gate) * up inside the gate/up GEMM: 7
    launches per layer instead of 10."""

    def __init__(self, layers, kcache_bits, vcache_bits, batch: int, n_q: int, n_kv: int, pos: int, device="cuda",
                 splits: int = 0, fused: bool = None):
        self.batch, self.n_q, self.n_kv, self.pos = batch, n_q, n_kv, pos
        self.fused = batch <= 16 if fused is None else bool(fused)
        if self.fused and batch > 16:
            raise ValueError("the fused decoder step is built on the weight-streaming GEMM (at most 16 rows)")
        # key ranges per (sequence, key/value head): enough workgroups for a few hundred CU slots
        units = (pos + 1 + 31) // 32
        self.splits = splits if splits > 0 else max(1, min(B.ATTN_MAX_SPLITS, units, -(-256 // (batch * n_kv))))
        H = layers[0]["w_qkv"].shape[0]
        self.H = H
        self.d = H // n_q
        self.F = layers[0]["w_d"].shape[0]
        self.cap = pos + 1
        self.w = []
        for L in layers:
            self.w.append(dict(rms1=_f32(L["rms1"], device), rms2=_f32(L["rms2"], device),
                               w_qkv=_wt(L["w_qkv"], device), w_o=_wt(L["w_o"], device),
                               w_gu=_wt(L["w_gu"], device), w_d=_wt(L["w_d"], device)))
        self.kc, self.vc = [], []
        for kb, vb in zip(kcache_bits, vcache_bits):
            for src, dst in ((kb, self.kc), (vb, self.vc)):
                c = torch.zeros((batch, self.cap, n_kv, self.d), dtype=torch.bfloat16, device=device)
                c[:, :pos].copy_(bits_to_torch(src))
                dst.append(c)
        f32 = torch.float32
        nqkv = (n_q + 2 * n_kv) * self.d
        self.x_in = torch.zeros((batch, H), dtype=f32, device=device)
        self.x = torch.zeros((batch, H), dtype=f32, device=device)
        self.n = torch.zeros((batch, H), dtype=f32, device=device)
        self.qkv = torch.zeros((batch, nqkv), dtype=f32, device=device)
        self.att = torch.zeros((batch, n_q * self.d), dtype=f32, device=device)
        self.ws = torch.zeros(B.attn_workspace_floats(batch, n_q, self.d, self.splits), dtype=f32, device=device)
        self.gu = torch.zeros((batch, 2 * self.F), dtype=f32, device=device)
        self.act = torch.zeros((batch, self.F), dtype=f32, device=device)
        self.out = self.x

    def ops(self) -> List[B.Op]:
        Bn, H, F, d, n_q, n_kv = self.batch, self.H, self.F, self.d, self.n_q, self.n_kv
        nqkv = (n_q + 2 * n_kv) * d
        ops = [B.bias_act_op(self.x_in, self.x, Bn, H, None, gelu=False)]      # working copy of the input
        S = self.splits
        for li, W in enumerate(self.w):
            if self.fused:
                ops.append(B.gemm_op(self.x, W["w_qkv"], self.qkv, Bn, nqkv, H, tb=True, norm_gamma=W["rms1"]))
            else:
                ops += [B.rmsnorm_op(self.x, W["rms1"], self.n, Bn, H),
                        B.gemm_op(self.n, W["w_qkv"], self.qkv, Bn, nqkv, H, tb=True)]
            ops += [
                B.rope_kv_op(self.qkv, self.kc[li], self.vc[li], Bn, n_q, n_kv, d, self.pos, self.cap),
                B.attn_dec_op(self.qkv, self.kc[li], self.vc[li], self.att, Bn, n_q, n_kv, d, self.pos + 1, self.cap,
                              1.0 / math.sqrt(d), ldq=nqkv, splits=S, workspace=self.ws if S > 1 else None),
            ]
            if S > 1:
                ops.append(B.attn_merge_op(self.ws, self.att, Bn, n_q, n_kv, d, S))
            ops.append(B.gemm_op(self.att, W["w_o"], self.x, Bn, H, n_q * d, tb=True, residual=self.x))
            if self.fused:
                ops.append(B.gemm_op(self.x, W["w_gu"], self.act, Bn, F, H, tb=True, norm_gamma=W["rms2"], glu=True))
            else:
                ops += [B.rmsnorm_op(self.x, W["rms2"], self.n, Bn, H),
                        B.gemm_op(self.n, W["w_gu"], self.gu, Bn, 2 * F, H, tb=True),
                        B.silu_mul_op(self.gu, self.act, Bn, F)]
            ops.append(B.gemm_op(self.act, W["w_d"], self.x, Bn, H, F, tb=True, residual=self.x))
        for i, o in enumerate(ops):
            o.op_id = i
        return ops

    def set_input(self, x32: np.ndarray):
        self.x_in.copy_(torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)))


def training_block_ops(n_layers=24, hidden=1024, ffn=4096, tokens=16384, split_cus=192):
    """Forward and backward GEMMs (Y = XW, dX = dY W^T, dW = X^T dY) of a transformer block stack."""
    dev, bf = "cuda", torch.bfloat16
    from . import inputs
    shapes = [("qkv", hidden, 3 * hidden), ("out", hidden, hidden), ("ffn1", hidden, ffn), ("ffn2", ffn, hidden)]
    x = {k: inputs.bits_to_torch(inputs.normal_bits((tokens, k), [12, k]), dev) for k in {s[1] for s in shapes}}
    dy = {n: inputs.bits_to_torch(inputs.normal_bits((tokens, n), [13, n]), dev) for n in {s[2] for s in shapes}}
    y = {n: torch.empty((tokens, n), dtype=bf, device=dev) for n in {s[2] for s in shapes}}
    dx = {k: torch.empty((tokens, k), dtype=bf, device=dev) for k in {s[1] for s in shapes}}
    ops, flop, keep, distinct = [], 0.0, [x, dy, y, dx], {}
    planes = None       # fp32 partial planes of the K-sliced weight gradients (one buffer: the queue is in order)
    for layer in range(n_layers):
        for name, k, n in shapes:
            w = inputs.bits_to_torch(inputs.normal_bits((k, n), [14, layer, k, n], 0.02), dev)
            dw = torch.empty((k, n), dtype=bf, device=dev)
            keep += [w, dw]
            trio = [B.gemm_op(x[k], w, y[n], tokens, n, k),                       # Y  = X W
                    B.gemm_op(dy[n], w, dx[k], tokens, k, n, tb=True),            # dX = dY W^T
                    B.gemm_op(x[k], dy[n], dw, k, n, tokens, ta=True)]            # dW = X^T dY
            # few output tiles, K = tokens: cut K so that every CU of the partition gets a tile
            tile, slices = B.lithos_gemm_split_hint(trio[2], split_cus)
            extra = []
            if slices > 1:
                if planes is None or planes.numel() < slices * k * n:     # grows during the first layer only
                    planes = torch.empty(slices * k * n, dtype=torch.float32, device=dev)
                    keep.append(planes)
                trio[2] = B.gemm_op(x[k], dy[n], planes, k, n, tokens, ta=True, tile=tile, k_slices=slices)
                extra = [B.sum_slices_op(planes, dw, k, n, slices)]
            ops += trio + extra
            flop += 3 * 2.0 * tokens * k * n
            if layer == 0:
                for kind, o in zip(("fwd", "dX", "dW"), trio):
                    distinct["be_%s_%s" % (name, kind)] = (o, 2.0 * tokens * k * n)
                if extra:
                    distinct["be_%s_dW_sum" % name] = (extra[0], 0.0)
    return ops, flop, keep, distinct
