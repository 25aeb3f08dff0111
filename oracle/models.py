"""CPU oracle for the three operator chains the tenants run.

TEST INFRASTRUCTURE ONLY.  Built from the single-operator oracles in
``ops.py``; all arithmetic between two tensors that the GPU graph stores is
fp64, and the oracle rounds to bf16 exactly on the edges where the GPU graph
stores a bf16 tensor (marked ``# bf16 edge``).  fp32 edges are not rounded
(2^-24 relative is far below every tolerance used).

The paper (LithOS) does not define these models; it only runs such models as
tenants (Sections 6 and 7.1).  The shapes are the benchmark configurations:
a GEMM+bias+GELU+LayerNorm MLP, a post-LayerNorm encoder layer stack with
full attention, and a pre-norm grouped-query decoder layer stack decoding one
token against a key/value cache.

Parameters arrive as dicts of numpy arrays: GEMM weights are bf16 bit
patterns (uint16) stored [K, N]; vectors (bias, norm scale/shift) are fp32.
"""
from __future__ import annotations

import math
import numpy as np

from . import ops


def _bits(x64):
    return ops.f64_to_bf16(x64)


# ------------------------------------------------------------------ MLP ----

def mlp_forward(x_bits, layers, eps: float = 1e-5):
    """h <- LN(GELU(h @ W + b)) per layer.

    x_bits [B,H] bf16 bits.  Every edge inside the chain is fp32 on the GPU
    (the weight-streaming GEMM reads fp32 activations), so nothing is rounded
    here after the input.  Returns fp64 [B,H].
    """
    h = ops.bf16_to_f64(np.asarray(x_bits, dtype=np.uint16))
    for L in layers:
        u = ops.gemm(h, L["w"])
        act = ops.bias_act(u, L["b"].astype(np.float64), gelu=True)      # fp32 edge
        h = ops.layernorm(act, L["gamma"].astype(np.float64), L["beta"].astype(np.float64), eps)  # fp32 edge
    return h


# -------------------------------------------------------------- encoder ----

def encoder_forward(x32, layers, batch: int, seq: int, heads: int, eps: float = 1e-5, edges: str = "stored"):
    """Post-LayerNorm encoder stack.

    x32 [batch*seq, H] fp32 hidden states.  The residual stream is fp32; the
    GEMM inputs are split-bf16 pairs (hi + lo, ~16 significant bits); the packed
    qkv tensor that attention reads is plain bf16.  Returns fp64 [batch*seq, H].

    ``edges="stored"`` rounds where the GPU graph stores a reduced-precision tensor;
    ``edges="none"`` rounds nowhere: the chain's plain definition in fp64, used to
    state how far the stored-edge graph (and the GPU) is from it.
    """
    if edges not in ("stored", "none"):
        raise ValueError("edges must be 'stored' or 'none'")
    if edges == "none":
        keep = lambda a: np.asarray(a, dtype=np.float64)
        return _encoder(x32, layers, batch, seq, heads, eps, keep, keep)
    return _encoder(x32, layers, batch, seq, heads, eps, ops.round_bf16x2, ops.round_bf16)


def _encoder(x32, layers, batch, seq, heads, eps, pair, single):
    """``pair`` is applied on the split-bf16 edges, ``single`` on the bf16 edge."""
    h = np.asarray(x32, dtype=np.float64)
    T, H = h.shape
    assert T == batch * seq and H % heads == 0
    d = H // heads
    for L in layers:
        f64 = lambda name: L[name].astype(np.float64)
        hs = pair(h)                                                     # split-bf16 edge
        qkv = ops.bias_act(ops.gemm(hs, L["w_qkv"]), f64("b_qkv"), gelu=False)
        qkv = single(qkv)                                                # bf16 edge
        qkv4 = qkv.reshape(batch, seq, 3, heads, d)
        att = ops.attention(qkv4[:, :, 0], qkv4[:, :, 1], qkv4[:, :, 2], 1.0 / math.sqrt(d))
        att_s = pair(att.reshape(T, H))                                  # split-bf16 edge
        r1 = ops.bias_act(ops.gemm(att_s, L["w_o"]), f64("b_o"), gelu=False) + h
        h1 = ops.layernorm(r1, f64("ln1_g"), f64("ln1_b"), eps)          # fp32 edge
        f = ops.bias_act(ops.gemm(pair(h1), L["w_1"]), f64("b_1"), gelu=True)
        f_s = pair(f)                                                    # split-bf16 edge
        r2 = ops.bias_act(ops.gemm(f_s, L["w_2"]), f64("b_2"), gelu=False) + h1
        h = ops.layernorm(r2, f64("ln2_g"), f64("ln2_b"), eps)           # fp32 edge
    return h


# -------------------------------------------------------------- decoder ----

def decoder_decode_step(x32, layers, kcache_bits, vcache_bits, n_q: int, n_kv: int,
                        pos: int, eps: float = 1e-5, theta: float = 10000.0):
    """One decode step of a pre-norm grouped-query decoder stack.

    x32 [B,H] fp32 hidden state of the current token (position ``pos``).
    kcache_bits / vcache_bits: per-layer lists of [B, pos, n_kv, d] bf16 bits
    holding the ``pos`` cached positions; the current token's key/value are
    rounded to bf16 (they are appended to the bf16 cache), so attention covers
    pos+1 bf16 keys.  Every other edge is fp32 on the GPU (all GEMMs are the
    weight-streaming kind that reads fp32 activations).
    Weights: w_qkv [H,(n_q+2 n_kv) d], w_o [n_q d, H], w_gu [H, 2F] (gate
    columns then up columns), w_d [F,H].  Returns fp64 [B,H] (no final norm).
    """
    x = np.asarray(x32, dtype=np.float64)
    B, H = x.shape
    d = H // n_q
    positions = np.full((B,), pos, dtype=np.int64)
    for li, L in enumerate(layers):
        n1 = ops.rmsnorm(x, L["rms1"].astype(np.float64), eps)
        qkv = ops.gemm(n1, L["w_qkv"])
        q = qkv[:, : n_q * d].reshape(B, n_q, d)
        k = qkv[:, n_q * d: (n_q + n_kv) * d].reshape(B, n_kv, d)
        v = qkv[:, (n_q + n_kv) * d:].reshape(B, n_kv, d)
        q = ops.rope(q, positions, theta)
        k = ops.round_bf16(ops.rope(k, positions, theta))               # bf16 edge (cache slot)
        v = ops.round_bf16(v)                                            # bf16 edge (cache slot)
        kc = ops.bf16_to_f64(kcache_bits[li])                            # [B,pos,n_kv,d]
        vc = ops.bf16_to_f64(vcache_bits[li])
        k_all = np.concatenate([kc, k[:, None]], axis=1)
        v_all = np.concatenate([vc, v[:, None]], axis=1)
        att = ops.attention(q[:, None], k_all, v_all, 1.0 / math.sqrt(d))  # [B,1,n_q,d]
        x = x + ops.gemm(att.reshape(B, n_q * d), L["w_o"])
        n2 = ops.rmsnorm(x, L["rms2"].astype(np.float64), eps)
        gu = ops.gemm(n2, L["w_gu"])
        F = gu.shape[1] // 2
        act = ops.silu_mul(gu[:, :F], gu[:, F:])
        x = x + ops.gemm(act, L["w_d"])
    return x
