"""Seeded synthetic inputs shaped like the benchmark configurations.

This module holds no arithmetic of the method: it only draws random numbers
(numpy PCG64) and stores them as bf16 bit patterns (uint16) or fp32 arrays.
The same host buffers go to the GPU path and to whatever checks it.
Rounding fp32 draws to bf16 is delegated to torch's dtype cast.
"""
from __future__ import annotations

import numpy as np
import torch


def to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """fp32 array -> bf16 bit patterns (uint16), via torch's cast."""
    t = torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bits_to_torch(bits: np.ndarray, device="cpu") -> torch.Tensor:
    """bf16 bit patterns -> torch.bfloat16 tensor with the same bits."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t.to(device)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def uniform_bits(shape, seed, lo=-1.0, hi=1.0):
    return to_bf16_bits(_rng(seed).uniform(lo, hi, size=shape).astype(np.float32))


def normal_bits(shape, seed, std=1.0):
    return to_bf16_bits((_rng(seed).standard_normal(size=shape, dtype=np.float32) * np.float32(std)))


def normal_f32(shape, seed, std=1.0, mean=0.0):
    return (_rng(seed).standard_normal(size=shape, dtype=np.float32) * np.float32(std)
            + np.float32(mean)).astype(np.float32)


def gemm_operands(m, n, k, seed=0, dist="uniform", ta=False, tb=False):
    """A and B of C = op(A) op(B); stored [K,M] / [N,K] when transposed."""
    ashape = (k, m) if ta else (m, k)
    bshape = (n, k) if tb else (k, n)
    if dist == "uniform":
        return uniform_bits(ashape, [seed, 0]), uniform_bits(bshape, [seed, 1])
    return normal_bits(ashape, [seed, 0]), normal_bits(bshape, [seed, 1])


def mlp_params(n_layers=6, hidden=4096, seed=1, w_std=0.02):
    """Per layer: w [H,H] bf16 bits N(0, w_std^2); b, gamma, beta fp32."""
    layers = []
    for i in range(n_layers):
        layers.append(dict(
            w=normal_bits((hidden, hidden), [seed, i, 0], w_std),
            b=normal_f32((hidden,), [seed, i, 1], w_std),
            gamma=normal_f32((hidden,), [seed, i, 2], 0.02, 1.0),
            beta=normal_f32((hidden,), [seed, i, 3], 0.02),
        ))
    return layers


def mlp_requests(pool=64, batch=8, hidden=4096, seed=2):
    """A pool of request inputs: [pool, batch, hidden] bf16 bits N(0,1)."""
    return normal_bits((pool, batch, hidden), seed)


def poisson_arrivals(rate_per_s, n, seed=3):
    """Arrival times in seconds of an open-loop Poisson process."""
    gaps = _rng(seed).exponential(1.0 / rate_per_s, size=n)
    return np.cumsum(gaps)


def encoder_params(n_layers=12, hidden=768, ffn=3072, seed=10, w_std=0.02):
    layers = []
    for i in range(n_layers):
        s = lambda j: [seed, i, j]
        layers.append(dict(
            w_qkv=normal_bits((hidden, 3 * hidden), s(0), w_std), b_qkv=normal_f32((3 * hidden,), s(1), w_std),
            w_o=normal_bits((hidden, hidden), s(2), w_std), b_o=normal_f32((hidden,), s(3), w_std),
            ln1_g=normal_f32((hidden,), s(4), 0.02, 1.0), ln1_b=normal_f32((hidden,), s(5), 0.02),
            w_1=normal_bits((hidden, ffn), s(6), w_std), b_1=normal_f32((ffn,), s(7), w_std),
            w_2=normal_bits((ffn, hidden), s(8), w_std), b_2=normal_f32((hidden,), s(9), w_std),
            ln2_g=normal_f32((hidden,), s(10), 0.02, 1.0), ln2_b=normal_f32((hidden,), s(11), 0.02),
        ))
    return layers


def encoder_hidden(batch, seq=128, hidden=768, seed=11):
    return normal_f32((batch * seq, hidden), seed)


def decoder_params(n_layers=32, hidden=4096, n_q=32, n_kv=8, ffn=14336, seed=20, w_std=0.02, first=0):
    """Layers first .. first+n_layers-1 (every layer draws from its own seed, so a model can be built in pieces)."""
    d = hidden // n_q
    layers = []
    for i in range(first, first + n_layers):
        s = lambda j: [seed, i, j]
        layers.append(dict(
            rms1=np.ones((hidden,), np.float32), rms2=np.ones((hidden,), np.float32),
            w_qkv=normal_bits((hidden, (n_q + 2 * n_kv) * d), s(0), w_std),
            w_o=normal_bits((n_q * d, hidden), s(1), w_std),
            w_gu=normal_bits((hidden, 2 * ffn), s(2), w_std),
            w_d=normal_bits((ffn, hidden), s(3), w_std),
        ))
    return layers


def decoder_kv_cache(n_layers, batch, tokens=2048, n_kv=8, d=128, seed=21):
    """Per layer: (k_bits, v_bits), each [batch, tokens, n_kv, d] N(0,1)."""
    ks, vs = [], []
    for i in range(n_layers):
        ks.append(normal_bits((batch, tokens, n_kv, d), [seed, i, 0]))
        vs.append(normal_bits((batch, tokens, n_kv, d), [seed, i, 1]))
    return ks, vs


def decoder_hidden(batch, hidden=4096, seed=22):
    return normal_f32((batch, hidden), seed)
