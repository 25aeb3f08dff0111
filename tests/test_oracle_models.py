"""Pins for the operator-chain oracles: each chain is re-derived with torch's
own fp64 operators and torch's bf16 cast (an independent library), on small
shapes, and a few structural properties are checked."""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import models, ops
from paper_2504_15465_amd import inputs


def bf(t):
    """torch-side bf16 edge: fp64 -> bf16 -> fp64 with ONE rounding.

    torch's cast goes fp64 -> fp32 -> bf16, which rounds twice.  Here the first step is done by
    hand with round-to-odd (truncate toward zero, then set the last mantissa bit if anything was
    lost): a value that went through round-to-odd at 24 bits rounds to nearest-even at 8 bits
    exactly as the fp64 value itself would.  torch's fp32 -> bf16 cast does the second step.
    """
    x = t.numpy()
    f = x.astype(np.float32)
    back = f.astype(np.float64)
    over = np.abs(back) > np.abs(x)                     # nearest went away from zero: step back
    f = np.where(over, np.nextafter(f, np.float32(0)), f)
    inexact = f.astype(np.float64) != x
    bits = f.view(np.uint32) | inexact.astype(np.uint32)
    return torch.from_numpy(bits.view(np.float32).copy()).to(torch.bfloat16).to(torch.float64)


def bf2(t):
    """split-bf16 edge: hi + lo with hi = bf16(t), lo = bf16(t - hi)."""
    hi = bf(t)
    return hi + bf(t - hi)


def w64(bits):
    return inputs.bits_to_torch(bits).to(torch.float64)


def test_mlp_chain_against_torch():
    layers = inputs.mlp_params(n_layers=3, hidden=64, seed=1, w_std=0.1)
    x_bits = inputs.normal_bits((5, 64), 2)
    got = models.mlp_forward(x_bits, layers)
    h = w64(x_bits)
    for i, L in enumerate(layers):
        u = h @ w64(L["w"]) + torch.from_numpy(L["b"]).double()
        a = F.gelu(u)                                         # erf form, fp64
        h = F.layer_norm(a, (64,), torch.from_numpy(L["gamma"]).double(),
                         torch.from_numpy(L["beta"]).double(), 1e-5)
    # no rounding inside the chain: the two fp64 evaluations agree closely
    assert np.abs(got - h.numpy()).max() < 1e-10
    assert got.shape == (5, 64)
    # last LayerNorm is an fp32 edge: per-row statistics are those of LN output
    gam = np.stack([layers[-1]["gamma"]] * 5).astype(np.float64)
    bet = np.stack([layers[-1]["beta"]] * 5).astype(np.float64)
    z = (got - bet) / gam
    assert np.allclose(z.mean(axis=1), 0, atol=1e-9)


def test_encoder_chain_against_torch():
    Bn, S, H, heads, ffn = 2, 8, 32, 4, 64
    layers = inputs.encoder_params(n_layers=2, hidden=H, ffn=ffn, seed=10, w_std=0.1)
    x = inputs.encoder_hidden(Bn, S, H, seed=11)
    got = models.encoder_forward(x, layers, Bn, S, heads)
    d = H // heads
    h = torch.from_numpy(x).double()
    tv = lambda L, n: torch.from_numpy(L[n]).double()
    for L in layers:
        qkv = bf(bf2(h) @ w64(L["w_qkv"]) + tv(L, "b_qkv"))
        q, k, v = [t.reshape(Bn, S, heads, d).permute(0, 2, 1, 3) for t in qkv.split(H, dim=1)]
        att = F.scaled_dot_product_attention(q, k, v).permute(0, 2, 1, 3).reshape(Bn * S, H)
        r1 = bf2(att) @ w64(L["w_o"]) + tv(L, "b_o") + h
        h1 = F.layer_norm(r1, (H,), tv(L, "ln1_g"), tv(L, "ln1_b"), 1e-5)
        f = bf2(F.gelu(bf2(h1) @ w64(L["w_1"]) + tv(L, "b_1")))
        r2 = f @ w64(L["w_2"]) + tv(L, "b_2") + h1
        h = F.layer_norm(r2, (H,), tv(L, "ln2_g"), tv(L, "ln2_b"), 1e-5)
    # same edges, each rounded once on both sides: what is left is fp64 summation order
    diff = np.abs(got - h.numpy())
    assert diff.max() < 1e-9, diff.max()
    # the chain with no rounding at any edge (the plain definition): the mirrored edges move the
    # result by about the bf16 rounding of q, k and v, the only coarse edge
    plain = models.encoder_forward(x, layers, Bn, S, heads, edges="none")
    h = torch.from_numpy(x).double()
    for L in layers:
        qkv = h @ w64(L["w_qkv"]) + tv(L, "b_qkv")
        q, k, v = [t.reshape(Bn, S, heads, d).permute(0, 2, 1, 3) for t in qkv.split(H, dim=1)]
        att = F.scaled_dot_product_attention(q, k, v).permute(0, 2, 1, 3).reshape(Bn * S, H)
        h1 = F.layer_norm(att @ w64(L["w_o"]) + tv(L, "b_o") + h, (H,), tv(L, "ln1_g"), tv(L, "ln1_b"), 1e-5)
        f = F.gelu(h1 @ w64(L["w_1"]) + tv(L, "b_1"))
        h = F.layer_norm(f @ w64(L["w_2"]) + tv(L, "b_2") + h1, (H,), tv(L, "ln2_g"), tv(L, "ln2_b"), 1e-5)
    assert np.abs(plain - h.numpy()).max() < 1e-10
    gap = np.abs(plain - got).max()
    assert 1e-6 < gap < 1e-2, gap


def test_decoder_chain_against_torch():
    Bn, H, n_q, n_kv, ffn, T, nl = 2, 64, 4, 2, 96, 9, 2
    d = H // n_q
    layers = inputs.decoder_params(nl, H, n_q, n_kv, ffn, seed=20, w_std=0.1)
    ks, vs = inputs.decoder_kv_cache(nl, Bn, T, n_kv, d, seed=21)
    x = inputs.decoder_hidden(Bn, H, seed=22)
    got = models.decoder_decode_step(x, layers, ks, vs, n_q, n_kv, pos=T)

    def rope_t(t, pos):                     # t [B, heads, d], rotate-half
        half = d // 2
        inv = 10000.0 ** (-torch.arange(0, half, dtype=torch.float64) * 2 / d)
        ang = pos * inv
        c, s = torch.cos(ang), torch.sin(ang)
        a, b = t[..., :half], t[..., half:]
        return torch.cat([a * c - b * s, b * c + a * s], dim=-1)

    h = torch.from_numpy(x).double()
    for li, L in enumerate(layers):
        rms = lambda t: t / torch.sqrt((t * t).mean(dim=1, keepdim=True) + 1e-5)
        n1 = rms(h)
        qkv = n1 @ w64(L["w_qkv"])
        q = rope_t(qkv[:, : n_q * d].reshape(Bn, n_q, d), T)
        k = bf(rope_t(qkv[:, n_q * d:(n_q + n_kv) * d].reshape(Bn, n_kv, d), T))
        v = bf(qkv[:, (n_q + n_kv) * d:].reshape(Bn, n_kv, d))
        k_all = torch.cat([w64(ks[li]), k[:, None]], dim=1)        # [B,T+1,n_kv,d]
        v_all = torch.cat([w64(vs[li]), v[:, None]], dim=1)
        k_e = k_all.repeat_interleave(n_q // n_kv, dim=2).permute(0, 2, 1, 3)
        v_e = v_all.repeat_interleave(n_q // n_kv, dim=2).permute(0, 2, 1, 3)
        att = F.scaled_dot_product_attention(q[:, :, None], k_e, v_e)[:, :, 0].reshape(Bn, n_q * d)
        h = h + att @ w64(L["w_o"])
        n2 = rms(h)
        gu = n2 @ w64(L["w_gu"])
        act = F.silu(gu[:, :ffn]) * gu[:, ffn:]
        h = h + act @ w64(L["w_d"])
    diff = np.abs(got - h.numpy())
    # only the appended key/value are rounded (bf16 cache), once on both sides
    assert diff.max() < 1e-9, diff.max()


def test_decoder_attends_to_cache_and_current_token():
    """Changing a cached key/value, or dropping the current token, changes the output."""
    Bn, H, n_q, n_kv, ffn, T = 1, 32, 4, 2, 48, 5
    d = H // n_q
    layers = inputs.decoder_params(1, H, n_q, n_kv, ffn, seed=3, w_std=0.2)
    ks, vs = inputs.decoder_kv_cache(1, Bn, T, n_kv, d, seed=4)
    x = inputs.decoder_hidden(Bn, H, seed=5)
    base = models.decoder_decode_step(x, layers, ks, vs, n_q, n_kv, pos=T)
    vs2 = [vs[0].copy()]
    vs2[0][0, 2, 1, :] ^= 0x8000                    # flip sign of one cached value row
    assert np.abs(models.decoder_decode_step(x, layers, ks, vs2, n_q, n_kv, pos=T) - base).max() > 1e-4
    # position matters through the rotary embedding of q and the new k
    assert np.abs(models.decoder_decode_step(x, layers, ks, vs, n_q, n_kv, pos=T + 7) - base).max() > 1e-5
