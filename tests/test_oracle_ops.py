"""Pins for the single-operator CPU oracle: closed forms, identities, brute
force and independent library routines (never the oracle's own formula)."""
import math

import numpy as np
import pytest
import torch

from oracle import ops
from paper_2504_15465_amd import inputs


# ------------------------------------------------------------------ bf16 ---

def test_bf16_ties_to_even_examples():
    # 1 + 2^-8 is a tie between 1.0 (even) and 1 + 2^-7 (odd)
    vals = np.array([1 + 2.0**-8, 1 + 3 * 2.0**-8, 1 + 2.0**-8 + 2.0**-20, 1 - 2.0**-9])
    got = ops.round_bf16(vals)
    assert got.tolist() == [1.0, 1 + 2.0**-6, 1 + 2.0**-7, 1.0]


def test_bf16_every_pattern_round_trips():
    bits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    vals = ops.bf16_to_f64(bits)
    back = ops.f64_to_bf16(vals)
    finite_or_inf = ~np.isnan(vals)
    assert np.array_equal(back[finite_or_inf], bits[finite_or_inf])
    assert np.all(np.isnan(ops.bf16_to_f64(back[~finite_or_inf])))


def test_bf16_specials():
    b = ops.f64_to_bf16(np.array([np.inf, -np.inf, 0.0, -0.0, 1e39, -1e39, 3.39e38]))
    assert b.tolist() == [0x7F80, 0xFF80, 0x0000, 0x8000, 0x7F80, 0xFF80, 0x7F7F]
    assert np.isnan(ops.bf16_to_f64(ops.f64_to_bf16(np.array([np.nan]))))[0]


def test_bf16_matches_torch_cast_on_fp32_data():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32) * 3,
                        (rng.standard_normal(5000) * 1e-39).astype(np.float32),
                        np.float32(2.0) ** rng.integers(-130, 127, 5000).astype(np.float32)])
    ours = ops.f64_to_bf16(x.astype(np.float64))
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)


def test_bf16_single_rounding_from_fp64():
    # Value just above the tie 1+2^-8: fp64 sees the excess, fp32 would not.
    v = 1 + 2.0**-8 + 2.0**-40
    assert float(np.float32(v)) == 1 + 2.0**-8           # excess lost in binary32
    assert ops.round_bf16(np.array([v]))[0] == 1 + 2.0**-7  # still rounds up


# ------------------------------------------------------------------ GEMM ---

def _naive(a, b):
    m, k = a.shape
    n = b.shape[1]
    c = [[0.0] * n for _ in range(m)]
    for i in range(m):
        for j in range(n):
            s = 0.0
            for kk in range(k):
                s += float(a[i, kk]) * float(b[kk, j])
            c[i][j] = s
    return np.array(c).reshape(m, n)


@pytest.mark.parametrize("shape", [(1, 1, 1), (2, 3, 4), (5, 7, 3), (17, 13, 9), (8, 1, 33)])
@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False), (True, True)])
def test_gemm_equals_python_triple_loop(shape, ta, tb):
    m, n, k = shape
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=m * 100 + n * 10 + k, ta=ta, tb=tb)
    a = ops.bf16_to_f64(a_bits)
    b = ops.bf16_to_f64(b_bits)
    ref = _naive(a.T if ta else a, b.T if tb else b)
    for fast in (False, True):
        got = ops.gemm(a_bits, b_bits, ta=ta, tb=tb, fast=fast)
        assert np.array_equal(got, ref)     # same sums in the same order: bit-equal


def test_gemm_identity_ones_and_exact_data():
    rng = np.random.default_rng(1)
    a_bits = inputs.uniform_bits((40, 64), 3)
    eye = inputs.to_bf16_bits(np.eye(64, dtype=np.float32))
    assert np.array_equal(ops.gemm(a_bits, eye), ops.bf16_to_f64(a_bits))
    ones_a = inputs.to_bf16_bits(np.ones((9, 300), np.float32))
    ones_b = inputs.to_bf16_bits(np.ones((300, 11), np.float32))
    assert np.all(ops.gemm(ones_a, ones_b) == 300.0)
    # entries from {+-1, +-0.5, +-2}: every partial sum is exact in any precision
    vals = np.array([1, -1, .5, -.5, 2, -2], np.float32)
    a = vals[rng.integers(0, 6, (33, 128))]
    b = vals[rng.integers(0, 6, (128, 21))]
    got = ops.gemm(inputs.to_bf16_bits(a), inputs.to_bf16_bits(b))
    assert np.array_equal(got, a.astype(np.float64) @ b.astype(np.float64))


def test_gemm_matches_blas_fp64_and_transposes():
    m, n, k = 96, 80, 512
    for ta in (False, True):
        for tb in (False, True):
            a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=7, ta=ta, tb=tb)
            a = ops.bf16_to_f64(a_bits)
            b = ops.bf16_to_f64(b_bits)
            ref = (a.T if ta else a) @ (b.T if tb else b)      # BLAS dgemm, independent
            got = ops.gemm(a_bits, b_bits, ta=ta, tb=tb)
            assert np.allclose(got, ref, rtol=0, atol=1e-11)
            # a transposed operand flag must not be silently ignored
            if m != k:
                with pytest.raises(ValueError):
                    ops.gemm(a_bits, b_bits, ta=not ta, tb=tb)


def test_sum_slices_closed_forms_and_k_cut_of_a_gemm():
    # planes of constants: 1 + 2 + ... + S
    for s in (1, 2, 5):
        planes = np.stack([np.full((3, 4), z + 1.0) for z in range(s)])
        assert np.all(ops.sum_slices(planes) == s * (s + 1) / 2)
    one = np.arange(12.0).reshape(1, 3, 4)
    assert np.array_equal(ops.sum_slices(one), one[0])
    # the cut covers K exactly once, in order, in whole 64-wide steps (the last range may be ragged)
    for k, s in ((200, 3), (64, 1), (1000, 7), (16384, 5)):
        b = ops.k_slice_bounds(k, s)
        assert b[0][0] == 0 and b[-1][1] == k and all(x[1] == y[0] for x, y in zip(b, b[1:]))
        assert all(lo % 64 == 0 and lo <= hi for lo, hi in b)
        assert max(hi - lo for lo, hi in b) - min(hi - lo for lo, hi in b) <= 64 + (-k) % 64
    # a GEMM on exactly representable data equals the sum of its K ranges bit for bit
    rng = np.random.default_rng(3)
    a = rng.choice([-2.0, -1.0, -0.5, 0.5, 1.0, 2.0], size=(9, 200))
    bm = rng.choice([-2.0, -1.0, -0.5, 0.5, 1.0, 2.0], size=(200, 7))
    a_bits, b_bits = inputs.to_bf16_bits(a), inputs.to_bf16_bits(bm)
    parts = np.stack([ops.gemm(a_bits[:, lo:hi], b_bits[lo:hi]) for lo, hi in ops.k_slice_bounds(200, 3)])
    assert np.array_equal(ops.sum_slices(parts), ops.gemm(a_bits, b_bits))
    # and on random data up to fp64 rounding of the regrouped sum
    a_bits, b_bits = inputs.gemm_operands(9, 7, 200, seed=5)
    parts = np.stack([ops.gemm(a_bits[:, lo:hi], b_bits[lo:hi]) for lo, hi in ops.k_slice_bounds(200, 3)])
    np.testing.assert_allclose(ops.sum_slices(parts), ops.gemm(a_bits, b_bits), rtol=0, atol=1e-12)


def test_gemm_frobenius_scale_of_uniform_inputs():
    # entries U[-1,1] have variance 1/3, so C elements have std sqrt(K)/3
    a_bits, b_bits = inputs.gemm_operands(128, 128, 512, seed=0)
    c = ops.gemm(a_bits, b_bits)
    assert abs(c.std() - math.sqrt(512) / 3) < 0.25


# ----------------------------------------------------------- bias + GELU ---

def test_gelu_closed_forms():
    assert ops.gelu(0.0) == 0.0
    # g(1) = Phi(1), the standard normal CDF at 1 (tabulated 0.8413447461)
    assert abs(ops.gelu(1.0) - 0.8413447460685429) < 1e-15
    for u in (0.3, 1.7, 4.0, 7.5):
        assert abs((ops.gelu(u) - ops.gelu(-u)) - u) < 1e-15      # g(u) - g(-u) = u
    assert abs(ops.gelu(8.0) - 8.0) < 1e-13 and abs(ops.gelu(-8.0)) < 1e-13


def test_bias_act_matches_scipy_erf_and_broadcasts_bias():
    from scipy.special import erf
    rng = np.random.default_rng(2)
    x = rng.standard_normal((7, 33))
    b = rng.standard_normal(33)
    u = x + b[None, :]
    ref = 0.5 * u * (1 + erf(u / np.sqrt(2)))
    assert np.allclose(ops.bias_act(x, b), ref, rtol=0, atol=1e-15)
    assert np.array_equal(ops.bias_act(x, b, gelu=False), u)
    assert np.array_equal(ops.bias_act(x, None, gelu=False), x)
    # a bias applied along rows instead of columns would break this
    assert not np.allclose(ops.bias_act(x, b, gelu=False), x + b[:7, None].repeat(33, 1))


# -------------------------------------------------------------- LayerNorm --

def test_layernorm_invariants_and_torch():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 257)) * 3 + 1.5
    ones, zeros = np.ones(257), np.zeros(257)
    y = ops.layernorm(x, ones, zeros, 1e-5)
    var = x.var(axis=1)                        # biased
    assert np.allclose(y.mean(axis=1), 0, atol=1e-14)
    assert np.allclose(y.var(axis=1), var / (var + 1e-5), rtol=1e-12)
    # constant row -> beta
    g, b = rng.standard_normal(257), rng.standard_normal(257)
    yc = ops.layernorm(np.full((2, 257), 4.25), g, b, 1e-5)
    assert np.allclose(yc, b[None, :], atol=1e-12)
    # scale invariance up to eps, permutation equivariance
    assert np.allclose(ops.layernorm(7 * x, ones, zeros, 0.0), ops.layernorm(x, ones, zeros, 0.0), atol=1e-12)
    perm = rng.permutation(257)
    assert np.allclose(ops.layernorm(x[:, perm], g[perm], b[perm]), ops.layernorm(x, g, b)[:, perm], atol=1e-13)
    # independent library routine
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (257,), torch.from_numpy(g),
                                         torch.from_numpy(b), 1e-5).numpy()
    assert np.allclose(ops.layernorm(x, g, b, 1e-5), ref, atol=1e-12)


def test_rmsnorm_closed_forms():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((4, 64))
    w = rng.standard_normal(64)
    y = ops.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose((y * y).mean(axis=1), 1.0, rtol=1e-13)   # unit RMS
    assert np.allclose(ops.rmsnorm(x, w, 0.0), y * w[None, :], rtol=1e-13)
    # +-c row: rms = c, so y = sign * w
    row = np.where(np.arange(64) % 2 == 0, 3.0, -3.0)[None, :]
    assert np.allclose(ops.rmsnorm(row, w, 0.0), np.sign(row) * w, rtol=1e-14)
    # eps enters under the root: zero row gives zero, tiny row is damped
    assert np.all(ops.rmsnorm(np.zeros((1, 64)), w, 1e-5) == 0)
    assert np.allclose(ops.rmsnorm(np.full((1, 64), 1e-3), np.ones(64), 1e-5),
                       1e-3 / math.sqrt(1e-6 + 1e-5), rtol=1e-13)


# ---------------------------------------------------------------- softmax --

def test_softmax_invariants_and_scipy():
    from scipy.special import softmax as sp_softmax
    rng = np.random.default_rng(6)
    s = rng.standard_normal((9, 130)) * 4
    p = ops.softmax(s)
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-14)
    assert np.allclose(ops.softmax(s + 1000.0), p, atol=1e-13)       # shift invariance, no overflow
    assert np.allclose(ops.softmax(np.full((2, 7), 3.3)), 1 / 7)
    hot = np.zeros((1, 10)); hot[0, 4] = 80.0
    assert ops.softmax(hot)[0, 4] == 1.0 and ops.softmax(hot)[0, 0] < 1e-30
    assert np.allclose(p, sp_softmax(s, axis=1), atol=1e-15)


# -------------------------------------------------------------- attention --

def test_attention_special_cases():
    rng = np.random.default_rng(7)
    B, S, H, d = 2, 5, 3, 8
    q = rng.standard_normal((B, S, H, d))
    k = rng.standard_normal((B, 1, H, d))
    v = rng.standard_normal((B, 1, H, d))
    o = ops.attention(q, k, v, 0.3)                       # single key -> its value
    assert np.allclose(o, np.broadcast_to(v, o.shape), atol=1e-15)
    k = np.broadcast_to(rng.standard_normal((B, 1, H, d)), (B, 6, H, d)).copy()
    v = rng.standard_normal((B, 6, H, d))
    o = ops.attention(q, k, v, 0.3)                       # equal keys -> mean of values
    assert np.allclose(o, np.broadcast_to(v.mean(axis=1, keepdims=True), o.shape), atol=1e-14)
    k = rng.standard_normal((B, 6, H, d))
    v = np.broadcast_to(rng.standard_normal((B, 1, H, d)), (B, 6, H, d)).copy()
    o = ops.attention(q, k, v, 0.3)                       # constant value -> that value
    assert np.allclose(o, np.broadcast_to(v[:, :1], o.shape), atol=1e-14)


def test_attention_matches_torch_sdpa_and_gqa_expansion():
    rng = np.random.default_rng(8)
    B, Sq, Sk, Hq, Hkv, d = 2, 4, 37, 8, 2, 16
    q = rng.standard_normal((B, Sq, Hq, d))
    k = rng.standard_normal((B, Sk, Hkv, d))
    v = rng.standard_normal((B, Sk, Hkv, d))
    scale = 1 / math.sqrt(d)
    got = ops.attention(q, k, v, scale)
    # grouped-query == multi-head on keys/values repeated per group (h -> h // 4)
    k_exp = np.repeat(k, Hq // Hkv, axis=2)
    v_exp = np.repeat(v, Hq // Hkv, axis=2)
    assert np.allclose(got, ops.attention(q, k_exp, v_exp, scale), atol=1e-14)
    t = lambda a: torch.from_numpy(a).permute(0, 2, 1, 3)            # [B,H,S,d]
    ref = torch.nn.functional.scaled_dot_product_attention(t(q), t(k_exp), t(v_exp), scale=scale)
    assert np.allclose(got, ref.permute(0, 2, 1, 3).numpy(), atol=1e-12)
    # strided views (a packed qkv tensor) are read through their strides
    packed = rng.standard_normal((B, Sk, 3, Hq, d))
    o1 = ops.attention(packed[:, :, 0], packed[:, :, 1], packed[:, :, 2], scale)
    o2 = ops.attention(packed[:, :, 0].copy(), packed[:, :, 1].copy(), packed[:, :, 2].copy(), scale)
    assert np.array_equal(o1, o2)


def test_causal_attention_is_attention_over_each_querys_prefix():
    """Query i sees keys 0..i: equal to plain attention of that one query over the key prefix (brute force
    over every query), to torch's causal SDPA, independent of later keys and values, and V[0] for query 0."""
    rng = np.random.default_rng(12)
    B, S, Hq, Hkv, d = 2, 11, 4, 2, 8
    q = rng.standard_normal((B, S, Hq, d))
    k = rng.standard_normal((B, S, Hkv, d))
    v = rng.standard_normal((B, S, Hkv, d))
    scale = 0.35
    got = ops.attention_causal(q, k, v, scale)
    for i in range(S):
        want = ops.attention(q[:, i:i + 1], k[:, :i + 1], v[:, :i + 1], scale)
        assert np.allclose(got[:, i:i + 1], want, atol=1e-14), i
    g = Hq // Hkv
    assert np.allclose(got[:, 0], np.repeat(v[:, 0], g, axis=1), atol=1e-15)           # one visible key
    t = lambda a: torch.from_numpy(a).permute(0, 2, 1, 3)
    ref = torch.nn.functional.scaled_dot_product_attention(t(q), t(np.repeat(k, g, axis=2)), t(np.repeat(v, g, axis=2)),
                                                           is_causal=True, scale=scale)
    assert np.allclose(got, ref.permute(0, 2, 1, 3).numpy(), atol=1e-12)
    k2, v2 = k.copy(), v.copy()
    k2[:, 7:] += 5.0
    v2[:, 7:] -= 3.0
    got2 = ops.attention_causal(q, k2, v2, scale)
    assert np.array_equal(got2[:, :7], got[:, :7]) and not np.allclose(got2[:, 7:], got[:, 7:])
    # without the mask the last query is the only one that agrees with plain attention
    full = ops.attention(q, k, v, scale)
    assert np.allclose(full[:, -1], got[:, -1], atol=1e-14) and not np.allclose(full[:, 0], got[:, 0])


# ------------------------------------------------------------------- rope --

def test_rope_rotation_properties():
    rng = np.random.default_rng(9)
    rows, heads, d = 3, 2, 16
    x = rng.standard_normal((rows, heads, d))
    assert np.allclose(ops.rope(x, np.zeros(rows, np.int64)), x, atol=0)      # position 0 is identity
    pos = np.array([1, 17, 2048])
    y = ops.rope(x, pos)
    # a rotation of (x[e], x[e+d/2]) pairs keeps each pair's norm
    n_in = x[..., :8] ** 2 + x[..., 8:] ** 2
    n_out = y[..., :8] ** 2 + y[..., 8:] ** 2
    assert np.allclose(n_in, n_out, rtol=1e-12)
    # pair 0 turns by exactly pos radians (theta^0 = 1): check against complex multiplication
    z = (x[..., 0] + 1j * x[..., 8]) * np.exp(1j * pos)[:, None]
    assert np.allclose(y[..., 0], z.real, atol=1e-12) and np.allclose(y[..., 8], z.imag, atol=1e-12)
    # pair e turns by pos * theta^(-2e/d)
    e = 5
    z = (x[..., e] + 1j * x[..., e + 8]) * np.exp(1j * pos * 10000.0 ** (-2 * e / d))[:, None]
    assert np.allclose(y[..., e], z.real, atol=1e-12) and np.allclose(y[..., e + 8], z.imag, atol=1e-12)
    # relative-position property: <rope(q,m), rope(k,n)> depends on m-n only
    q, k = x[:1], rng.standard_normal((1, heads, d))
    a = (ops.rope(q, [10]) * ops.rope(k, [3])).sum()
    b = (ops.rope(q, [1010]) * ops.rope(k, [1003])).sum()
    assert abs(a - b) < 1e-9


def test_silu_mul_closed_forms():
    g = np.array([0.0, 1.0, -1.0, 30.0, -30.0])
    u = np.array([5.0, 2.0, 2.0, 1.0, 1.0])
    y = ops.silu_mul(g, u)
    assert y[0] == 0.0
    assert abs(y[1] - 2.0 / (1 + math.exp(-1))) < 1e-15
    assert abs(y[1] - y[2] - 2.0) < 1e-15         # silu(g) - silu(-g) = g, times u = 2
    assert abs(y[3] - 30.0) < 1e-11 and abs(y[4]) < 1e-11
    ref = torch.nn.functional.silu(torch.from_numpy(g)) * torch.from_numpy(u)
    assert np.allclose(y, ref.numpy(), atol=1e-15)


def test_split_bf16_pair_properties():
    rng = np.random.default_rng(12)
    x = np.concatenate([rng.standard_normal(5000) * 3, [1.0, 1 + 2.0**-8, 1 + 2.0**-9, 0.0, -2.5]])
    v = ops.round_bf16x2(x)
    hi = ops.round_bf16(x)
    assert np.array_equal(v, hi + ops.round_bf16(x - hi))
    nz = x != 0
    assert np.all(np.abs(v[nz] - x[nz]) <= 2.0**-17 * np.abs(x[nz]))     # two 8-bit significands
    assert ops.round_bf16x2(np.array([1 + 2.0**-9]))[0] == 1 + 2.0**-9   # exactly representable as a pair
    assert np.array_equal(ops.round_bf16x2(hi), hi)                     # bf16 values split as (v, 0)


# ---------------------------------------- fused forms of the GEMM's row kernels ---

def test_normalised_rows_times_weights_is_a_scaled_and_shifted_product():
    """The identities that let a GEMM normalise its rows without a pass over them first (what the
    weight-streaming kernel's NORM_LN / NORM_RMS forms compute), checked with the oracle's own
    operators in fp64: statistics act on whole output rows, and the two column vectors of
    LayerNorm are the products of gamma and of beta with the weights."""
    rng = np.random.default_rng(5)
    m, n, k, eps = 5, 24, 64, 1e-5
    x = 0.7 + 1.9 * rng.standard_normal((m, k))
    gamma, beta = 1.0 + 0.3 * rng.standard_normal(k), 0.2 * rng.standard_normal(k)
    _, w_bits = inputs.gemm_operands(m, n, k, seed=3, tb=True, dist="normal")
    w = ops.bf16_to_f64(w_bits)                                     # [n, k]
    # RMSNorm
    r = 1.0 / np.sqrt((x * x).mean(axis=1) + eps)
    want = ops.gemm(ops.rmsnorm(x, gamma, eps), w_bits, tb=True)
    got = r[:, None] * ops.gemm(x * gamma, w_bits, tb=True)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    # LayerNorm, sums shifted by the row's first element
    c = x[:, :1]
    dm = (x - c).mean(axis=1)
    var = ((x - c) ** 2).mean(axis=1) - dm ** 2
    assert np.allclose(var, x.var(axis=1), rtol=1e-12)
    rstd = 1.0 / np.sqrt(var + eps)
    colsums = ops.gemm(np.stack([gamma, beta]), w_bits, tb=True)   # [2, n]
    assert np.allclose(colsums[0], w @ gamma) and np.allclose(colsums[1], w @ beta)
    want = ops.gemm(ops.layernorm(x, gamma, beta, eps), w_bits, tb=True)
    got = rstd[:, None] * (ops.gemm((x - c) * gamma, w_bits, tb=True) - dm[:, None] * colsums[0]) + colsums[1]
    assert np.allclose(got, want, rtol=1e-11, atol=1e-11)
    # gated epilogue: the [m, 2f] product halves, gate first
    f = n // 2
    p = ops.gemm(x, w_bits, tb=True)
    g, u = p[:, :f], p[:, f:]
    assert np.allclose(ops.silu_mul(g, u), g / (1.0 + np.exp(-g)) * u, rtol=1e-13)
