"""GPU parity of the row / elementwise kernels against the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

from oracle import ops as O
from paper_2504_15465_amd import binding as B
from paper_2504_15465_amd import inputs
from gpu_util import bits_equal, bf16_close, counters, ctx, dev_bits, nan_like

pytestmark = pytest.mark.gpu


def launch(op, atom_blocks=0, count=True):
    grid, _ = B.lithos_op_grid(ctx(), op)
    total = grid[0] * grid[1] * grid[2]
    cnt = counters(total)
    if count:
        B.lithos_debug_block_counters(ctx(), cnt)
    torch.cuda.synchronize()        # torch's fills/copies run on its own stream
    try:
        B.lithos_launch_atomized(ctx(), op, (0, 0, 0), atom_blocks, None, None)
        B.lithos_partition_sync(ctx(), None)
    finally:
        B.lithos_debug_block_counters(ctx(), None)
    if count:
        assert cnt.cpu().tolist() == [1] * total
    return total


def f32_close(y, ref, tol):
    d = np.abs(y.cpu().numpy().astype(np.float64) - ref)
    assert d.max() <= tol, d.max()


@pytest.mark.parametrize("rows,cols", [(8, 4096), (128, 768), (37, 1000), (5, 2056)])
@pytest.mark.parametrize("in32,out32", [(True, True), (True, False), (False, False), (False, True)])
def test_layernorm(rows, cols, in32, out32):
    x32 = inputs.normal_f32((rows, cols), 1, 2.0, 0.5)
    g, b = inputs.normal_f32((cols,), 2, 0.02, 1.0), inputs.normal_f32((cols,), 3, 0.02)
    if in32:
        x, x64 = torch.from_numpy(x32).cuda(), x32.astype(np.float64)
    else:
        bits = inputs.to_bf16_bits(x32)
        x, x64 = dev_bits(bits), O.bf16_to_f64(bits)
    ref = O.layernorm(x64, g.astype(np.float64), b.astype(np.float64), 1e-5)
    y = nan_like((rows, cols), torch.float32 if out32 else torch.bfloat16)
    y2 = nan_like((rows, cols), torch.bfloat16) if out32 else None
    op = B.layernorm_op(x, torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), y, rows, cols, 1e-5, y_bf16=y2)
    launch(op)
    if out32:
        f32_close(y, ref, 5e-5)
        bf16_close(y2, ref)
    else:
        bf16_close(y, ref)
    ya = nan_like(y.shape, y.dtype)
    opa = B.layernorm_op(x, torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), ya, rows, cols, 1e-5)
    launch(opa, atom_blocks=3)
    assert bits_equal(y, ya)


@pytest.mark.parametrize("rows,cols", [(8, 4096), (16, 14336), (3, 520), (5, 1001), (70, 1024)])
@pytest.mark.parametrize("in32,out32", [(True, False), (True, True), (False, False)])
def test_rmsnorm(rows, cols, in32, out32):
    """Rows that fit in registers (cols % 4 == 0, at most 4096) take the single-read kernel,
    the others the two-pass one."""
    x32 = inputs.normal_f32((rows, cols), 4, 3.0)
    if not in32:
        x32 = O.bf16_to_f64(inputs.to_bf16_bits(x32)).astype(np.float32)
    w = inputs.normal_f32((cols,), 5, 0.1, 1.0)
    ref = O.rmsnorm(x32.astype(np.float64), w.astype(np.float64), 1e-5)
    x = torch.from_numpy(x32).cuda()
    if not in32:
        x = x.to(torch.bfloat16)
    y = nan_like((rows, cols), torch.float32 if out32 else torch.bfloat16)
    op = B.rmsnorm_op(x, torch.from_numpy(w).cuda(), y, rows, cols, 1e-5)
    launch(op)
    if out32:
        assert np.abs(y.cpu().numpy().astype(np.float64) - ref).max() <= 2e-6 * max(1.0, np.abs(ref).max())
    else:
        bf16_close(y, ref)
    ya = nan_like(y.shape, y.dtype)
    launch(B.rmsnorm_op(x, torch.from_numpy(w).cuda(), ya, rows, cols, 1e-5), atom_blocks=2)
    assert bits_equal(y, ya)


@pytest.mark.parametrize("rows,cols", [(8, 4096), (300, 3072), (7, 1001)])
@pytest.mark.parametrize("in32,out32", [(False, False), (True, True), (True, False)])
def test_bias_gelu(rows, cols, in32, out32):
    x32 = inputs.normal_f32((rows, cols), 6, 2.0)
    bias = inputs.normal_f32((cols,), 7, 0.5)
    if in32:
        x, x64 = torch.from_numpy(x32).cuda(), x32.astype(np.float64)
    else:
        bits = inputs.to_bf16_bits(x32)
        x, x64 = dev_bits(bits), O.bf16_to_f64(bits)
    ref = O.bias_act(x64, bias.astype(np.float64), gelu=True)
    y = nan_like((rows, cols), torch.float32 if out32 else torch.bfloat16)
    total = launch(B.bias_act_op(x, y, rows, cols, torch.from_numpy(bias).cuda(), gelu=True))
    assert total == (rows * cols + 2047) // 2048
    if out32:
        f32_close(y, ref, 2e-6 * max(1.0, np.abs(ref).max()))
    else:
        # fp32 erf is good to ~2e-7 absolute, so GELU's far negative tail
        # (u/2 * (1 + erf) with 1 + erf ~ 1e-6) carries ~1e-6 absolute error
        bf16_close(y, ref, abs_tol=1e-6)
    ya = nan_like(y.shape, y.dtype)
    launch(B.bias_act_op(x, ya, rows, cols, torch.from_numpy(bias).cuda(), gelu=True), atom_blocks=2)
    assert bits_equal(y, ya)


@pytest.mark.parametrize("rows,n", [(1536, 128), (9, 2049), (4, 1000)])
def test_softmax(rows, n):
    s32 = inputs.normal_f32((rows, n), 8, 3.0)
    ref = O.softmax(s32.astype(np.float64) * 0.125)
    p = nan_like((rows, n), torch.float32)
    launch(B.softmax_op(torch.from_numpy(s32).cuda(), p, rows, n, scale=0.125))
    f32_close(p, ref, 2e-6)
    assert abs(float(p.sum(dim=1).max()) - 1.0) < 1e-5
    bits = inputs.to_bf16_bits(s32)
    pb = nan_like((rows, n), torch.bfloat16)
    launch(B.softmax_op(dev_bits(bits), pb, rows, n, scale=0.125), atom_blocks=5)
    bf16_close(pb, O.softmax(O.bf16_to_f64(bits) * 0.125))


@pytest.mark.parametrize("rows,f", [(8, 14336), (3, 1000)])
def test_silu_mul(rows, f):
    bits = inputs.normal_bits((rows, 2 * f), 9, 2.0)
    gu = O.bf16_to_f64(bits)
    ref = O.silu_mul(gu[:, :f], gu[:, f:])
    y = nan_like((rows, f), torch.bfloat16)
    launch(B.silu_mul_op(dev_bits(bits), y, rows, f), atom_blocks=4)
    bf16_close(y, ref)


@pytest.mark.parametrize("rows,n_q,n_kv,d,pos", [(4, 32, 8, 128, 2048), (3, 4, 2, 16, 5), (1, 8, 8, 64, 0)])
def test_rope_and_cache_append(rows, n_q, n_kv, d, pos):
    cap = pos + 1
    bits = inputs.normal_bits((rows, (n_q + 2 * n_kv) * d), 10)
    qkv = dev_bits(bits).clone()
    kc = torch.zeros((rows, cap, n_kv, d), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros((rows, cap, n_kv, d), dtype=torch.bfloat16, device="cuda")
    launch(B.rope_kv_op(qkv, kc, vc, rows, n_q, n_kv, d, pos, cap), atom_blocks=3)
    x = O.bf16_to_f64(bits)
    q = x[:, : n_q * d].reshape(rows, n_q, d)
    k = x[:, n_q * d:(n_q + n_kv) * d].reshape(rows, n_kv, d)
    v = x[:, (n_q + n_kv) * d:].reshape(rows, n_kv, d)
    positions = np.full((rows,), pos, dtype=np.int64)
    q_ref, k_ref = O.rope(q, positions), O.rope(k, positions)
    out = qkv.cpu().to(torch.float64).numpy()
    # fp32 angle arithmetic at position 2048 is good to ~1e-4 rad: allow 2 bf16 ulp there
    def close(g, r):
        r16 = O.round_bf16(r)
        assert np.all(np.abs(g - r16) <= np.abs(r16) * 2.0 ** -6 + 2e-3)
        assert (g == r16).mean() > 0.9
    close(out[:, : n_q * d].reshape(rows, n_q, d), q_ref)
    close(out[:, n_q * d:(n_q + n_kv) * d].reshape(rows, n_kv, d), k_ref)
    # cache slot `pos` holds exactly the rotated k and the untouched v; other slots stay zero
    assert torch.equal(kc[:, pos].reshape(rows, -1), qkv[:, n_q * d:(n_q + n_kv) * d])
    assert torch.equal(vc[:, pos].reshape(rows, -1), dev_bits(bits)[:, (n_q + n_kv) * d:])
    if pos > 0:
        assert float(kc[:, :pos].abs().max()) == 0.0 and float(vc[:, :pos].abs().max()) == 0.0


def test_row_ops_refuse_bad_arguments():
    x = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    y = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    bad = [
        B.layernorm_op(x, None, None, y, 4, 64),
        B.layernorm_op(x, x, x, y, 0, 64),
        B.layernorm_op(x, x, x, y, 4, 64, y_bf16=y),      # bf16 copy without fp32 main output
        B.rmsnorm_op(x, None, y, 4, 64),
        B.rope_kv_op(y, y, y, 1, 2, 1, 15, 0, 1),         # odd head width
        B.rope_kv_op(y, y, y, 1, 2, 1, 16, 3, 3),         # pos outside the cache
        B.make_op(99, (1, 1)),
    ]
    for op in bad:
        with pytest.raises(B.LithosError) as e:
            B.lithos_launch_atomized(ctx(), op)
        assert e.value.code == B.EINVAL
