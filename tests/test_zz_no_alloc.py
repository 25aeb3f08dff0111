"""The entry point that allocates nothing (split decode attention on the library's fixed workspace)
against the existing one (caller's workspace, ATTN_DEC then ATTN_MERGE): same bits, on two calls in a
row, the second with a smaller input that leaves part of the workspace holding the first call's data."""
import math

import numpy as np
import pytest
import torch

from oracle import ops as O
from paper_2504_15465_amd import binding as B
from paper_2504_15465_amd import inputs
from gpu_util import bits_equal, counters, ctx, dev_bits, nan_like

pytestmark = pytest.mark.gpu


def _case(batch, n_q, n_kv, keys, splits, seed):
    d, cap = 128, keys + 2
    qb = inputs.normal_bits((batch, n_q * d), [seed, 0])
    kb = inputs.normal_bits((batch, cap, n_kv, d), [seed, 1])
    vb = inputs.normal_bits((batch, cap, n_kv, d), [seed, 2])
    q, k, v = dev_bits(qb).float(), dev_bits(kb), dev_bits(vb)
    scale = 1 / math.sqrt(d)
    # existing entry point: caller's workspace, two launches
    ws = nan_like((B.attn_workspace_floats(batch, n_q, d, splits),), torch.float32)
    o_ref = nan_like((batch, n_q * d), torch.float32)
    torch.cuda.synchronize()
    B.lithos_launch_atomized(ctx(), B.attn_dec_op(q, k, v, o_ref, batch, n_q, n_kv, d, keys, cap, scale, splits=splits, workspace=ws),
                             (0, 0, 0), 3, None, None)
    B.lithos_launch_atomized(ctx(), B.attn_merge_op(ws, o_ref, batch, n_q, n_kv, d, splits), (0, 0, 0), 0, None, None)
    B.lithos_partition_sync(ctx(), None)
    # new entry point: no workspace argument
    o = nan_like((batch, n_q * d), torch.float32)
    op = B.attn_dec_op(q, k, v, o, batch, n_q, n_kv, d, keys, cap, scale, splits=splits)
    cnt = counters(batch * n_kv * splits)
    B.lithos_debug_block_counters(ctx(), cnt)
    torch.cuda.synchronize()
    try:
        B.lithos_launch_attn_dec_static(ctx(), op, 3, None, None)
        B.lithos_partition_sync(ctx(), None)
    finally:
        B.lithos_debug_block_counters(ctx(), None)
    assert cnt.cpu().tolist() == [1] * (batch * n_kv * splits)
    assert not torch.isnan(o).any()
    assert bits_equal(o, o_ref)
    ref = O.attention(O.bf16_to_f64(qb).reshape(batch, 1, n_q, d), O.bf16_to_f64(kb)[:, :keys], O.bf16_to_f64(vb)[:, :keys],
                      scale).reshape(batch, n_q * d)
    assert np.abs(o.cpu().numpy().astype(np.float64) - ref).max() <= 2e-5


def test_static_workspace_entry_point_matches_the_callers_workspace_one_twice_in_a_row():
    _case(4, 32, 8, 2049, 9, seed=71)        # 4*32*9*130 floats of the fixed workspace
    _case(2, 8, 4, 300, 5, seed=72)          # smaller: the rest still holds the first call's partials


def test_static_workspace_entry_point_on_a_partition_with_an_ordering_stream():
    batch, n_q, n_kv, d, keys, splits = 3, 8, 8, 128, 70, 2
    cap = keys
    q = dev_bits(inputs.normal_bits((batch, n_q * d), 73)).float()
    k, v = dev_bits(inputs.normal_bits((batch, cap, n_kv, d), 74)), dev_bits(inputs.normal_bits((batch, cap, n_kv, d), 75))
    ws = nan_like((B.attn_workspace_floats(batch, n_q, d, splits),), torch.float32)
    o_ref, o = nan_like((batch, n_q * d), torch.float32), nan_like((batch, n_q * d), torch.float32)
    part = B.lithos_create_partition(ctx(), B.lithos_make_mask(ctx(), 64))
    order = torch.cuda.Stream()
    try:
        torch.cuda.synchronize()
        B.lithos_launch_atomized(ctx(), B.attn_dec_op(q, k, v, o_ref, batch, n_q, n_kv, d, keys, cap, 0.1, splits=splits, workspace=ws),
                                 (0, 0, 0), 0, part, None)
        B.lithos_launch_atomized(ctx(), B.attn_merge_op(ws, o_ref, batch, n_q, n_kv, d, splits), (0, 0, 0), 0, part, None)
        B.lithos_partition_sync(ctx(), part)
        B.lithos_launch_attn_dec_static(ctx(), B.attn_dec_op(q, k, v, o, batch, n_q, n_kv, d, keys, cap, 0.1, splits=splits),
                                        0, part, order.cuda_stream)
        with torch.cuda.stream(order):
            snap = o.clone()                  # the caller's work on the ordering stream sees the result
        order.synchronize()
        assert bits_equal(snap, o_ref)
    finally:
        B.lithos_destroy_partition(part)


def test_static_workspace_entry_point_refuses_what_it_cannot_hold():
    x = torch.zeros((16, 32 * 128), dtype=torch.float32, device="cuda")
    kv = torch.zeros((16, 64, 8, 128), dtype=torch.bfloat16, device="cuda")
    too_big = B.attn_dec_op(x, kv, kv, x, 16, 32, 8, 128, 64, 64, 1.0, splits=64)       # 16*32*64*130 > 2^21 floats
    assert 16 * 32 * 64 * 130 > B.STATIC_SCRATCH_FLOATS
    with pytest.raises(B.LithosError) as e:
        B.lithos_launch_attn_dec_static(ctx(), too_big)
    assert e.value.code == B.ELIMIT and "workspace" in str(e.value)
    for bad in (B.attn_dec_op(x, kv, kv, x, 16, 32, 8, 128, 64, 64, 1.0, splits=1),                  # no workspace needed
                B.attn_dec_op(x, kv, kv, x, 16, 32, 8, 128, 64, 64, 1.0, splits=2, workspace=x),    # caller's workspace
                B.rmsnorm_op(x, x, x, 16, 4096)):                                                    # another operator
        with pytest.raises(B.LithosError) as e:
            B.lithos_launch_attn_dec_static(ctx(), bad)
        assert e.value.code == B.EINVAL
