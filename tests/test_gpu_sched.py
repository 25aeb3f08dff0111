"""Two tenants on CU-masked queues under the spatial scheduler: results stay
bit-exact while kernels are cut in atoms and CUs are stolen and handed back."""
import time

import numpy as np
import pytest
import torch

from paper_2504_15465_amd import binding as B
from paper_2504_15465_amd import inputs
from paper_2504_15465_amd.models import MlpChain, run_ops
from gpu_util import bits_equal, dev_bits, nan_like

pytestmark = pytest.mark.gpu


def make_world(cfg):
    c = B.lithos_init(0, cfg)
    p_hp = B.lithos_create_partition(c, B.lithos_make_mask(c, 64, B.MASK_STRIPED, 0))
    p_be = B.lithos_create_partition(c, B.lithos_make_mask(c, 192, B.MASK_STRIPED, 64))
    return c, p_hp, p_be


def drop_world(c, parts, tenants):
    for t in tenants:
        B.lithos_tenant_destroy(t)
    for p in parts:
        B.lithos_destroy_partition(p)
    B.lithos_shutdown(c)


@pytest.mark.parametrize("steal,atomize", [(1, 1), (1, 0), (0, 1), (0, 0)])
def test_stacked_tenants_bit_exact_and_stats(steal, atomize):
    cfg = B.Config.default(atom_duration_us=100.0, max_outstanding=2, max_outstanding_hp=16, steal=steal, atomize=atomize)
    c, p_hp, p_be = make_world(cfg)
    t_hp = B.lithos_tenant_create(c, B.CLASS_HP, p_hp)
    t_be = B.lithos_tenant_create(c, B.CLASS_BE, p_be)
    try:
        # best-effort: 4096^3 GEMM (256 tiles of 256x256), reference from a plain launch
        m = 4096
        a_bits, b_bits = inputs.gemm_operands(m, m, m, seed=4)
        a, b = dev_bits(a_bits), dev_bits(b_bits)
        c_ref = nan_like((m, m), torch.bfloat16)
        torch.cuda.synchronize()
        B.lithos_launch_atomized(c, B.gemm_op(a, b, c_ref, m, m, m, tile=256))
        B.lithos_partition_sync(c, None)
        c_be = nan_like((m, m), torch.bfloat16)
        be_op = B.gemm_op(a, b, c_be, m, m, m, tile=256)
        # high-priority: a small MLP
        layers = inputs.mlp_params(2, 1024, seed=1)
        x = inputs.mlp_requests(pool=1, batch=8, hidden=1024, seed=2)[0]
        chain = MlpChain(layers, 8)
        chain.set_input(x)
        run_ops(c, chain.ops(), p_hp)
        hp_ref = chain.out.clone()
        hp_ops = chain.ops()

        torch.cuda.synchronize()
        drv = B.lithos_drive_closed_loop_start(t_be, [be_op], depth=2)
        time.sleep(0.05)
        for i in range(30):
            chain.out.fill_(float("nan"))
            torch.cuda.synchronize()
            for op in hp_ops:
                B.lithos_submit(t_hp, op)
            B.lithos_sync(t_hp)
            assert bits_equal(chain.out, hp_ref), "request %d" % i
            time.sleep(0.002)
        iters, secs = B.lithos_drive_closed_loop_stop(drv)
        B.lithos_sync(t_be)
        assert iters >= 3
        assert bits_equal(c_be, c_ref)
        s_be, s_hp = B.lithos_tenant_stats(t_be), B.lithos_tenant_stats(t_hp)
        assert s_hp.kernels == 30 * len(hp_ops)
        assert s_be.kernels >= iters
        if atomize:
            assert s_be.atoms > s_be.kernels          # the long GEMM was cut
        else:
            assert s_be.atoms == s_be.kernels
        if steal and atomize:
            # a kernel's measured latency includes the wait for lent CUs to drain, so the predictor can
            # take a blocked microsecond kernel for a long one and cut its next instance: rare, harmless
            assert s_hp.kernels <= s_hp.atoms <= s_hp.kernels * 1.2
        else:
            assert s_hp.atoms == s_hp.kernels         # microsecond kernels stay whole
        if steal:
            assert s_be.stolen_atoms > 0              # idle high-priority CUs were lent
        else:
            assert s_be.stolen_atoms == 0 and s_hp.stolen_atoms == 0
        # a revocation is an inner atom boundary of a kernel: none without atoms or without lending
        assert s_be.revocations <= s_be.atoms - s_be.kernels
        if not (steal and atomize):
            assert s_be.revocations == 0 and s_hp.revocations == 0
        tot = B.lithos_stats(c)
        for f in ("kernels", "atoms", "stolen_atoms", "revocations", "predictions", "mispredicts"):
            assert getattr(tot, f) == getattr(s_be, f) + getattr(s_hp, f), f
    finally:
        drop_world(c, [p_hp, p_be], [t_hp, t_be])


def test_lent_cus_go_back_at_the_next_atom_boundary():
    """A long best-effort kernel runs on its quota plus the idle high-priority CUs; a high-priority kernel
    submitted in the middle of it gets them back at the next atom boundary, which the context counts as a
    revocation (Section 4.4 'Operation'); once the high-priority tenant is idle again they are lent again."""
    cfg = B.Config.default(atom_duration_us=100.0, max_outstanding=1, max_outstanding_hp=16, steal=1, atomize=1)
    c, p_hp, p_be = make_world(cfg)
    t_hp = B.lithos_tenant_create(c, B.CLASS_HP, p_hp)
    t_be = B.lithos_tenant_create(c, B.CLASS_BE, p_be)
    try:
        long_op = B.spin_op(16384, 5000)              # 50 us per block, 2 per CU: 32 waves on 256 CUs, > 1.6 ms
        tiny = B.spin_op(8, 100)
        for _ in range(3):                            # the predictor learns the kernel on the wide mask
            B.lithos_submit(t_be, long_op)
            B.lithos_sync(t_be)
        assert B.lithos_tenant_stats(t_be).revocations == 0
        seen = 0
        for attempt in range(5):
            before = B.lithos_tenant_stats(t_be)
            B.lithos_submit(t_be, long_op)
            time.sleep(0.0005)
            B.lithos_submit(t_hp, tiny)
            B.lithos_sync(t_hp)
            B.lithos_sync(t_be)
            after = B.lithos_tenant_stats(t_be)
            assert after.atoms - before.atoms >= 4    # the kernel was cut
            seen += after.revocations - before.revocations
            if seen:
                break
        assert 1 <= seen <= 2
        assert B.lithos_tenant_stats(t_hp).revocations == 0
        assert B.lithos_stats(c).revocations == seen
    finally:
        drop_world(c, [p_hp, p_be], [t_hp, t_be])


def test_open_loop_driver_and_passthrough_tenants():
    c = B.lithos_init(0, None)
    t_hp = B.lithos_tenant_create(c, B.CLASS_HP, None)       # pass-through: plain queue, no atoms
    try:
        ops = [B.spin_op(8, 1000)]                            # ~10 us per request
        arr = inputs.poisson_arrivals(2000.0, 200, seed=3)
        lat = B.lithos_drive_open_loop(t_hp, [ops], arr)
        assert lat.shape == (200,) and np.all(lat > 5.0) and np.median(lat) < 500.0
        s = B.lithos_tenant_stats(t_hp)
        assert s.kernels == 200 and s.atoms == 200
        tot = B.lithos_stats(c)                                # pass-through kernels count in the context totals
        assert tot.kernels == 200 and tot.atoms == 200 and tot.stolen_atoms == 0 and tot.revocations == 0
    finally:
        B.lithos_tenant_destroy(t_hp)
        B.lithos_shutdown(c)


def test_overlapping_quotas_and_shutdown_with_tenants_are_refused():
    c = B.lithos_init(0, None)
    p1 = B.lithos_create_partition(c, B.lithos_make_mask(c, 64, B.MASK_STRIPED, 0))
    p2 = B.lithos_create_partition(c, B.lithos_make_mask(c, 64, B.MASK_STRIPED, 32))
    t1 = B.lithos_tenant_create(c, B.CLASS_HP, p1)
    try:
        with pytest.raises(B.LithosError) as e:
            B.lithos_tenant_create(c, B.CLASS_BE, p2)
        assert e.value.code == B.EMASK
        with pytest.raises(B.LithosError) as e:
            B.lithos_shutdown(c)
        assert e.value.code == B.ESTATE
        with pytest.raises(B.LithosError):
            B.lithos_submit(t1, B.make_op(99, (1, 1)))
    finally:
        B.lithos_tenant_destroy(t1)
        B.lithos_destroy_partition(p1)
        B.lithos_destroy_partition(p2)
        B.lithos_shutdown(c)


def test_tenant_queues_do_not_share_a_command_processor_pipe():
    """Queues created a multiple of the pipe count apart delay each other while a grid
    is partly dispatched; tenant creation must hand out independent queues."""
    c = B.lithos_init(0, None)
    parts = [B.lithos_create_partition(c, B.lithos_make_mask(c, 24, B.MASK_STRIPED, 24 * i)) for i in range(9)]
    try:
        coupled = [B.lithos_partitions_coupled(c, parts[0], parts[j]) for j in range(1, 9)]
        assert any(coupled), "expected at least one of 8 later queues to share a pipe with the first"
        assert not all(coupled)
        # tenants on partitions 0 and the first coupled one: creation must decouple them
        j = 1 + coupled.index(True)
        t0 = B.lithos_tenant_create(c, B.CLASS_HP, parts[0])
        t1 = B.lithos_tenant_create(c, B.CLASS_BE, parts[j])
        try:
            assert not B.lithos_partitions_coupled(c, parts[0], parts[j])
            assert not B.lithos_partitions_coupled(c, parts[j], parts[0])
        finally:
            B.lithos_tenant_destroy(t0)
            B.lithos_tenant_destroy(t1)
    finally:
        for p in parts:
            B.lithos_destroy_partition(p)
        B.lithos_shutdown(c)


def test_three_tenants_bit_exact_with_stealing_between_all_of_them():
    """Two high-priority tenants (128 and 64 CUs) and a best-effort tenant (64 CUs): every tenant's results
    equal its solo results bit for bit while CUs move between all three at atom boundaries."""
    cfg = B.Config.default(atom_duration_us=100.0, max_outstanding=2, max_outstanding_hp=16, steal=1, atomize=1)
    c = B.lithos_init(0, cfg)
    parts = [B.lithos_create_partition(c, B.lithos_make_mask(c, n, B.MASK_STRIPED, first)) for n, first in ((128, 0), (64, 128), (64, 192))]
    ts = [B.lithos_tenant_create(c, cls, p) for cls, p in zip((B.CLASS_HP, B.CLASS_HP, B.CLASS_BE), parts)]
    try:
        m = 4096
        a_bits, b_bits = inputs.gemm_operands(m, m, m, seed=4)
        a, b = dev_bits(a_bits), dev_bits(b_bits)
        c_ref, c_be = nan_like((m, m), torch.bfloat16), nan_like((m, m), torch.bfloat16)
        torch.cuda.synchronize()
        B.lithos_launch_atomized(c, B.gemm_op(a, b, c_ref, m, m, m, tile=256))
        B.lithos_partition_sync(c, None)
        be_op = B.gemm_op(a, b, c_be, m, m, m, tile=256)
        chains = []
        for seed in (1, 5):
            ch = MlpChain(inputs.mlp_params(2, 1024, seed=seed), 8)
            ch.set_input(inputs.mlp_requests(pool=1, batch=8, hidden=1024, seed=seed + 1)[0])
            run_ops(c, ch.ops(), parts[0])
            chains.append((ch, ch.out.clone(), ch.ops()))
        torch.cuda.synchronize()
        drv = B.lithos_drive_closed_loop_start(ts[2], [be_op], depth=2)
        time.sleep(0.05)
        for i in range(20):
            for ch, _, _ in chains:
                ch.out.fill_(float("nan"))
            torch.cuda.synchronize()
            for t, (ch, ref, ops) in zip(ts[:2], chains):
                for op in ops:
                    B.lithos_submit(t, op)
            for t, (ch, ref, ops) in zip(ts[:2], chains):
                B.lithos_sync(t)
                assert bits_equal(ch.out, ref), "request %d" % i
            time.sleep(0.002)
        iters, _ = B.lithos_drive_closed_loop_stop(drv)
        B.lithos_sync(ts[2])
        assert iters >= 3 and bits_equal(c_be, c_ref)
        st = [B.lithos_tenant_stats(t) for t in ts]
        assert st[0].kernels == 20 * len(chains[0][2]) and st[1].kernels == 20 * len(chains[1][2])
        assert st[2].stolen_atoms > 0 and st[2].atoms > st[2].kernels
    finally:
        drop_world(c, parts, ts)


def test_online_right_sizing_borrows_only_when_it_pays():
    """Section 4.5 'Operation' in the dispatcher.  A tenant with a 64-CU quota beside an idle tenant that
    owns 192: a kernel that cannot fill more than 64 CUs never borrows (occupancy filter); a kernel that
    scales borrows, after one run on each CU set has given the model its two points."""
    cfg = B.Config.default(atom_duration_us=1e6, max_outstanding=2, steal=1, atomize=1, rightsize_slip=1.1)
    c, p_a, p_b = make_world(cfg)
    t_a = B.lithos_tenant_create(c, B.CLASS_BE, p_a)       # 64 CUs
    t_b = B.lithos_tenant_create(c, B.CLASS_HP, p_b)       # 192 CUs, never submits
    try:
        small = B.spin_op(128, 2000)                        # two blocks per CU: fills exactly 64 CUs
        for _ in range(4):
            B.lithos_submit(t_a, small)
            B.lithos_sync(t_a)
        s = B.lithos_tenant_stats(t_a)
        assert s.kernels == 4 and s.stolen_atoms == 0 and s.rightsized_kernels == 4
        # the scaling kernel follows the small one in every batch, so it has its own ordinal (the
        # predictor is keyed by a kernel's position since the last synchronisation, Section 4.7)
        big = B.spin_op(4096, 4000)                         # 32 waves on 64 CUs, 8 on 256: scales
        t = []
        for _ in range(5):
            t0 = time.perf_counter()
            B.lithos_submit(t_a, small)
            B.lithos_submit(t_a, big)
            B.lithos_sync(t_a)
            t.append(time.perf_counter() - t0)
        s2 = B.lithos_tenant_stats(t_a)
        assert s2.kernels - s.kernels == 10
        assert s2.rightsized_kernels - s.rightsized_kernels == 5 + 1  # the small ones, and the one run that gave the second point
        assert s2.stolen_atoms - s.stolen_atoms == 4                  # first run (nothing known) and the three after the fit
        assert t[1] > 2.5 * t[0] and t[4] < 0.5 * t[1]                # 64 CUs take four times as long as 256
        assert B.lithos_stats(c).rightsized_kernels == 10
    finally:
        drop_world(c, [p_a, p_b], [t_a, t_b])
