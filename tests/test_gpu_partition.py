"""CU-masked queues: a masked launch stays inside its CUs, disjoint masks use
disjoint CUs, every die is covered, and the right-size sweep returns a curve."""
import numpy as np
import pytest
import torch

from oracle import ops as O
from oracle import rightsize as R
from paper_2504_15465_amd import binding as B
from paper_2504_15465_amd import inputs
from gpu_util import bits_equal, counters, ctx, dev_bits, nan_like, rel_fro

pytestmark = pytest.mark.gpu


def cu_ids(xcd, hwid):
    """(die, shader engine, array, CU) from the hardware id register."""
    return set(zip(xcd.tolist(), ((hwid >> 13) & 7).tolist(), ((hwid >> 12) & 1).tolist(), ((hwid >> 8) & 15).tolist()))


def test_device_shape():
    info = B.lithos_device_info(ctx())
    assert info.n_cu == 256 and info.n_xcd == 8 and info.cu_per_xcd == 32
    assert info.arch.decode().startswith("gfx950")


def test_masked_launch_stays_in_its_cus_and_masks_are_disjoint():
    c = ctx()
    m_hp = B.lithos_make_mask(c, 64, B.MASK_STRIPED, 0)
    m_be = B.lithos_make_mask(c, 192, B.MASK_STRIPED, 64)
    assert not np.any(m_hp & m_be)
    assert sum(bin(int(w)).count("1") for w in m_hp) == 64
    p_hp, p_be = B.lithos_create_partition(c, m_hp), B.lithos_create_partition(c, m_be)
    try:
        assert B.lithos_partition_cus(p_hp) == 64 and B.lithos_partition_cus(p_be) == 192
        x1, h1 = B.lithos_probe_partition(c, p_hp, 4096)
        x2, h2 = B.lithos_probe_partition(c, p_be, 8192)
        x0, h0 = B.lithos_probe_partition(c, None, 8192)
        s1, s2, s0 = cu_ids(x1, h1), cu_ids(x2, h2), cu_ids(x0, h0)
        assert len(s1) <= 64 and len(s2) <= 192 and len(s0) <= 256
        assert len(s1) >= 56 and len(s2) >= 170          # nearly every CU of the mask was used
        assert not (s1 & s2)                              # disjoint masks -> disjoint CUs
        assert s1 <= s0 and s2 <= s0
        # striped masks put the same number of CUs on every die
        for s, per_die in ((s1, 8), (s2, 24)):
            by_die = {}
            for die, *_ in s:
                by_die[die] = by_die.get(die, 0) + 1
            assert sorted(by_die) == list(range(8))
            assert max(by_die.values()) <= per_die
    finally:
        B.lithos_destroy_partition(p_hp)
        B.lithos_destroy_partition(p_be)


def test_masks_that_empty_a_die_or_are_empty_are_refused():
    c = ctx()
    with pytest.raises(B.LithosError) as e:
        B.lithos_create_partition(c, [0] * 8)
    assert e.value.code == B.EMASK
    whole = B.lithos_make_mask(c, 32, B.MASK_WHOLE_XCD, 0)     # all of die 0, nothing elsewhere
    with pytest.raises(B.LithosError) as e:
        B.lithos_create_partition(c, whole)
    assert e.value.code == B.EMASK
    with pytest.raises(B.LithosError):
        B.lithos_make_mask(c, 300)
    with pytest.raises(B.LithosError):
        B.lithos_make_mask(c, 8, B.MASK_STRIPED, 252)


def test_rightsize_sweep_on_a_spin_kernel_and_selection_rule():
    """512 blocks, two fit on a CU, each holds its slot for 50 us: latency ~ 50 us * ceil(512/(2 CUs))."""
    c = ctx()
    op = B.spin_op(512, 5000)
    r = B.lithos_rightsize(c, op, 32, 256, 32, 2, 7, 0.04)
    cus = list(r.cus[: r.n_points])
    lat = list(r.median_us[: r.n_points])
    assert cus == list(range(32, 257, 32))
    assert 40.0 < lat[-1] < 120.0                       # one wave of blocks on the full GPU
    assert lat[0] > 5 * lat[-1]                         # 32 CUs need 8 waves
    assert r.chosen_cus == R.select_from_sweep(cus, lat, 0.04)
    assert r.occupancy_bound_cus == 256
    m, b = r.model_m, r.model_b
    assert abs(m / cus[0] + b - lat[0]) < 1e-6 * lat[0] and abs(m / cus[-1] + b - lat[-1]) < 1e-6 * lat[-1]
    # the model's pick is the oracle's, from the oracle's own fit through the measured end points
    mo, bo = R.fit_through(cus[0], lat[0], cus[-1], lat[-1])
    assert abs(mo - m) <= 1e-9 * abs(m) and abs(bo - b) <= 1e-6 * max(1.0, abs(b))
    assert r.model_cus == R.min_units_for_slip(mo, bo, cus[-1], 1.04)
    assert r.online_cus == r.model_cus                  # the kernel can fill all 256 CUs: the model decides
    small = B.lithos_rightsize(c, B.spin_op(64, 5000), 32, 256, 32, 1, 3, 0.04)
    assert small.occupancy_bound_cus == R.occupancy_bound(64, 2) == 32
    assert small.online_cus == 32                       # 64 blocks, two per CU: the occupancy filter decides
    with pytest.raises(B.LithosError):
        B.lithos_rightsize(c, op, 8, 512, 8, 1, 3, 0.04)


def test_prelude_form_of_algorithm_1_gives_the_same_bits():
    """Every atom launches the whole grid and blocks outside its range leave at once (the paper's
    Prelude): same results bit for bit as the remapping form, each block still runs exactly once."""
    from paper_2504_15465_amd.models import MlpChain, run_ops
    m, n, k = 520, 776, 320
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=3)
    a, b = dev_bits(a_bits), dev_bits(b_bits)
    outs = {}
    for prelude in (0, 1):
        c = B.lithos_init(0, B.Config.default(prelude=prelude))
        part = B.lithos_create_partition(c, B.lithos_make_mask(c, 64))
        try:
            for tile, atom_blocks in ((64, 7), (256, 1), (128, 0)):
                out = nan_like((m, n), torch.float32)
                op = B.gemm_op(a, b, out, m, n, k, tile=tile)
                grid, _ = B.lithos_op_grid(c, op)
                cnt = counters(grid[0] * grid[1])
                B.lithos_debug_block_counters(c, cnt)
                torch.cuda.synchronize()
                B.lithos_launch_atomized(c, op, (0, 0, 0), atom_blocks, part, None)
                B.lithos_partition_sync(c, part)
                B.lithos_debug_block_counters(c, None)
                assert cnt.cpu().tolist() == [1] * (grid[0] * grid[1])
                outs[(prelude, tile)] = out
            chain = MlpChain(inputs.mlp_params(2, 1024, seed=1), 8)          # row kernels and the skinny GEMM
            chain.set_input(inputs.mlp_requests(pool=1, batch=8, hidden=1024, seed=2)[0])
            run_ops(c, chain.ops(), part, atom_blocks=3)
            outs[(prelude, "mlp")] = chain.out.clone()
        finally:
            B.lithos_destroy_partition(part)
            B.lithos_shutdown(c)
    for key in ((64,), (256,), (128,), ("mlp",)):
        assert bits_equal(outs[(0,) + key], outs[(1,) + key])
    assert rel_fro(outs[(1, 256)], O.gemm(a_bits, b_bits)) <= 1e-4


@pytest.mark.parametrize("xcd_remap,prelude", [(1, 0), (0, 0), (1, 1)])
def test_random_grids_atom_sizes_and_partitions_run_every_block_once_with_the_same_bits(xcd_remap, prelude):
    """Seeded random GEMM shapes (ragged), tiles, atom sizes (1 block up to more than the grid, not
    dividing it) and partition sizes: each logical block exactly once, and the bits of a whole launch on
    the full device, whatever the remapping inside an atom and whichever form of Algorithm 1 is used."""
    import random
    rnd = random.Random(17 + 2 * xcd_remap + prelude)
    base = B.lithos_init(0, None)
    c = B.lithos_init(0, B.Config.default(xcd_remap=xcd_remap, prelude=prelude))
    parts = {n: B.lithos_create_partition(c, B.lithos_make_mask(c, n)) for n in (8, 40, 64, 256)}
    try:
        for case in range(10):
            tile = rnd.choice([64, 64, 128, 256])
            m, n = rnd.randrange(8, 1400, 8), rnd.randrange(8, 1400, 8)
            k = rnd.randrange(64, 640, 64) if tile == 256 else rnd.randrange(8, 520, 8)
            a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=100 + case)
            a, b = dev_bits(a_bits), dev_bits(b_bits)
            whole = nan_like((m, n), torch.float32)
            torch.cuda.synchronize()
            B.lithos_launch_atomized(base, B.gemm_op(a, b, whole, m, n, k, tile=tile), (0, 0, 0), 0, None, None)
            B.lithos_partition_sync(base, None)
            out = nan_like((m, n), torch.float32)
            op = B.gemm_op(a, b, out, m, n, k, tile=tile)
            grid, _ = B.lithos_op_grid(c, op)
            total = grid[0] * grid[1] * grid[2]
            atom_blocks = rnd.choice([1, 2, 3, 5, 7, 13, max(1, total - 1), total + 5, rnd.randint(1, total)])
            part = parts[rnd.choice([8, 40, 64, 256])]
            cnt = counters(total)
            B.lithos_debug_block_counters(c, cnt)
            try:
                B.lithos_launch_atomized(c, op, (0, 0, 0), atom_blocks, part, None)
                B.lithos_partition_sync(c, part)
            finally:
                B.lithos_debug_block_counters(c, None)
            assert cnt.cpu().tolist() == [1] * total, (case, m, n, k, tile, atom_blocks)
            assert bits_equal(out, whole), (case, m, n, k, tile, atom_blocks)
    finally:
        for p in parts.values():
            B.lithos_destroy_partition(p)
        B.lithos_shutdown(c)
        B.lithos_shutdown(base)


def test_ordering_stream_chains_launches_on_different_partitions():
    """Kernels of one chain launched on queues with different CU masks, ordered through a stream of the
    caller's: same bits as the chain on one queue, and the caller's own work on that stream runs after."""
    from paper_2504_15465_amd.models import MlpChain, run_ops
    c = ctx()
    parts = [B.lithos_create_partition(c, B.lithos_make_mask(c, n, B.MASK_STRIPED, first)) for n, first in ((64, 0), (128, 64), (32, 192))]
    try:
        chain = MlpChain(inputs.mlp_params(4, 1024, seed=1), 8)
        chain.set_input(inputs.mlp_requests(pool=1, batch=8, hidden=1024, seed=2)[0])
        ops = chain.ops()
        run_ops(c, ops, parts[0])
        ref = chain.out.clone()
        order = torch.cuda.Stream()
        assert order.cuda_stream != 0
        for rep in range(5):
            chain.out.fill_(float("nan"))
            torch.cuda.synchronize()
            for i, op in enumerate(ops):
                B.lithos_launch_atomized(c, op, (0, 0, 0), 2 if i % 3 == 0 else 0, parts[i % 3], order.cuda_stream)
            with torch.cuda.stream(order):
                snap = chain.out.clone()          # the caller's own work on the ordering stream
            order.synchronize()
            assert bits_equal(snap, ref), "repetition %d" % rep
    finally:
        for p in parts:
            B.lithos_destroy_partition(p)


def test_two_threads_launch_on_one_context_with_their_own_ordering_streams():
    """lithos_launch_atomized is serialised inside the library: two host threads, each chaining its
    kernels over two partitions through its own stream, get the bits of the single-queue runs."""
    import threading
    from paper_2504_15465_amd.models import MlpChain, run_ops
    c = ctx()
    parts = [B.lithos_create_partition(c, B.lithos_make_mask(c, 64, B.MASK_STRIPED, first)) for first in (0, 64, 128, 192)]
    try:
        chains, refs = [], []
        for i in range(2):
            ch = MlpChain(inputs.mlp_params(3, 1024, seed=1 + i), 8)
            ch.set_input(inputs.mlp_requests(pool=1, batch=8, hidden=1024, seed=2 + i)[0])
            run_ops(c, ch.ops(), parts[0])
            chains.append(ch)
            refs.append(ch.out.clone())
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        torch.cuda.synchronize()
        bad = []

        def work(i):
            ops = chains[i].ops()
            for rep in range(40):
                for j, op in enumerate(ops):
                    B.lithos_launch_atomized(c, op, (0, 0, 0), 3 if j % 2 else 0, parts[2 * i + j % 2], streams[i].cuda_stream)
                with torch.cuda.stream(streams[i]):
                    snap = chains[i].out.clone()
                streams[i].synchronize()
                if not bits_equal(snap, refs[i]):
                    bad.append((i, rep))
        th = [threading.Thread(target=work, args=(i,)) for i in range(2)]
        [t.start() for t in th]
        [t.join() for t in th]
        assert not bad, bad[:5]
    finally:
        for p in parts:
            B.lithos_destroy_partition(p)
