"""GPU parity of the atomized bf16 GEMM against the fp64 oracle (C-ABI calls)."""
import numpy as np
import pytest
import torch

from oracle import atoms as A
from oracle import ops as O
from paper_2504_15465_amd import binding as B
from paper_2504_15465_amd import inputs
from gpu_util import bits_equal, bf16_close, counters, ctx, dev_bits, nan_like, rel_fro

pytestmark = pytest.mark.gpu

FRO_TOL = 1e-4      # per-GEMM bar: relative Frobenius error vs fp64 accumulation on the same bf16 inputs


def run_gemm(a_bits, b_bits, m, n, k, ta=False, tb=False, tile=0, atom_blocks=0, part=None, out_dtype=torch.float32,
             bias=None, gelu=False, residual=None, count=False):
    c = nan_like((m, n), out_dtype)
    a, b = dev_bits(a_bits), dev_bits(b_bits)
    op = B.gemm_op(a, b, c, m, n, k, ta=ta, tb=tb, tile=tile, bias=bias, gelu=gelu, residual=residual)
    grid, _ = B.lithos_op_grid(ctx(), op)
    cnt = None
    if count:
        cnt = counters(grid[0] * grid[1] * grid[2])
        B.lithos_debug_block_counters(ctx(), cnt)
    torch.cuda.synchronize()        # torch's fills/copies run on its own stream
    try:
        B.lithos_launch_atomized(ctx(), op, (0, 0, 0), atom_blocks, part, None)
        B.lithos_partition_sync(ctx(), part)
    finally:
        B.lithos_debug_block_counters(ctx(), None)
    return c, grid, cnt


def test_config1_single_atomized_gemm():
    """512^3, U[-1,1] seed 0, 64x64 tiles = 64 blocks, 8 atoms of 8 on a 32-CU mask."""
    m = n = k = 512
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=0)
    part = B.lithos_create_partition(ctx(), B.lithos_make_mask(ctx(), 32))
    try:
        c_atom, grid, cnt = run_gemm(a_bits, b_bits, m, n, k, tile=64, atom_blocks=8, part=part, count=True)
        assert grid == (8, 8, 1)
        assert len(A.decompose(grid, 8)) == 8
        assert cnt.cpu().tolist() == [1] * 64                     # every block exactly once
        c_full, _, _ = run_gemm(a_bits, b_bits, m, n, k, tile=64, atom_blocks=0, part=part)
        assert bits_equal(c_atom, c_full)                         # bit-exact vs the unatomized launch
        c_nomask, _, _ = run_gemm(a_bits, b_bits, m, n, k, tile=64, atom_blocks=0, part=None)
        assert bits_equal(c_atom, c_nomask)
        ref = O.gemm(a_bits, b_bits)
        assert rel_fro(c_atom, ref) <= FRO_TOL
    finally:
        B.lithos_destroy_partition(part)


@pytest.mark.parametrize("tile", [64, 128, 256])
@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False), (True, True)])
def test_tiles_layouts_ragged_shapes(tile, ta, tb):
    # several tiles in each direction plus a ragged tail in M, N and K
    m, n, k = (200, 328, 136) if tile == 64 else (392, 520, 200) if tile == 128 else (520, 776, 264)
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=tile + 2 * ta + tb, ta=ta, tb=tb)
    ref = O.gemm(a_bits, b_bits, ta=ta, tb=tb)
    c_full, grid, _ = run_gemm(a_bits, b_bits, m, n, k, ta, tb, tile)
    assert not torch.isnan(c_full).any()
    assert rel_fro(c_full, ref) <= FRO_TOL
    total = grid[0] * grid[1]
    for atom_blocks in (1, 3, total - 1):
        c_atom, _, cnt = run_gemm(a_bits, b_bits, m, n, k, ta, tb, tile, atom_blocks=atom_blocks, count=True)
        assert cnt.cpu().tolist() == [1] * total
        assert bits_equal(c_atom, c_full)


@pytest.mark.parametrize("m,n,k", [(520, 776, 320), (256, 256, 64), (300, 260, 128), (1, 8, 192)])
def test_nt_256_tile_with_k_multiple_of_64(m, n, k):
    """A [M,K] times B [N,K] with 256x256 tiles and K % 64 == 0 takes the kernel that loads
    global memory straight into LDS: odd and even numbers of k-tiles, ragged M and N."""
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=77, tb=True)
    ref = O.gemm(a_bits, b_bits, tb=True)
    c_full, grid, _ = run_gemm(a_bits, b_bits, m, n, k, False, True, 256)
    assert not torch.isnan(c_full).any()
    assert rel_fro(c_full, ref) <= FRO_TOL
    total = grid[0] * grid[1]
    for atom_blocks in sorted({1, max(1, total - 1)}):
        c_atom, _, cnt = run_gemm(a_bits, b_bits, m, n, k, False, True, 256, atom_blocks=atom_blocks, count=True)
        assert cnt.cpu().tolist() == [1] * total
        assert bits_equal(c_atom, c_full)


@pytest.mark.parametrize("ta,tb", [(False, False), (True, False), (True, True)])
@pytest.mark.parametrize("m,n,k", [(520, 776, 320), (256, 256, 64), (304, 264, 128), (8, 8, 192)])
def test_256_tile_k_strided_operands_read_through_transposing_lds_loads(ta, tb, m, n, k):
    """256x256 tiles with K % 64 == 0 and an operand stored [K,rows]: the tile lies in LDS as in
    memory and the fragments come from the transposing LDS load; ragged M and N, bf16 and fp32 C."""
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=78 + 2 * ta + tb, ta=ta, tb=tb)
    ref = O.gemm(a_bits, b_bits, ta=ta, tb=tb)
    c_full, grid, _ = run_gemm(a_bits, b_bits, m, n, k, ta, tb, 256)
    assert not torch.isnan(c_full).any()
    assert rel_fro(c_full, ref) <= FRO_TOL
    total = grid[0] * grid[1]
    for atom_blocks in sorted({1, max(1, total - 1)}):
        c_atom, _, cnt = run_gemm(a_bits, b_bits, m, n, k, ta, tb, 256, atom_blocks=atom_blocks, count=True)
        assert cnt.cpu().tolist() == [1] * total
        assert bits_equal(c_atom, c_full)
    c16, _, _ = run_gemm(a_bits, b_bits, m, n, k, ta, tb, 256, out_dtype=torch.bfloat16)
    bf16_close(c16, ref, abs_tol=2.0 ** -22 * k)


def test_exactly_representable_data_matches_oracle_bit_for_bit():
    rng = np.random.default_rng(1)
    vals = np.array([1, -1, .5, -.5, 2, -2], np.float32)
    m, n, k = 256, 192, 512
    a = vals[rng.integers(0, 6, (m, k))]
    b = vals[rng.integers(0, 6, (k, n))]
    a_bits, b_bits = inputs.to_bf16_bits(a), inputs.to_bf16_bits(b)
    ref = O.gemm(a_bits, b_bits)
    for tile in (64, 128, 256):
        c, _, _ = run_gemm(a_bits, b_bits, m, n, k, tile=tile)
        assert np.array_equal(c.cpu().numpy().astype(np.float64), ref)
    ones_a = inputs.to_bf16_bits(np.ones((64, 1024), np.float32))
    ones_b = inputs.to_bf16_bits(np.ones((1024, 64), np.float32))
    c, _, _ = run_gemm(ones_a, ones_b, 64, 64, 1024, tile=64)
    assert bool((c == 1024.0).all())


@pytest.mark.parametrize("tile,tb,k", [(64, False, 264), (128, True, 264), (B.TILE_SKINNY, True, 264),
                                       (256, False, 320), (256, True, 320), (256, False, 264)])
def test_fused_epilogue_bias_gelu_residual(tile, tb, k):
    """Bias, GELU and residual in the epilogue, fp32 and bf16 C; full tiles (through LDS, or 16 bytes per
    lane for fp32) and ragged edge tiles (element by element) must agree with the oracle alike."""
    m, n = (24, 200) if tile == B.TILE_SKINNY else (136, 200) if tile < 256 else (520, 776)
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=9, tb=tb)
    bias = inputs.normal_f32((n,), 10, 0.5)
    resid = inputs.normal_f32((m, n), 11, 1.0)
    acc = O.gemm(a_bits, b_bits, tb=tb)
    ref = O.bias_act(acc, bias.astype(np.float64), gelu=True) + resid.astype(np.float64)
    bias_d, resid_d = torch.from_numpy(bias).cuda(), torch.from_numpy(resid).cuda()
    c32, _, _ = run_gemm(a_bits, b_bits, m, n, k, tb=tb, tile=tile, bias=bias_d, gelu=True, residual=resid_d)
    assert np.abs(c32.cpu().numpy().astype(np.float64) - ref).max() <= 2e-4 * max(1.0, np.abs(ref).max())
    c16, _, _ = run_gemm(a_bits, b_bits, m, n, k, tb=tb, tile=tile, bias=bias_d, gelu=True, residual=resid_d,
                         out_dtype=torch.bfloat16)
    bf16_close(c16, ref, abs_tol=2.0 ** -22 * k)
    c16a, _, _ = run_gemm(a_bits, b_bits, m, n, k, tb=tb, tile=tile, bias=bias_d, gelu=True, residual=resid_d,
                          out_dtype=torch.bfloat16, atom_blocks=2)
    assert bits_equal(c16, c16a)


@pytest.mark.parametrize("m", [1, 8, 13, 16, 32])
@pytest.mark.parametrize("n,k", [(4096, 4096), (1000, 520)])
def test_skinny_weight_streaming_gemm(m, n, k):
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=m, tb=True, dist="normal")
    ref = O.gemm(a_bits, b_bits, tb=True)
    c, grid, cnt = run_gemm(a_bits, b_bits, m, n, k, tb=True, tile=B.TILE_SKINNY, count=True)
    assert grid == ((n + 31) // 32, 1, 1)
    assert cnt.cpu().tolist() == [1] * grid[0]
    assert not torch.isnan(c).any()
    assert rel_fro(c, ref) <= FRO_TOL
    c_atom, _, _ = run_gemm(a_bits, b_bits, m, n, k, tb=True, tile=B.TILE_SKINNY, atom_blocks=7)
    assert bits_equal(c, c_atom)
    # auto selection picks the same kernel for small M with a [N,K] weight
    c_auto, grid_auto, _ = run_gemm(a_bits, b_bits, m, n, k, tb=True, tile=0)
    assert grid_auto == grid and bits_equal(c, c_auto)


def _launch(op, atom_blocks=0):
    torch.cuda.synchronize()
    B.lithos_launch_atomized(ctx(), op, (0, 0, 0), atom_blocks, None, None)
    B.lithos_partition_sync(ctx(), None)


@pytest.mark.parametrize("m", [1, 2, 3, 6, 7, 8, 9, 14, 16])
@pytest.mark.parametrize("n,k", [(4096, 4096), (1000, 520)])
@pytest.mark.parametrize("norm", ["ln", "rms"])
def test_weight_streaming_gemm_normalises_its_rows_on_load(m, n, k, norm):
    """GEMM with NORM_LN / NORM_RMS against the oracle's row kernel followed by its GEMM (the row counts
    on both sides of every kernel variant's limit)."""
    from paper_2504_15465_amd.models import norm_colsums
    rng = np.random.default_rng(100 * m + k)
    _, w_bits = inputs.gemm_operands(m, n, k, seed=m + 3, tb=True, dist="normal")
    x = (0.4 + 1.3 * rng.standard_normal((m, k))).astype(np.float32)     # a mean well away from zero
    gamma = (1.0 + 0.2 * rng.standard_normal(k)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(k)).astype(np.float32)
    eps = 1e-5
    xn = O.layernorm(x, gamma, beta, eps) if norm == "ln" else O.rmsnorm(x, gamma, eps)
    ref = O.gemm(xn, w_bits, tb=True)
    xd, wd = torch.from_numpy(x).cuda(), dev_bits(w_bits)
    gd, bd = torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda()
    c = nan_like((m, n), torch.float32)
    cs = norm_colsums(ctx(), gd, bd, wd) if norm == "ln" else None
    if cs is not None:       # the column sums are the oracle's products of gamma and beta with the weights
        assert rel_fro(cs, O.gemm(np.stack([gamma, beta]).astype(np.float64), w_bits, tb=True)) <= FRO_TOL
    op = B.gemm_op(xd, wd, c, m, n, k, tb=True, norm_gamma=gd, norm_colsums=cs, norm_eps=eps)
    grid, _ = B.lithos_op_grid(ctx(), op)
    assert grid == ((n + 31) // 32, 1, 1)
    _launch(op)
    assert not torch.isnan(c).any()
    assert rel_fro(c, ref) <= FRO_TOL
    # the row kernel followed by the plain GEMM agrees to fp32 rounding of the statistics
    xn_d = nan_like((m, k), torch.float32)
    _launch(B.layernorm_op(xd, gd, bd, xn_d, m, k, eps) if norm == "ln" else B.rmsnorm_op(xd, gd, xn_d, m, k, eps))
    c2 = nan_like((m, n), torch.float32)
    _launch(B.gemm_op(xn_d, wd, c2, m, n, k, tb=True))
    assert rel_fro(c, c2.double().cpu().numpy()) <= 1e-5
    c_atom = nan_like((m, n), torch.float32)
    _launch(B.gemm_op(xd, wd, c_atom, m, n, k, tb=True, norm_gamma=gd, norm_colsums=cs, norm_eps=eps), 5)
    assert bits_equal(c, c_atom)


@pytest.mark.parametrize("m", [1, 4, 7, 16])
@pytest.mark.parametrize("f,k", [(2048, 1024), (1000, 520)])
@pytest.mark.parametrize("a32,rms", [(True, True), (True, False), (False, False)])
def test_weight_streaming_gemm_with_gated_epilogue(m, f, k, a32, rms):
    """GLU: [2F,K] weights (gate rows, then up rows) -> silu(x gate^T) * (x up^T), optionally RMS-normalised x."""
    rng = np.random.default_rng(7 * m + f)
    a_bits, w_bits = inputs.gemm_operands(m, 2 * f, k, seed=m + 11, tb=True, dist="normal")
    gamma = (1.0 + 0.2 * rng.standard_normal(k)).astype(np.float32)
    if a32:
        x = (0.5 * rng.standard_normal((m, k))).astype(np.float32)
        xd = torch.from_numpy(x).cuda()
        xin = O.rmsnorm(x, gamma, 1e-6) if rms else x.astype(np.float64)
    else:
        xd, xin = dev_bits(a_bits), a_bits
    p = O.gemm(xin, w_bits, tb=True)
    ref = O.silu_mul(p[:, :f], p[:, f:])
    wd, gd = dev_bits(w_bits), torch.from_numpy(gamma).cuda()
    for dt in (torch.float32, torch.bfloat16):
        c = nan_like((m, f), dt)
        mk = lambda out: B.gemm_op(xd, wd, out, m, f, k, tb=True, glu=True, norm_gamma=gd if rms else None, norm_eps=1e-6)
        op = mk(c)
        grid, _ = B.lithos_op_grid(ctx(), op)
        assert grid == ((f + 15) // 16, 1, 1)
        cnt = counters(grid[0])
        B.lithos_debug_block_counters(ctx(), cnt)
        try:
            _launch(op)
        finally:
            B.lithos_debug_block_counters(ctx(), None)
        assert cnt.cpu().tolist() == [1] * grid[0]
        assert not torch.isnan(c.float()).any()
        if dt == torch.float32:
            assert rel_fro(c, ref) <= FRO_TOL
        else:
            bf16_close(c, ref, abs_tol=2.0 ** -22 * k)
        c_atom = nan_like((m, f), dt)
        _launch(mk(c_atom), 3)
        assert bits_equal(c, c_atom)


@pytest.mark.parametrize("seed", range(24))
def test_weight_streaming_gemm_random_shapes_and_options(seed):
    """Seeded random rows (1..16), ragged N and K, fp32 or bf16 activations, bias + GELU, residual, the
    fused normalisations and the gated epilogue in the combinations the kernel takes: against the oracle's
    operators composed in fp64, and atomized == whole bit for bit."""
    import random
    from paper_2504_15465_amd.models import norm_colsums
    rnd = random.Random(500 + seed)
    rng = np.random.default_rng(500 + seed)
    m = rnd.randint(1, 16)
    n = rnd.choice([8, 24, 40, 72, 136, 200, 328, 600, 1000])
    k = rnd.choice([8, 16, 40, 64, 72, 200, 256, 520, 776, 1200])
    a32 = rnd.random() < 0.7
    norm = rnd.choice([None, None, "rms", "ln"]) if a32 else None
    glu = rnd.random() < 0.35
    use_bias = (not glu) and rnd.random() < 0.5
    use_gelu = (not glu) and rnd.random() < 0.5
    use_res = (not glu) and rnd.random() < 0.4
    out_dt = rnd.choice([torch.float32, torch.bfloat16])
    rows_b = 2 * n if glu else n
    a_bits, w_bits = inputs.gemm_operands(m, rows_b, k, seed=seed + 40, tb=True, dist="normal")
    gamma = (1.0 + 0.2 * rng.standard_normal(k)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(k)).astype(np.float32)
    bias = (0.3 * rng.standard_normal(n)).astype(np.float32)
    res = rng.standard_normal((m, n)).astype(np.float32)
    if a32:
        x = (0.3 + 0.8 * rng.standard_normal((m, k))).astype(np.float32)
        xd = torch.from_numpy(x).cuda()
        xin = x.astype(np.float64)
        if norm == "rms":
            xin = O.rmsnorm(x, gamma, 1e-5)
        elif norm == "ln":
            xin = O.layernorm(x, gamma, beta, 1e-5)
    else:
        xd, xin = dev_bits(a_bits), a_bits
    p = O.gemm(xin, w_bits, tb=True)
    if glu:
        ref = O.silu_mul(p[:, :n], p[:, n:])
    else:
        ref = O.bias_act(p, bias if use_bias else None, gelu=use_gelu) if (use_bias or use_gelu) else p
        if use_res:
            ref = ref + res
    wd, gd, bd = dev_bits(w_bits), torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda()
    cs = norm_colsums(ctx(), gd, bd, wd) if norm == "ln" else None
    biasd = torch.from_numpy(bias).cuda() if use_bias else None
    resd = torch.from_numpy(res).cuda() if use_res else None
    mk = lambda out: B.gemm_op(xd, wd, out, m, n, k, tb=True, bias=biasd, gelu=use_gelu, residual=resd, glu=glu,
                               norm_gamma=gd if norm else None, norm_colsums=cs, norm_eps=1e-5)
    c = nan_like((m, n), out_dt)
    op = mk(c)
    grid, _ = B.lithos_op_grid(ctx(), op)
    cnt = counters(grid[0])
    B.lithos_debug_block_counters(ctx(), cnt)
    try:
        _launch(op)
    finally:
        B.lithos_debug_block_counters(ctx(), None)
    what = dict(m=m, n=n, k=k, a32=a32, norm=norm, glu=glu, bias=use_bias, gelu=use_gelu, res=use_res, out=str(out_dt))
    assert cnt.cpu().tolist() == [1] * grid[0], what
    assert not torch.isnan(c.float()).any(), what
    if out_dt == torch.float32:
        err = np.abs(c.double().cpu().numpy() - ref)
        assert rel_fro(c, ref) <= FRO_TOL and err.max() <= 1e-5 * max(1.0, np.abs(ref).max()) + 2.0 ** -22 * k, (what, err.max())
    else:
        bf16_close(c, ref, exact_frac=0.97, abs_tol=2.0 ** -22 * k + 1e-6)
    c_atom = nan_like((m, n), out_dt)
    _launch(mk(c_atom), rnd.choice([1, 2, 3, 5]))
    assert bits_equal(c, c_atom), what


def test_fused_forms_refuse_what_they_were_not_built_for():
    x32 = torch.zeros((32, 64), dtype=torch.float32, device="cuda")
    x16 = torch.zeros((32, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((128, 64), dtype=torch.bfloat16, device="cuda")
    g = torch.ones(64, dtype=torch.float32, device="cuda")
    c = torch.zeros((32, 64), dtype=torch.float32, device="cuda")
    cases = [
        B.gemm_op(x32, w, c, 32, 64, 64, tb=True, norm_gamma=g),                 # more than 16 rows
        B.gemm_op(x16, w, c, 8, 64, 64, tb=True, norm_gamma=g),                  # bf16 activations
        B.gemm_op(x16, w, c, 8, 64, 64, tb=False, glu=True),                     # not the weight-streaming form
        B.gemm_op(x16, w, c, 64, 64, 64, tb=True, glu=True, tile=64),            # a tile kernel
        B.gemm_op(x16, w, c, 8, 64, 64, tb=True, glu=True, bias=g),              # GLU with a bias
        B.gemm_op(x32, w, c, 8, 64, 64, tb=True, glu=True, residual=c),          # GLU with a residual
    ]
    cs = torch.zeros((2, 128), dtype=torch.float32, device="cuda")
    op = B.gemm_op(x32, w, c, 8, 64, 64, tb=True, norm_gamma=g, norm_colsums=cs)
    op.flags |= B.F_NORM_RMS                                                     # both kinds at once
    cases.append(op)
    op = B.gemm_op(x32, w, c, 8, 64, 64, tb=True, norm_gamma=g, norm_colsums=cs)
    op.dim[7] = 32                                                               # column sums shorter than B has rows
    cases.append(op)
    op = B.gemm_op(x32, w, c, 8, 64, 64, tb=True, norm_gamma=g, norm_colsums=cs)
    op.inp[5] = None                                                             # LayerNorm without its column sums
    cases.append(op)
    op = B.gemm_op(x32, w, c, 8, 64, 64, tb=True, norm_gamma=g)
    op.inp[4] = None                                                             # flag without gamma
    cases.append(op)
    op = B.gemm_op(x32, w, c, 8, 64, 64, tb=True, norm_gamma=g, norm_eps=-1.0)   # negative eps
    cases.append(op)
    torch.cuda.synchronize()
    for op in cases:
        with pytest.raises(B.LithosError) as e:
            B.lithos_launch_atomized(ctx(), op)
        assert e.value.code == B.EINVAL


@pytest.mark.parametrize("tb", [True, False])
def test_full_size_8192_cubed_sampled_rows(tb):
    """The benchmark's best-effort GEMM at full size, 256x256 tiles, in the
    launch shape bench.py times (weights stored [N,K]; unatomized and cut in
    atoms of 256 blocks), and the [K,N] layout beside it; 64 sampled full rows
    of C are checked against the oracle."""
    m = n = k = 8192
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=4, tb=tb)
    a, b = dev_bits(a_bits), dev_bits(b_bits)
    c_full = nan_like((m, n), torch.float32)
    c_atom = nan_like((m, n), torch.float32)
    op_full = B.gemm_op(a, b, c_full, m, n, k, tile=256, tb=tb)
    op_atom = B.gemm_op(a, b, c_atom, m, n, k, tile=256, tb=tb)
    grid, _ = B.lithos_op_grid(ctx(), op_full)
    assert grid == (32, 32, 1)
    cnt = counters(1024)
    torch.cuda.synchronize()
    B.lithos_launch_atomized(ctx(), op_full, (0, 0, 0), 0, None, None)
    B.lithos_debug_block_counters(ctx(), cnt)
    try:
        B.lithos_launch_atomized(ctx(), op_atom, (0, 0, 0), 256, None, None)
        B.lithos_partition_sync(ctx(), None)
    finally:
        B.lithos_debug_block_counters(ctx(), None)
    assert cnt.cpu().tolist() == [1] * 1024
    assert bits_equal(c_full, c_atom)
    rows = np.sort(np.random.default_rng(0).choice(m, 64, replace=False))
    ref = O.gemm(a_bits[rows], b_bits, tb=tb)
    assert rel_fro(c_full[torch.from_numpy(rows).cuda()], ref) <= FRO_TOL


def test_bf16_output_full_size_edge():
    m, n, k = 2048, 2048, 2048
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=5, dist="normal")
    c, _, _ = run_gemm(a_bits, b_bits, m, n, k, tile=256, out_dtype=torch.bfloat16)
    # fp32 accumulation of K products of N(0,1) values: absolute error ~ 2^-22 * K
    bf16_close(c, O.gemm(a_bits, b_bits), abs_tol=2.0 ** -22 * k)


def test_bad_arguments_are_refused_before_launch():
    a = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    c = torch.zeros((64, 64), dtype=torch.float32, device="cuda")
    cases = [
        B.gemm_op(a, a, c, 64, 64, 60),                      # K not a multiple of 8
        B.gemm_op(a, a, c, 64, 64, 64, lda=60),              # lda not a multiple of 8
        B.gemm_op(a, a, c, 64, 60, 64),                      # N % 8 with non-transposed B
        B.gemm_op(a, a, c, 0, 64, 64),                       # empty
        B.gemm_op(a, a, c, 64, 64, 64, ldc=32),              # ldc < N
        B.gemm_op(None, a, c, 64, 64, 64),                   # null operand
        B.gemm_op(a.view(-1)[1:].data_ptr(), a, c, 8, 8, 8), # misaligned A
        B.gemm_op(a, a, c, 64, 64, 64, tile=77),             # unknown tile
        B.gemm_op(a, a, c, 64, 64, 64, tile=B.TILE_SKINNY),  # skinny needs M <= 32 and TRANS_B
    ]
    torch.cuda.synchronize()
    for op in cases:
        with pytest.raises(B.LithosError) as e:
            B.lithos_launch_atomized(ctx(), op)
        assert e.value.code == B.EINVAL
    op = B.gemm_op(a, a, c, 64, 64, 64, tile=64)
    with pytest.raises(B.LithosError):
        B.lithos_launch_atomized(ctx(), op, grid=(3, 1, 1))   # grid with another total
    with pytest.raises(B.LithosError):
        B.lithos_launch_atom(ctx(), op, 0, 2)                 # beyond the single block
    B.lithos_launch_atomized(ctx(), op, grid=(1, 1, 1))       # same total, other factorisation: fine
    B.lithos_partition_sync(ctx(), None)


@pytest.mark.parametrize("tile,tb", [(64, False), (128, True), (128, False)])
def test_split_bf16_activations_and_outputs(tile, tb):
    """A given as hi + lo bf16 planes (~16 significant bits) and C written as such a pair."""
    m, n, k = 200, 264, 328
    x32 = inputs.normal_f32((m, k), 50)
    hi = inputs.to_bf16_bits(x32)
    lo = inputs.to_bf16_bits(x32 - O.bf16_to_f64(hi).astype(np.float32))
    b_bits = inputs.normal_bits((n, k) if tb else (k, n), 51, 0.05)
    a_val = O.bf16_to_f64(hi) + O.bf16_to_f64(lo)
    assert np.array_equal(a_val, O.round_bf16x2(x32.astype(np.float64)))      # same split as the oracle's
    ref = O.gemm(a_val, b_bits, tb=tb)
    a_pair = dev_bits(np.stack([hi, lo]))
    b = dev_bits(b_bits)
    c = nan_like((m, n), torch.float32)
    torch.cuda.synchronize()
    B.lithos_launch_atomized(ctx(), B.gemm_op(a_pair, b, c, m, n, k, tb=tb, tile=tile, a_split=True))
    B.lithos_partition_sync(ctx(), None)
    assert rel_fro(c, ref) <= 1e-6          # far tighter than the bf16-input bar: the lo plane is really used
    # bf16 pair output
    cp = nan_like((2, m, n), torch.bfloat16)
    B.lithos_launch_atomized(ctx(), B.gemm_op(a_pair, b, cp, m, n, k, tb=tb, tile=tile, a_split=True, c_split=True), (0, 0, 0), 3)
    B.lithos_partition_sync(ctx(), None)
    got = cp[0].cpu().to(torch.float64).numpy() + cp[1].cpu().to(torch.float64).numpy()
    assert np.abs(got - ref).max() <= 2.0 ** -15 * np.abs(ref).max() + 1e-6
    with pytest.raises(B.LithosError):
        B.lithos_launch_atomized(ctx(), B.gemm_op(a_pair, b, c, m, n, k, tb=tb, tile=256, a_split=True))


@pytest.mark.parametrize("tile,ta,tb,m,n,k,slices", [
    (64, True, False, 200, 136, 1000, 7),       # dW-shaped: both operands k-strided, ragged everywhere
    (128, False, False, 392, 264, 520, 3),
    (128, True, True, 256, 128, 512, 8),        # one k-tile per slice
    (256, False, True, 520, 776, 640, 4),       # k-contiguous operands, K % 64 == 0: the direct-to-LDS kernel
    (256, False, True, 256, 512, 320, 2),       # odd number of k-tiles, uneven cut (2 + 3)
    (256, True, False, 512, 264, 2048, 5),
])
def test_k_sliced_gemm_and_sum_of_slices(tile, ta, tb, m, n, k, slices):
    """K cut into ranges on the logical grid's z axis: every plane equals the oracle's product over
    its K range, the planes' ordered sum equals the whole product, any atom size gives the same bits
    and runs every (tile, slice) block once; SUM_SLICES with the fused epilogue against the oracle."""
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=31 + slices, ta=ta, tb=tb)
    a, b = dev_bits(a_bits), dev_bits(b_bits)

    def planes_with(atom_blocks, count=False):
        ws = nan_like((slices, m, n), torch.float32)
        op = B.gemm_op(a, b, ws, m, n, k, ta=ta, tb=tb, tile=tile, k_slices=slices)
        grid, _ = B.lithos_op_grid(ctx(), op)
        cnt = counters(grid[0] * grid[1] * grid[2]) if count else None
        if count:
            B.lithos_debug_block_counters(ctx(), cnt)
        torch.cuda.synchronize()
        try:
            B.lithos_launch_atomized(ctx(), op, (0, 0, 0), atom_blocks, None, None)
            B.lithos_partition_sync(ctx(), None)
        finally:
            B.lithos_debug_block_counters(ctx(), None)
        return ws, grid, cnt

    ws, grid, _ = planes_with(0)
    assert grid[2] == slices and not torch.isnan(ws).any()
    bounds = O.k_slice_bounds(k, slices)
    ref_planes = []
    for z, (lo, hi) in enumerate(bounds):
        az = a_bits[lo:hi] if ta else a_bits[:, lo:hi]
        bz = b_bits[:, lo:hi] if tb else b_bits[lo:hi]
        ref_planes.append(O.gemm(az, bz, ta=ta, tb=tb))
        assert rel_fro(ws[z], ref_planes[z]) <= FRO_TOL
    total = grid[0] * grid[1] * grid[2]
    for atom_blocks in (1, 5, total - 1):
        ws_atom, _, cnt = planes_with(atom_blocks, count=True)
        assert cnt.cpu().tolist() == [1] * total
        assert bits_equal(ws_atom, ws)

    ref = O.gemm(a_bits, b_bits, ta=ta, tb=tb)
    def summed(out_dtype, atom_blocks=0, **epi):
        y = nan_like((m, n), out_dtype)
        op = B.sum_slices_op(ws, y, m, n, slices, **epi)
        torch.cuda.synchronize()
        B.lithos_launch_atomized(ctx(), op, (0, 0, 0), atom_blocks, None, None)
        B.lithos_partition_sync(ctx(), None)
        return y
    y32 = summed(torch.float32)
    assert rel_fro(y32, ref) <= FRO_TOL
    assert bits_equal(summed(torch.float32, atom_blocks=3), y32)
    # the ordered fp32 sum of the GPU's own planes, formed on the host in the same order
    host = ws[0].cpu().numpy().copy()
    for z in range(1, slices):
        host = (host + ws[z].cpu().numpy()).astype(np.float32)
    assert np.array_equal(host, y32.cpu().numpy())
    bias = inputs.normal_f32((n,), 10, 0.5)
    resid = inputs.normal_f32((m, n), 11, 1.0)
    ref_epi = O.bias_act(O.sum_slices(np.stack(ref_planes)), bias.astype(np.float64), gelu=True) + resid.astype(np.float64)
    y16 = summed(torch.bfloat16, bias=torch.from_numpy(bias).cuda(), gelu=True, residual=torch.from_numpy(resid).cuda())
    bf16_close(y16, ref_epi, abs_tol=2.0 ** -22 * k)
    y16a = summed(torch.bfloat16, atom_blocks=2, bias=torch.from_numpy(bias).cuda(), gelu=True, residual=torch.from_numpy(resid).cuda())
    assert bits_equal(y16, y16a)


def test_sum_slices_unaligned_shapes_take_the_scalar_path():
    rows, cols, s = 37, 101, 3
    planes = inputs.normal_f32((s, rows, cols), 3, 1.0)
    y = nan_like((rows, cols), torch.float32)
    op = B.sum_slices_op(torch.from_numpy(planes).cuda(), y, rows, cols, s)
    torch.cuda.synchronize()
    B.lithos_launch_atomized(ctx(), op, (0, 0, 0), 0, None, None)
    B.lithos_partition_sync(ctx(), None)
    want = ((planes[0] + planes[1]).astype(np.float32) + planes[2]).astype(np.float32)
    assert np.array_equal(y.cpu().numpy(), want)
    assert np.abs(y.cpu().numpy().astype(np.float64) - O.sum_slices(planes.astype(np.float64))).max() <= 1e-6


def test_k_slices_bad_arguments():
    a = torch.zeros((64, 256), dtype=torch.bfloat16, device="cuda")
    c16 = torch.zeros((4, 64, 64), dtype=torch.bfloat16, device="cuda")
    c32 = torch.zeros((4, 64, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(B.LithosError):      # partial planes are fp32
        B.lithos_op_grid(ctx(), B.gemm_op(a, a, c16, 64, 64, 256, tb=True, tile=64, k_slices=4))
    with pytest.raises(B.LithosError):      # more slices than k-tiles
        B.lithos_op_grid(ctx(), B.gemm_op(a, a, c32, 64, 64, 256, tb=True, tile=64, k_slices=5))
    with pytest.raises(B.LithosError):      # plane stride too small
        B.lithos_op_grid(ctx(), B.gemm_op(a, a, c32, 64, 64, 256, tb=True, tile=64, k_slices=4, slice_plane=64 * 63))
    with pytest.raises(B.LithosError):      # the epilogue belongs to SUM_SLICES
        B.lithos_op_grid(ctx(), B.gemm_op(a, a, c32, 64, 64, 256, tb=True, tile=64, k_slices=4, gelu=True))
    assert B.lithos_op_grid(ctx(), B.gemm_op(a, a, c32, 64, 64, 256, tb=True, tile=64, k_slices=4))[0] == (1, 1, 4)


def test_training_shapes_full_size_sampled_rows():
    """The training-shaped tenant's GEMMs at full size in the launch shapes bench.py runs (16384 tokens,
    hidden 1024): Y = X W and dX = dY W^T whole, dW = X^T dY cut along K as the split hint says and summed;
    64 sampled rows of each result against the oracle, atomized launches bit-equal to whole ones."""
    tokens, k, n = 16384, 1024, 3072
    x_bits = inputs.normal_bits((tokens, k), [12, k])
    dy_bits = inputs.normal_bits((tokens, n), [13, n])
    w_bits = inputs.normal_bits((k, n), [14, 0, k, n], 0.02)
    x, dy, w = dev_bits(x_bits), dev_bits(dy_bits), dev_bits(w_bits)
    rng = np.random.default_rng(0)

    def launch(op, atom_blocks):
        torch.cuda.synchronize()
        B.lithos_launch_atomized(ctx(), op, (0, 0, 0), atom_blocks, None, None)
        B.lithos_partition_sync(ctx(), None)

    # forward and input gradient: bf16 outputs
    for name, a_bits, b_bits, a, b, m_, n_, k_, tb in (("fwd", x_bits, w_bits, x, w, tokens, n, k, False),
                                                         ("dX", dy_bits, w_bits, dy, w, tokens, k, n, True)):
        outs = []
        for atom_blocks in (0, 256):
            c = nan_like((m_, n_), torch.bfloat16)
            launch(B.gemm_op(a, b, c, m_, n_, k_, tb=tb), atom_blocks)
            outs.append(c)
        assert bits_equal(outs[0], outs[1]), name
        rows = np.sort(rng.choice(m_, 64, replace=False))
        ref = O.gemm(a_bits[rows], b_bits, tb=tb)
        bf16_close(outs[0][torch.from_numpy(rows).cuda()], ref, abs_tol=2.0 ** -22 * k_ * 4)
    # weight gradient: K = tokens, sliced
    probe = B.gemm_op(x, dy, nan_like((8,), torch.float32), k, n, tokens, ta=True)
    tile, slices = B.lithos_gemm_split_hint(probe, 256)
    assert tile == 256 and slices == 5
    outs = []
    for atom_blocks in (0, 64):
        planes = nan_like((slices, k, n), torch.float32)
        dw = nan_like((k, n), torch.bfloat16)
        launch(B.gemm_op(x, dy, planes, k, n, tokens, ta=True, tile=tile, k_slices=slices), atom_blocks)
        launch(B.sum_slices_op(planes, dw, k, n, slices), atom_blocks * 8)
        outs.append(dw)
    assert bits_equal(outs[0], outs[1])
    rows = np.sort(rng.choice(k, 64, replace=False))
    ref = O.gemm(np.ascontiguousarray(x_bits[:, rows]), dy_bits, ta=True)
    # sums of 16384 products of N(0,1) values: |dW| ~ 128, fp32 accumulation error ~ 2^-22 * K * |terms|
    bf16_close(outs[0][torch.from_numpy(rows).cuda()], ref, abs_tol=2.0 ** -22 * tokens * 4)


@pytest.mark.parametrize("tile,k", [(128, 320), (256, 320), (256, 264)])
def test_split_bf16_output_of_plain_bf16_gemm(tile, k):
    """C written as a hi + lo bf16 pair by the kernels that take ordinary bf16 operands (full tiles through
    LDS in two passes where the kernel has that path, ragged tiles element by element): the hi plane is the
    single-plane result bit for bit, hi + lo carries ~16 significant bits."""
    m, n = 520, 776
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=61)
    ref = O.gemm(a_bits, b_bits)
    a, b = dev_bits(a_bits), dev_bits(b_bits)
    single = nan_like((m, n), torch.bfloat16)
    pair = nan_like((2, m, n), torch.bfloat16)
    torch.cuda.synchronize()
    B.lithos_launch_atomized(ctx(), B.gemm_op(a, b, single, m, n, k, tile=tile))
    B.lithos_launch_atomized(ctx(), B.gemm_op(a, b, pair, m, n, k, tile=tile, c_split=True), (0, 0, 0), 2)
    B.lithos_partition_sync(ctx(), None)
    assert bits_equal(pair[0], single)
    got = pair[0].cpu().to(torch.float64).numpy() + pair[1].cpu().to(torch.float64).numpy()
    assert np.abs(got - ref).max() <= 2.0 ** -15 * np.abs(ref).max() + 2.0 ** -22 * k


@pytest.mark.parametrize("grid", [(64, 1, 1), (4, 16, 1), (1, 8, 8), (2, 2, 16)])
def test_callers_grid_of_the_same_total_changes_nothing(grid):
    """Atoms are ranges of the linear block index; another factorisation of the same total numbers
    the blocks alike, so the result equals the default launch and every block runs once."""
    m = n = k = 512
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=0)
    a, b = dev_bits(a_bits), dev_bits(b_bits)
    c0, c1 = nan_like((m, n), torch.float32), nan_like((m, n), torch.float32)
    torch.cuda.synchronize()
    B.lithos_launch_atomized(ctx(), B.gemm_op(a, b, c0, m, n, k, tile=64), (0, 0, 0), 0, None, None)
    cnt = counters(64)
    B.lithos_debug_block_counters(ctx(), cnt)
    try:
        B.lithos_launch_atomized(ctx(), B.gemm_op(a, b, c1, m, n, k, tile=64), grid, 8, None, None)
        B.lithos_partition_sync(ctx(), None)
    finally:
        B.lithos_debug_block_counters(ctx(), None)
    assert cnt.cpu().tolist() == [1] * 64
    assert not torch.isnan(c1).any()
    assert bits_equal(c0, c1)
    assert rel_fro(c1, O.gemm(a_bits, b_bits)) <= 1e-4
    with pytest.raises(B.LithosError) as e:
        B.lithos_launch_atomized(ctx(), B.gemm_op(a, b, c1, m, n, k, tile=64), (8, 7, 1), 8, None, None)
    assert e.value.code == B.EINVAL


def test_k_sliced_gemm_keeps_its_slices_under_a_callers_grid():
    """The K slices live on the operator's z axis; a caller's flat grid of the same total must not lose them."""
    m, n, k, S = 256, 256, 1024, 2
    a_bits, b_bits = inputs.gemm_operands(m, n, k, seed=5)
    a, b = dev_bits(a_bits), dev_bits(b_bits)
    p0, p1 = nan_like((S, m, n), torch.float32), nan_like((S, m, n), torch.float32)
    op0 = B.gemm_op(a, b, p0, m, n, k, tile=128, k_slices=S)
    grid, _ = B.lithos_op_grid(ctx(), op0)
    total = grid[0] * grid[1] * grid[2]
    assert grid[2] == S
    torch.cuda.synchronize()
    B.lithos_launch_atomized(ctx(), op0, (0, 0, 0), 0, None, None)
    B.lithos_launch_atomized(ctx(), B.gemm_op(a, b, p1, m, n, k, tile=128, k_slices=S), (total, 1, 1), 3, None, None)
    B.lithos_partition_sync(ctx(), None)
    assert not torch.isnan(p1).any()
    assert bits_equal(p0, p1)
