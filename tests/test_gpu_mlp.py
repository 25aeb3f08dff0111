"""End-to-end parity of the high-priority MLP tenant (6 x GEMM+bias+GELU+LayerNorm,
batch 8, hidden 4096) against the chain oracle: max-abs <= 1e-2, and atomized
== unatomized bit for bit."""
import numpy as np
import pytest
import torch

from oracle import models as OM
from oracle import ops as O
from paper_2504_15465_amd import binding as B
from paper_2504_15465_amd import inputs
from paper_2504_15465_amd.models import MlpChain, run_ops
from gpu_util import bits_equal, ctx, dev_bits, nan_like, rel_fro

pytestmark = pytest.mark.gpu

E2E_TOL = 1e-2


@pytest.mark.parametrize("hidden,batch,n_layers,fused", [(4096, 8, 6, True), (4096, 8, 6, False), (512, 5, 3, True),
                                                         (1024, 16, 2, True), (1024, 16, 2, False), (1024, 32, 2, False),
                                                         (4096, 1, 6, True)])
def test_mlp_chain_matches_oracle(hidden, batch, n_layers, fused):
    """``fused``: each LayerNorm runs inside the next layer's GEMM (one launch per layer and a last LayerNorm)."""
    layers = inputs.mlp_params(n_layers, hidden, seed=1)
    reqs = inputs.mlp_requests(pool=2, batch=batch, hidden=hidden, seed=2)
    chain = MlpChain(layers, batch, fused=fused, ctx=ctx())
    assert len(chain.ops()) == (n_layers + 1 if fused else 2 * n_layers)
    part = B.lithos_create_partition(ctx(), B.lithos_make_mask(ctx(), 64))
    try:
        for r in range(2):
            chain.set_input(reqs[r])
            run_ops(ctx(), chain.ops(), part)
            out_full = chain.out.clone()
            ref = OM.mlp_forward(reqs[r], layers)
            err = np.abs(out_full.cpu().numpy().astype(np.float64) - ref).max()
            assert err <= E2E_TOL, err
            assert err <= 1e-4, err          # fp32 edges throughout: far inside the bar
            chain.out.fill_(float("nan"))
            run_ops(ctx(), chain.ops(), part, atom_blocks=5)
            assert bits_equal(chain.out, out_full)
    finally:
        B.lithos_destroy_partition(part)


@pytest.mark.parametrize("m,n,k", [(8, 4096, 4096), (16, 1000, 520), (32, 2048, 1536), (3, 72, 8)])
def test_skinny_gemm_with_fp32_activations(m, n, k):
    x32 = inputs.normal_f32((m, k), 31)
    w_bits = inputs.normal_bits((n, k), 32, 0.05)
    ref = O.gemm(x32.astype(np.float64), w_bits, tb=True)
    c = nan_like((m, n), torch.float32)
    op = B.gemm_op(torch.from_numpy(x32).cuda(), dev_bits(w_bits), c, m, n, k, tb=True)
    torch.cuda.synchronize()
    B.lithos_launch_atomized(ctx(), op)
    B.lithos_partition_sync(ctx(), None)
    assert rel_fro(c, ref) <= 1e-4
    ca = nan_like((m, n), torch.float32)
    torch.cuda.synchronize()
    B.lithos_launch_atomized(ctx(), B.gemm_op(torch.from_numpy(x32).cuda(), dev_bits(w_bits), ca, m, n, k, tb=True),
                             (0, 0, 0), 3, None, None)
    B.lithos_partition_sync(ctx(), None)
    assert bits_equal(c, ca)
    # fp32 activations are refused by the MFMA tile kernels
    with pytest.raises(B.LithosError):
        B.lithos_launch_atomized(ctx(), B.gemm_op(torch.from_numpy(x32).cuda(), dev_bits(w_bits), c, m, n, k, tb=True, tile=64))
