"""End-to-end parity of the high-priority MLP tenant (6 x GEMM+bias+GELU+LayerNorm,
batch 8, hidden 4096) against the chain oracle: max-abs <= 1e-2, and atomized
== unatomized bit for bit."""
import numpy as np
import pytest
import torch

from oracle import models as OM
from paper_2504_15465_amd import binding as B
from paper_2504_15465_amd import inputs
from paper_2504_15465_amd.models import MlpChain, run_ops
from gpu_util import bits_equal, ctx

pytestmark = pytest.mark.gpu

E2E_TOL = 1e-2


@pytest.mark.parametrize("hidden,batch,n_layers", [(4096, 8, 6), (512, 5, 3)])
def test_mlp_chain_matches_oracle(hidden, batch, n_layers):
    layers = inputs.mlp_params(n_layers, hidden, seed=1)
    reqs = inputs.mlp_requests(pool=2, batch=batch, hidden=hidden, seed=2)
    chain = MlpChain(layers, batch)
    part = B.lithos_create_partition(ctx(), B.lithos_make_mask(ctx(), 64))
    try:
        for r in range(2):
            chain.set_input(reqs[r])
            run_ops(ctx(), chain.ops(), part)
            out_full = chain.out.clone()
            ref = OM.mlp_forward(reqs[r], layers)
            err = np.abs(out_full.cpu().numpy().astype(np.float64) - ref).max()
            assert err <= E2E_TOL, err
            chain.out.fill_(float("nan"))
            run_ops(ctx(), chain.ops(), part, atom_blocks=5)
            assert bits_equal(chain.out, out_full)
    finally:
        B.lithos_destroy_partition(part)


def test_mlp_chain_tile_kernel_variant_agrees():
    """The same model through the 64x64 MFMA tile GEMM ([K,N] weights) stays within the bar."""
    layers = inputs.mlp_params(2, 1024, seed=1)
    x = inputs.mlp_requests(pool=1, batch=8, hidden=1024, seed=2)[0]
    chain = MlpChain(layers, 8, tile=B.TILE_64)
    chain.set_input(x)
    run_ops(ctx(), chain.ops())
    ref = OM.mlp_forward(x, layers)
    assert np.abs(chain.out.cpu().numpy().astype(np.float64) - ref).max() <= E2E_TOL
