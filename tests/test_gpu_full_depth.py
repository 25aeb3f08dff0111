"""End-to-end parity of the high-priority chains at the depth the configurations name:
the 32-layer decoder step (configuration 5) and the 12-layer encoder at batch 8 and 32
(configuration 3), against the oracle, max-abs <= 1e-2.  The error at intermediate depths is
printed (run with -s) so that its growth is on record."""
import numpy as np
import pytest
import torch

from oracle import models as OM
from paper_2504_15465_amd import inputs
from paper_2504_15465_amd.models import DecoderChain, EncoderChain, run_ops
from gpu_util import bits_equal, ctx

pytestmark = pytest.mark.gpu

E2E_TOL = 1e-2


@pytest.mark.parametrize("batch", [1, 16])
def test_decoder_32_layers_matches_oracle(batch):
    """All 32 layers (hidden 4096, 32/8 heads, FFN 14336, 2048 cached positions).  The oracle walks the
    layers one by one; the GPU result after 1, 2, 4, 8, 16 and 32 layers is a prefix of the same
    operator list, so every depth is compared, not only the last."""
    H, n_q, n_kv, F, pos, n_layers = 4096, 32, 8, 14336, 2048, 32
    layers = inputs.decoder_params(n_layers, H, n_q, n_kv, F, seed=20)
    ks, vs = inputs.decoder_kv_cache(n_layers, batch, pos, n_kv, H // n_q, seed=21)
    x = inputs.decoder_hidden(batch, H, seed=22)
    chain = DecoderChain(layers, ks, vs, batch, n_q, n_kv, pos)
    chain.set_input(x)
    ops = chain.ops()
    per_layer = (len(ops) - 1) // n_layers
    assert 1 + per_layer * n_layers == len(ops)
    depths = (1, 2, 4, 8, 16, 32)
    gpu = {}
    for depth in depths:                     # each prefix restarts from the input copy (ops[0])
        run_ops(ctx(), ops[: 1 + per_layer * depth])
        gpu[depth] = chain.out.cpu().numpy().astype(np.float64)
    ref, curve = np.asarray(x, dtype=np.float64), []
    for li in range(n_layers):
        ref = OM.decoder_decode_step(ref, layers[li:li + 1], ks[li:li + 1], vs[li:li + 1], n_q, n_kv, pos)
        if li + 1 in gpu:
            err = np.abs(gpu[li + 1] - ref)
            curve.append((li + 1, float(err.max()), float(err.mean()), float(np.abs(ref).max())))
    print("\ndecoder batch %d: (layers, max-abs error, mean-abs error, max |reference|)" % batch)
    for row in curve:
        print("  %2d  %.3e  %.3e  %.2f" % row)
    for depth, emax, _, _ in curve:
        assert emax <= E2E_TOL, (depth, emax)
    out = chain.out.clone()
    run_ops(ctx(), ops, None, atom_blocks=5)
    assert bits_equal(chain.out, out)


@pytest.mark.parametrize("batch,plain", [(8, True), (32, False)])
def test_encoder_12_layers_matches_oracle(batch, plain):
    """12 layers, hidden 768, 12 heads, sequences of 128, at the batch sizes the benchmark serves.
    Batch 8 is also compared with the chain's plain definition (no rounding at any edge): the
    distance of the GPU from that chain, not only from the oracle that rounds the stored edges."""
    layers = inputs.encoder_params(12, 768, 3072, seed=10)
    x = inputs.encoder_hidden(batch, 128, 768, seed=11)
    chain = EncoderChain(layers, batch, 128, 12)
    chain.set_input(x)
    run_ops(ctx(), chain.ops())
    out = chain.out.cpu().numpy().astype(np.float64)
    ref = OM.encoder_forward(x, layers, batch, 128, 12)
    err = np.abs(out - ref)
    print("\nencoder batch %d, 12 layers: max-abs %.3e mean-abs %.3e vs the stored-edge oracle" % (batch, err.max(), err.mean()))
    assert err.max() <= E2E_TOL, (err.max(), err.mean())
    if plain:
        ref0 = OM.encoder_forward(x, layers, batch, 128, 12, edges="none")
        e0, o0 = np.abs(out - ref0), np.abs(ref - ref0)
        print("  vs the plain fp64 chain: GPU max-abs %.3e mean-abs %.3e; stored-edge oracle max-abs %.3e mean-abs %.3e"
              % (e0.max(), e0.mean(), o0.max(), o0.mean()))
        assert e0.max() <= E2E_TOL, e0.max()
