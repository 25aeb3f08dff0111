"""Run a named kernel a few times, for use under rocprofv3.

    rocprofv3 --kernel-trace --stats -d OUT -- python3 -m paper_2504_15465_amd.profile_kernels --what gemm8192
    rocprofv3 --pmc FETCH_SIZE -d OUT -- python3 -m paper_2504_15465_amd.profile_kernels --what gemm8192 --copy-calibration

``--copy-calibration`` first runs a plain device-to-device copy of 1 GiB (torch's
copy kernel: reads 1 GiB, writes 1 GiB) so that the same counter can be read for
a kernel whose HBM traffic is known, then the kernel under study.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as B
from . import inputs
from .models import DecoderChain, EncoderChain, MlpChain, training_block_ops


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--what", default="gemm8192", choices=["gemm8192", "gemm8192_atoms", "prefill", "mlp", "skinny", "encoder", "decoder", "train", "atom_sweep"])
    ap.add_argument("--tile", type=int, default=256)
    ap.add_argument("--batch", type=int, default=4)
    ap.add_argument("--layers", type=int, default=4)
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--warm", type=int, default=0, help="gemm8192: launches before the --reps ones (the profiler sees them too; "
                    "profile_summary --skip sets them apart), so that the clocks have settled")
    ap.add_argument("--cus", type=int, default=256)
    ap.add_argument("--tokens", type=int, default=8192, help="prefill: prompt length")
    ap.add_argument("--copy-calibration", action="store_true")
    ap.add_argument("--nt", action="store_true", help="gemm8192: B stored [N,K] (TRANS_B)")
    args = ap.parse_args()

    ctx = B.lithos_init(0, None)
    part = B.lithos_create_partition(ctx, B.lithos_make_mask(ctx, args.cus))
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(1)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if args.what.startswith("gemm8192"):
        n = 8192
        a_bits, b_bits = inputs.gemm_operands(n, n, n, seed=4)
        a, b = inputs.bits_to_torch(a_bits, "cuda"), inputs.bits_to_torch(b_bits, "cuda")
        c = torch.empty((n, n), dtype=torch.bfloat16, device="cuda")
        op = B.gemm_op(a, b, c, n, n, n, tile=args.tile, tb=args.nt)      # square: the same buffer serves as [N,K]
        grid, wg = B.lithos_op_grid(ctx, op)
        atom = 0 if args.what == "gemm8192" else args.cus * wg
        torch.cuda.synchronize()
        for _ in range(args.warm + args.reps):
            B.lithos_launch_atomized(ctx, op, (0, 0, 0), atom, part, None)
        B.lithos_partition_sync(ctx, part)
    elif args.what == "prefill":        # causal attention over one prompt of --tokens positions, 32 / 8 heads of 128
        import math
        n_q, n_kv, d, T = 32, 8, 128, args.tokens
        q = inputs.bits_to_torch(inputs.normal_bits((T, n_q * d), 54), "cuda")
        kc = inputs.bits_to_torch(inputs.normal_bits((1, T, n_kv, d), 55), "cuda")
        vc = inputs.bits_to_torch(inputs.normal_bits((1, T, n_kv, d), 56), "cuda")
        o = torch.empty((T, n_q * d), dtype=torch.bfloat16, device="cuda")
        op = B.attn_prefill_op(q, kc, vc, o, 1, n_q, n_kv, d, T, T, 1.0 / math.sqrt(d))
        torch.cuda.synchronize()
        mean, med = B.lithos_time_launch(ctx, op, 0, part, args.warm + 2, args.reps)
        flop = 2.0 * T * T * d * n_q
        print("prefill %d tokens on %d CUs: median %.1f us, %.0f TFLOP/s (causal flops)" % (T, args.cus, med, flop / med * 1e-6))
    elif args.what in ("mlp", "skinny"):
        layers = inputs.mlp_params(6, 4096, seed=1)
        chain = MlpChain(layers, 8, fused=True)
        chain.set_input(inputs.mlp_requests(1, 8, 4096, 2)[0])
        ops = chain.ops()
        if args.what == "skinny":
            ops = [o for o in ops if o.kind == B.OP_GEMM]
        torch.cuda.synchronize()
        for _ in range(args.reps):
            for o in ops:
                B.lithos_launch_atomized(ctx, o, (0, 0, 0), 0, part, None)
        B.lithos_partition_sync(ctx, part)
    elif args.what == "atom_sweep":
        # Atom overhead against atom size (device time stamps on the launch's own queue, whole and atomized
        # launches alternating): the 8192^3 GEMM on all CUs, and configuration 1 (512^3, 64x64 tiles, 32 CUs).
        def sweep(title, op, p, sizes, reps):
            grid, wg = B.lithos_op_grid(ctx, op)
            total = grid[0] * grid[1] * grid[2]
            print("## %s: %d blocks, %d resident per CU" % (title, total, wg))
            print("| atom_blocks | atoms | whole us | atomized us | overhead % |\n|---|---|---|---|---|")
            B.lithos_time_launch(ctx, op, 0, p, 3, 3)
            for ab in sizes:
                rounds = [(B.lithos_time_launch(ctx, op, 0, p, 1, reps)[1], B.lithos_time_launch(ctx, op, ab, p, 1, reps)[1])
                          for _ in range(4)]
                w = sorted(r[0] for r in rounds)[2]
                a = sorted(r[1] for r in rounds)[2]
                print("| %d | %d | %.1f | %.1f | %+.1f |" % (ab, -(-total // ab), w, a, (a / w - 1) * 100), flush=True)
        n = 8192
        a_bits, b_bits = inputs.gemm_operands(n, n, n, seed=4)
        a, b = inputs.bits_to_torch(a_bits, "cuda"), inputs.bits_to_torch(b_bits, "cuda")
        c = torch.empty((n, n), dtype=torch.bfloat16, device="cuda")
        torch.cuda.synchronize()
        sweep("8192^3 bf16 GEMM, 256x256 tiles, %d CUs" % args.cus, B.gemm_op(a, b, c, n, n, n, tile=256), part,
              (512, 256, 128, 64, 32), 5)
        a_bits, b_bits = inputs.gemm_operands(512, 512, 512, seed=0)
        a, b = inputs.bits_to_torch(a_bits, "cuda"), inputs.bits_to_torch(b_bits, "cuda")
        c32 = torch.empty((512, 512), dtype=torch.float32, device="cuda")
        p32 = B.lithos_create_partition(ctx, B.lithos_make_mask(ctx, 32))
        torch.cuda.synchronize()
        sweep("configuration 1: 512^3 bf16 GEMM, 64x64 tiles, 32 CUs", B.gemm_op(a, b, c32, 512, 512, 512, tile=64), p32,
              (32, 16, 8, 4), 20)
        B.lithos_destroy_partition(p32)
    elif args.what == "train":          # fwd, dX, dW GEMMs of --layers transformer blocks (hidden 1024, FFN 4096, 16384 tokens)
        ops, _, keep, _ = training_block_ops(n_layers=args.layers, split_cus=args.cus)
        torch.cuda.synchronize()
        for _ in range(args.reps):
            for o in ops:
                B.lithos_launch_atomized(ctx, o, (0, 0, 0), 0, part, None)
        B.lithos_partition_sync(ctx, part)
    elif args.what in ("encoder", "decoder"):
        if args.what == "encoder":      # 12 layers, hidden 768, 12 heads, FFN 3072, sequences of 128
            chain = EncoderChain(inputs.encoder_params(12, 768, 3072, seed=10), args.batch, 128, 12)
            chain.set_input(inputs.encoder_hidden(args.batch, 128, 768, seed=11))
        else:                           # hidden 4096, 32 query / 8 key-value heads, FFN 14336, 2048 cached positions
            nl, H, nq, nkv, F, pos = args.layers, 4096, 32, 8, 14336, 2048
            ks, vs = inputs.decoder_kv_cache(nl, args.batch, pos, nkv, H // nq, seed=21)
            chain = DecoderChain(inputs.decoder_params(nl, H, nq, nkv, F, seed=20), ks, vs, args.batch, nq, nkv, pos)
            chain.set_input(inputs.decoder_hidden(args.batch, H, seed=22))
        ops = chain.ops()
        torch.cuda.synchronize()
        for _ in range(args.reps):
            for o in ops:
                B.lithos_launch_atomized(ctx, o, (0, 0, 0), 0, part, None)
        B.lithos_partition_sync(ctx, part)
    B.lithos_destroy_partition(part)
    B.lithos_shutdown(ctx)


if __name__ == "__main__":
    main()
