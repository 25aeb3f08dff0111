"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

from oracle import ops as O
from paper_2504_15465_amd import binding as B
from paper_2504_15465_amd.inputs import bits_to_torch

_ctx = None


def ctx():
    """One library context per test process."""
    global _ctx
    if _ctx is None:
        _ctx = B.lithos_init(0, None)
    return _ctx


def dev_bits(bits):
    return bits_to_torch(bits, "cuda").contiguous()


def nan_like(shape, dtype):
    return torch.full(shape, float("nan"), dtype=dtype, device="cuda")


def bits_equal(a: torch.Tensor, b: torch.Tensor) -> bool:
    it = torch.int32 if a.dtype == torch.float32 else torch.int16
    return bool(torch.equal(a.view(it), b.view(it)))


def rel_fro(c_gpu: torch.Tensor, c_ref: np.ndarray) -> float:
    g = c_gpu.detach().to("cpu").to(torch.float64).numpy()
    return float(np.linalg.norm(g - c_ref) / np.linalg.norm(c_ref))


def bf16_close(y_gpu: torch.Tensor, ref64: np.ndarray, exact_frac=0.98, abs_tol=1e-30):
    """bf16 output vs fp64 oracle: every element within one bf16 ulp of the
    rounded oracle value (fp32 vs fp64 arithmetic may land on the other side
    of a rounding boundary), and nearly all exactly equal.  ``abs_tol`` is the
    absolute error of the fp32 arithmetic before the rounding (it dominates
    where a sum of large terms cancels to almost zero)."""
    g = y_gpu.detach().to("cpu").to(torch.float64).numpy()
    r = O.round_bf16(ref64)
    tol = np.abs(r) * 2.0 ** -7 + abs_tol
    bad = np.abs(g - r) > tol
    assert not bad.any(), "max diff %g at %s" % (np.abs(g - r).max(), np.argwhere(bad)[:3])
    assert (g == r).mean() >= exact_frac, "only %.4f of elements equal the rounded oracle" % (g == r).mean()


def counters(n):
    return torch.zeros(n, dtype=torch.int32, device="cuda")
