"""Thin ctypes binding of ``liblithos.so`` (argument marshalling only).

Function names are those of ``include/lithos.h``.  Tensors are torch CUDA
tensors; only their ``data_ptr()`` crosses the boundary.  A missing library is
an ImportError-like RuntimeError: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch  # loads the HIP runtime that liblithos.so binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblithos.so")

OK, EINVAL, EHIP, EMASK, ESTATE, ELIMIT = 0, -1, -2, -3, -4, -5
MASK_WORDS = 8
MAX_SWEEP = 64

OP_GEMM, OP_BIAS_ACT, OP_LAYERNORM, OP_SOFTMAX, OP_ATTN_ENC, OP_ATTN_DEC, OP_RMSNORM, OP_ROPE_KV, OP_SILU_MUL, OP_SPIN, OP_ATTN_MERGE, OP_SUM_SLICES, OP_ATTN_PREFILL = range(1, 14)
ATTN_MAX_SPLITS = 64
F_TRANS_A, F_TRANS_B, F_BIAS, F_GELU, F_RESIDUAL, F_OUT_F32, F_IN_F32, F_SPLIT_A, F_OUT_SPLIT, F_NORM_LN, F_NORM_RMS, F_GLU = (1 << i for i in range(12))
TILE_AUTO, TILE_SKINNY, TILE_64, TILE_128, TILE_256 = 0, 1, 64, 128, 256
MASK_STRIPED, MASK_WHOLE_XCD = 0, 1
CLASS_HP, CLASS_BE = 0, 1


class Dim3(C.Structure):
    _fields_ = [("x", C.c_uint32), ("y", C.c_uint32), ("z", C.c_uint32)]


class Op(C.Structure):
    _fields_ = [("kind", C.c_int32), ("flags", C.c_uint32), ("op_id", C.c_int32), ("tile", C.c_int32),
                ("dim", C.c_int64 * 8), ("ld", C.c_int64 * 4), ("fparam", C.c_float * 4),
                ("inp", C.c_void_p * 6), ("out", C.c_void_p * 2)]


class Config(C.Structure):
    _fields_ = [("atom_duration_us", C.c_double), ("max_outstanding", C.c_int32),
                ("max_outstanding_hp", C.c_int32), ("steal", C.c_int32), ("atomize", C.c_int32),
                ("xcd_remap", C.c_int32), ("prelude", C.c_int32), ("ema_alpha", C.c_double),
                ("rightsize_slip", C.c_double)]

    @classmethod
    def default(cls, **kw):
        c = cls(250.0, 2, 0, 1, 1, 1, 0, 0.25, 0.0)
        for k, v in kw.items():
            setattr(c, k, v)
        return c


class DevInfo(C.Structure):
    _fields_ = [("n_cu", C.c_int32), ("n_xcd", C.c_int32), ("cu_per_xcd", C.c_int32), ("wave_size", C.c_int32),
                ("lds_bytes_per_cu", C.c_int32), ("clock_khz", C.c_int32), ("mask_bits_interleaved", C.c_int32),
                ("arch", C.c_char * 32)]


class RightsizeResult(C.Structure):
    _fields_ = [("n_points", C.c_int32), ("cus", C.c_int32 * MAX_SWEEP), ("median_us", C.c_double * MAX_SWEEP),
                ("chosen_cus", C.c_int32), ("chosen_us", C.c_double), ("full_us", C.c_double),
                ("occupancy_bound_cus", C.c_int32), ("model_m", C.c_double), ("model_b", C.c_double),
                ("model_cus", C.c_int32), ("online_cus", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [("kernels", C.c_uint64), ("atoms", C.c_uint64), ("stolen_atoms", C.c_uint64),
                ("revocations", C.c_uint64), ("rightsized_kernels", C.c_uint64), ("predictions", C.c_uint64), ("mispredicts", C.c_uint64), ("abs_err_sum_us", C.c_double)]


class CoreAtom(C.Structure):
    _fields_ = [("atom_id", C.c_uint64), ("tenant", C.c_int32), ("kernel_id", C.c_uint64), ("ordinal", C.c_int32),
                ("lo", C.c_uint32), ("hi", C.c_uint32), ("group_mask", C.c_uint32), ("stolen", C.c_int32),
                ("has_prediction", C.c_int32), ("predicted_us", C.c_double)]


EXPORTS = [
    "lithos_init", "lithos_shutdown", "lithos_device_info", "lithos_last_error",
    "lithos_make_mask", "lithos_create_partition", "lithos_destroy_partition", "lithos_partition_cus",
    "lithos_partition_stream", "lithos_probe_partition", "lithos_partitions_coupled",
    "lithos_op_grid", "lithos_gemm_split_hint", "lithos_launch_atomized", "lithos_launch_attn_dec_static",
    "lithos_launch_atom", "lithos_partition_sync",
    "lithos_debug_block_counters", "lithos_rightsize", "lithos_time_launch",
    "lithos_tenant_create", "lithos_tenant_destroy", "lithos_submit", "lithos_sync_mark", "lithos_sync",
    "lithos_poll", "lithos_tenant_stats", "lithos_stats",
    "lithos_drive_open_loop", "lithos_drive_closed_loop_start", "lithos_drive_closed_loop_stop",
    "lithos_core_create", "lithos_core_destroy", "lithos_core_add_tenant", "lithos_core_submit",
    "lithos_core_sync_mark", "lithos_core_next_atom", "lithos_core_complete", "lithos_core_stats",
]

_lib = None


class LithosError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("liblithos error %d: %s" % (code, text))
        self.code = code


def lib():
    """Load liblithos.so (built in-tree).  Fails loudly if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("liblithos.so is not built: run `python -m paper_2504_15465_amd.build` "
                               "(there is no fallback path)")
        _lib = C.CDLL(LIB_PATH)
        _lib.lithos_last_error.restype = C.c_char_p
        for name in EXPORTS:
            if name != "lithos_last_error":
                getattr(_lib, name).restype = C.c_int
    return _lib


def _check(rc):
    if rc != OK:
        raise LithosError(rc, lib().lithos_last_error().decode(errors="replace"))


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        return t.data_ptr()
    return int(t)


# ---- operator descriptors -------------------------------------------------------

def make_op(kind, dims=(), flags=0, tile=0, ld=(), fparam=(), inputs=(), outputs=(), op_id=0) -> Op:
    op = Op()
    op.kind, op.flags, op.op_id, op.tile = kind, flags, op_id, tile
    for i, v in enumerate(dims):
        op.dim[i] = int(v)
    for i, v in enumerate(ld):
        op.ld[i] = int(v)
    for i, v in enumerate(fparam):
        op.fparam[i] = float(v)
    for i, t in enumerate(inputs):
        op.inp[i] = _ptr(t)
    for i, t in enumerate(outputs):
        op.out[i] = _ptr(t)
    # the descriptor holds raw pointers: keep the tensors alive as long as it lives
    op._keep = (tuple(inputs), tuple(outputs))
    return op


def gemm_op(a, b, c, m, n, k, ta=False, tb=False, bias=None, gelu=False, residual=None, tile=0,
            lda=None, ldb=None, ldc=None, ldr=None, op_id=0, a_split=False, c_split=False, k_slices=0, slice_plane=None,
            norm_gamma=None, norm_colsums=None, norm_eps=1e-5, glu=False) -> Op:
    """``a_split``: ``a`` is a [2, M, K] bf16 pair (hi, lo planes); ``c_split``: ``c`` is a [2, M, N] pair;
    ``k_slices`` > 1: ``c`` is an fp32 [k_slices, M, N] stack of partial planes for ``sum_slices_op``;
    ``norm_gamma``: rows of ``a`` are RMS-normalised on load; with ``norm_colsums`` (the fp32 [2, rows of b]
    product of the rows gamma and beta with ``b``, made once per weight matrix by this same GEMM) layer-normalised;
    ``glu``: ``b`` is [2N, K], gate rows then up rows, and ``c`` = silu(gate product) * (up product)."""
    flags = (F_TRANS_A if ta else 0) | (F_TRANS_B if tb else 0) | (F_BIAS if bias is not None else 0)
    flags |= (F_GELU if gelu else 0) | (F_RESIDUAL if residual is not None else 0)
    if isinstance(c, torch.Tensor) and c.dtype == torch.float32:
        flags |= F_OUT_F32
    if isinstance(a, torch.Tensor) and a.dtype == torch.float32:
        flags |= F_IN_F32
    lda = lda if lda is not None else (m if ta else k)
    ldb = ldb if ldb is not None else (k if tb else n)
    ldc = ldc if ldc is not None else n
    ldr = ldr if ldr is not None else n
    flags |= (F_SPLIT_A if a_split else 0) | (F_OUT_SPLIT if c_split else 0) | (F_GLU if glu else 0)
    if norm_gamma is not None:
        flags |= F_NORM_LN if norm_colsums is not None else F_NORM_RMS
    if k_slices > 1 and slice_plane is None:
        slice_plane = m * ldc
    cs_stride = norm_colsums.shape[-1] if isinstance(norm_colsums, torch.Tensor) else 0
    return make_op(OP_GEMM, (m, n, k, m * lda if a_split else 0, m * ldc if c_split else 0, k_slices, slice_plane or 0, cs_stride), flags, tile,
                   (lda, ldb, ldc, ldr), (norm_eps if norm_gamma is not None else 0.0,), (a, b, bias, residual, norm_gamma, norm_colsums), (c,), op_id)


def sum_slices_op(planes, y, rows, cols, slices, bias=None, gelu=False, residual=None, slice_plane=None,
                  ldx=None, ldy=None, ldr=None, op_id=0) -> Op:
    """Second step of a K-sliced GEMM: ``y = act(sum_z planes[z] + bias) + residual``, planes added in slice order."""
    flags = (F_BIAS if bias is not None else 0) | (F_GELU if gelu else 0) | (F_RESIDUAL if residual is not None else 0)
    if isinstance(y, torch.Tensor) and y.dtype == torch.float32:
        flags |= F_OUT_F32
    ldx = ldx if ldx is not None else cols
    return make_op(OP_SUM_SLICES, (rows, cols, slices, slice_plane if slice_plane is not None else rows * ldx), flags,
                   ld=(ldx, ldy if ldy is not None else cols, ldr if ldr is not None else cols),
                   inputs=(planes, bias, residual), outputs=(y,), op_id=op_id)


def bias_act_op(x, y, rows, cols, bias=None, gelu=True, op_id=0) -> Op:
    flags = (F_BIAS if bias is not None else 0) | (F_GELU if gelu else 0)
    flags |= F_IN_F32 if x.dtype == torch.float32 else 0
    flags |= F_OUT_F32 if y.dtype == torch.float32 else 0
    return make_op(OP_BIAS_ACT, (rows, cols), flags, inputs=(x, bias), outputs=(y,), op_id=op_id)


def split_op(x, y_pair, rows, cols, op_id=0) -> Op:
    """fp32 (or bf16) x -> [2, rows, cols] bf16 pair: hi = bf16(x), lo = bf16(x - hi)."""
    flags = (F_IN_F32 if x.dtype == torch.float32 else 0) | F_OUT_SPLIT
    return make_op(OP_BIAS_ACT, (rows, cols), flags, inputs=(x, None), outputs=(y_pair,), op_id=op_id)


def layernorm_op(x, gamma, beta, y, rows, h, eps=1e-5, y_bf16=None, op_id=0, split=False) -> Op:
    """``split``: ``y_bf16`` is a [2, rows, h] bf16 pair (hi, lo planes)."""
    flags = (F_IN_F32 if x.dtype == torch.float32 else 0) | (F_OUT_F32 if y.dtype == torch.float32 else 0)
    flags |= F_OUT_SPLIT if split else 0
    return make_op(OP_LAYERNORM, (rows, h), flags, fparam=(eps,), inputs=(x, gamma, beta), outputs=(y, y_bf16), op_id=op_id)


def rmsnorm_op(x, w, y, rows, h, eps=1e-5, op_id=0) -> Op:
    flags = (F_IN_F32 if x.dtype == torch.float32 else 0) | (F_OUT_F32 if y.dtype == torch.float32 else 0)
    return make_op(OP_RMSNORM, (rows, h), flags, fparam=(eps,), inputs=(x, w), outputs=(y,), op_id=op_id)


def softmax_op(s, p, rows, n, scale=1.0, op_id=0) -> Op:
    flags = (F_IN_F32 if s.dtype == torch.float32 else 0) | (F_OUT_F32 if p.dtype == torch.float32 else 0)
    return make_op(OP_SOFTMAX, (rows, n), flags, fparam=(scale,), inputs=(s,), outputs=(p,), op_id=op_id)


def silu_mul_op(gu, y, rows, f, op_id=0) -> Op:
    flags = (F_IN_F32 if gu.dtype == torch.float32 else 0) | (F_OUT_F32 if y.dtype == torch.float32 else 0)
    return make_op(OP_SILU_MUL, (rows, f), flags, inputs=(gu,), outputs=(y,), op_id=op_id)


def rope_kv_op(qkv, kcache, vcache, rows, n_q, n_kv, d, pos, cap, theta=10000.0, op_id=0) -> Op:
    flags = F_IN_F32 if qkv.dtype == torch.float32 else 0
    return make_op(OP_ROPE_KV, (rows, n_q, n_kv, d, pos, cap), flags, fparam=(theta,), inputs=(qkv,),
                   outputs=(kcache, vcache), op_id=op_id)


def attn_enc_op(qkv, o, batch, heads, seq, d, scale, op_id=0, split=False) -> Op:
    """``split``: ``o`` is a [2, batch*seq, heads*d] bf16 pair (hi, lo planes)."""
    return make_op(OP_ATTN_ENC, (batch, heads, seq, d), F_OUT_SPLIT if split else 0, fparam=(scale,),
                   inputs=(qkv,), outputs=(o,), op_id=op_id)


def attn_dec_op(q, kcache, vcache, o, batch, n_q, n_kv, d, keys, cap, scale, ldq=None, op_id=0,
                splits=1, workspace=None) -> Op:
    """splits > 1 needs an fp32 workspace of attn_workspace_floats(...) elements and an attn_merge_op after it."""
    flags = (F_IN_F32 if q.dtype == torch.float32 else 0) | (F_OUT_F32 if o.dtype == torch.float32 else 0)
    ins = (q, kcache, vcache) if workspace is None else (q, kcache, vcache, workspace)
    return make_op(OP_ATTN_DEC, (batch, n_q, n_kv, d, keys, cap, splits), flags, ld=(ldq if ldq is not None else n_q * d,),
                   fparam=(scale,), inputs=ins, outputs=(o,), op_id=op_id)


def attn_prefill_op(q, kcache, vcache, o, batch, n_q, n_kv, d, tokens, cap, scale, ldq=None, ldo=None, op_id=0) -> Op:
    """Causal self-attention over a prompt of ``tokens`` positions per sequence (query i sees keys 0..i)."""
    return make_op(OP_ATTN_PREFILL, (batch, n_q, n_kv, d, tokens, cap), 0,
                   ld=(ldq if ldq is not None else n_q * d, ldo if ldo is not None else n_q * d),
                   fparam=(scale,), inputs=(q, kcache, vcache), outputs=(o,), op_id=op_id)


def attn_workspace_floats(batch, n_q, d, splits) -> int:
    return batch * n_q * splits * (d + 2)


def attn_merge_op(workspace, o, batch, n_q, n_kv, d, splits, op_id=0) -> Op:
    flags = F_OUT_F32 if o.dtype == torch.float32 else 0
    return make_op(OP_ATTN_MERGE, (batch, n_q, n_kv, d, splits), flags, inputs=(workspace,), outputs=(o,), op_id=op_id)


def spin_op(blocks, ticks, op_id=0) -> Op:
    return make_op(OP_SPIN, (blocks, ticks), op_id=op_id)


# ---- context / partitions ---------------------------------------------------------

def lithos_init(device=0, cfg: Optional[Config] = None):
    ctx = C.c_void_p()
    _check(lib().lithos_init(int(device), C.byref(cfg) if cfg is not None else None, C.byref(ctx)))
    return ctx


def lithos_shutdown(ctx):
    _check(lib().lithos_shutdown(ctx))


def lithos_device_info(ctx) -> DevInfo:
    info = DevInfo()
    _check(lib().lithos_device_info(ctx, C.byref(info)))
    return info


def lithos_make_mask(ctx, n_cus, policy=MASK_STRIPED, first=0) -> np.ndarray:
    mask = (C.c_uint32 * MASK_WORDS)()
    _check(lib().lithos_make_mask(ctx, int(n_cus), int(policy), int(first), mask))
    return np.frombuffer(mask, dtype=np.uint32).copy()


def lithos_create_partition(ctx, mask: Sequence[int]):
    arr = (C.c_uint32 * len(mask))(*[int(w) for w in mask])
    p = C.c_void_p()
    _check(lib().lithos_create_partition(ctx, arr, C.c_uint32(len(mask)), C.byref(p)))
    return p


def lithos_destroy_partition(p):
    _check(lib().lithos_destroy_partition(p))


def lithos_partition_cus(p) -> int:
    n = C.c_int()
    _check(lib().lithos_partition_cus(p, C.byref(n)))
    return n.value


def lithos_partition_stream(p) -> int:
    s = C.c_void_p()
    _check(lib().lithos_partition_stream(p, C.byref(s)))
    return s.value or 0


def lithos_partitions_coupled(ctx, busy, probe) -> bool:
    c = C.c_int()
    _check(lib().lithos_partitions_coupled(ctx, busy, probe, C.byref(c)))
    return bool(c.value)


def lithos_probe_partition(ctx, p, n_wg):
    xcd = np.zeros(n_wg, dtype=np.uint32)
    hwid = np.zeros(n_wg, dtype=np.uint32)
    _check(lib().lithos_probe_partition(ctx, p, C.c_uint32(n_wg), xcd.ctypes.data_as(C.c_void_p),
                                        hwid.ctypes.data_as(C.c_void_p)))
    return xcd, hwid


# ---- atomized launch -----------------------------------------------------------------

def lithos_op_grid(ctx, op: Op):
    g = Dim3()
    w = C.c_uint32()
    _check(lib().lithos_op_grid(ctx, C.byref(op), C.byref(g), C.byref(w)))
    return (g.x, g.y, g.z), w.value


def lithos_gemm_split_hint(op: Op, n_cus=256):
    """(tile, k_slices) that fill ``n_cus`` compute units; k_slices == 1: leave the GEMM whole."""
    tile, slices = C.c_int32(0), C.c_int32(0)
    _check(lib().lithos_gemm_split_hint(C.byref(op), int(n_cus), C.byref(tile), C.byref(slices)))
    return tile.value, slices.value


def lithos_launch_atomized(ctx, op: Op, grid=(0, 0, 0), atom_blocks=0, part=None, stream=None):
    g = Dim3(*grid)
    _check(lib().lithos_launch_atomized(ctx, C.byref(op), g, C.c_uint32(atom_blocks), part,
                                        C.c_void_p(stream) if stream else None))


STATIC_SCRATCH_FLOATS = 2 << 20


def lithos_launch_attn_dec_static(ctx, op: Op, atom_blocks=0, part=None, stream=None):
    _check(lib().lithos_launch_attn_dec_static(ctx, C.byref(op), C.c_uint32(atom_blocks), part,
                                               C.c_void_p(stream) if stream else None))


def lithos_launch_atom(ctx, op: Op, lo, hi, part=None):
    _check(lib().lithos_launch_atom(ctx, C.byref(op), C.c_uint32(lo), C.c_uint32(hi), part))


def lithos_partition_sync(ctx, part=None):
    _check(lib().lithos_partition_sync(ctx, part))


def lithos_debug_block_counters(ctx, counters: Optional[torch.Tensor]):
    if counters is None:
        _check(lib().lithos_debug_block_counters(ctx, None, C.c_uint32(0)))
    else:
        assert counters.dtype == torch.int32 and counters.is_cuda
        _check(lib().lithos_debug_block_counters(ctx, C.c_void_p(counters.data_ptr()), C.c_uint32(counters.numel())))


def lithos_rightsize(ctx, op: Op, cu_lo=8, cu_hi=256, cu_step=8, warmup=5, reps=50, slowdown=0.04) -> RightsizeResult:
    r = RightsizeResult()
    _check(lib().lithos_rightsize(ctx, C.byref(op), cu_lo, cu_hi, cu_step, warmup, reps, C.c_double(slowdown), C.byref(r)))
    return r


def lithos_time_launch(ctx, op: Op, atom_blocks=0, part=None, warmup=3, reps=20):
    """(mean_us, median_us) of `reps` launches, device time stamps."""
    mean, med = C.c_double(), C.c_double()
    _check(lib().lithos_time_launch(ctx, C.byref(op), C.c_uint32(atom_blocks), part, int(warmup), int(reps),
                                    C.byref(mean), C.byref(med)))
    return mean.value, med.value


# ---- tenants ------------------------------------------------------------------------------

def lithos_tenant_create(ctx, cls, quota=None):
    t = C.c_void_p()
    _check(lib().lithos_tenant_create(ctx, int(cls), quota, C.byref(t)))
    return t


def lithos_tenant_destroy(t):
    _check(lib().lithos_tenant_destroy(t))


def lithos_submit(t, op: Op) -> int:
    ticket = C.c_uint64()
    _check(lib().lithos_submit(t, C.byref(op), C.byref(ticket)))
    return ticket.value


def lithos_sync_mark(t):
    _check(lib().lithos_sync_mark(t))


def lithos_sync(t):
    _check(lib().lithos_sync(t))


def lithos_poll(t, ticket) -> bool:
    done = C.c_int()
    _check(lib().lithos_poll(t, C.c_uint64(ticket), C.byref(done)))
    return bool(done.value)


def lithos_tenant_stats(t) -> Stats:
    s = Stats()
    _check(lib().lithos_tenant_stats(t, C.byref(s)))
    return s


def lithos_stats(ctx) -> Stats:
    s = Stats()
    _check(lib().lithos_stats(ctx, C.byref(s)))
    return s


def _op_array(ops: Sequence[Op]):
    arr = (Op * len(ops))()
    for i, o in enumerate(ops):
        C.memmove(C.byref(arr, i * C.sizeof(Op)), C.byref(o), C.sizeof(Op))
    return arr


def lithos_drive_open_loop(t, requests: Sequence[Sequence[Op]], arrivals_s: np.ndarray) -> np.ndarray:
    """requests: list of variants, each a list of the same number of ops."""
    per = len(requests[0])
    assert all(len(r) == per for r in requests)
    flat = _op_array([o for r in requests for o in r])
    arr = np.ascontiguousarray(arrivals_s, dtype=np.float64)
    lat = np.zeros(len(arr), dtype=np.float64)
    _check(lib().lithos_drive_open_loop(t, flat, per, len(requests), arr.ctypes.data_as(C.c_void_p), len(arr),
                                        lat.ctypes.data_as(C.c_void_p)))
    return lat


def lithos_drive_closed_loop_start(t, ops: Sequence[Op], depth=2):
    d = C.c_void_p()
    _check(lib().lithos_drive_closed_loop_start(t, _op_array(ops), len(ops), int(depth), C.byref(d)))
    return d


def lithos_drive_closed_loop_stop(d):
    it = C.c_uint64()
    sec = C.c_double()
    _check(lib().lithos_drive_closed_loop_stop(d, C.byref(it), C.byref(sec)))
    return it.value, sec.value


# ---- steppable policy core ----------------------------------------------------------------

def lithos_core_create(cfg: Optional[Config], n_groups, cus_per_group):
    c = C.c_void_p()
    _check(lib().lithos_core_create(C.byref(cfg) if cfg is not None else None, n_groups, cus_per_group, C.byref(c)))
    return c


def lithos_core_destroy(c):
    _check(lib().lithos_core_destroy(c))


def lithos_core_add_tenant(c, cls, quota_groups) -> int:
    t = C.c_int()
    _check(lib().lithos_core_add_tenant(c, cls, C.c_uint32(quota_groups), C.byref(t)))
    return t.value


def lithos_core_submit(c, tenant, total_blocks, wg_per_cu=1) -> int:
    k = C.c_uint64()
    _check(lib().lithos_core_submit(c, tenant, C.c_uint32(total_blocks), C.c_uint32(wg_per_cu), C.byref(k)))
    return k.value


def lithos_core_sync_mark(c, tenant):
    _check(lib().lithos_core_sync_mark(c, tenant))


def lithos_core_next_atom(c, tenant, now_us) -> Optional[CoreAtom]:
    a = CoreAtom()
    have = C.c_int()
    _check(lib().lithos_core_next_atom(c, tenant, C.c_double(now_us), C.byref(a), C.byref(have)))
    return a if have.value else None


def lithos_core_complete(c, atom_id, now_us, measured_us):
    _check(lib().lithos_core_complete(c, C.c_uint64(atom_id), C.c_double(now_us), C.c_double(measured_us)))


def lithos_core_stats(c, tenant) -> Stats:
    s = Stats()
    _check(lib().lithos_core_stats(c, tenant, C.byref(s)))
    return s
