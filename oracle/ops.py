"""ctypes front-end of the CPU oracle (``lithos_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
``cpu_baseline`` leg of the benchmark.  The product package never imports it
and it never imports the product package.

Every function takes and returns numpy arrays: fp64 for values, uint16 for
bf16 bit patterns.  The arithmetic lives in the C file; this module only
marshals arguments and (re)builds the shared object with gcc when needed.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lithos_oracle.c")
_LIB = os.path.join(_HERE, "liblithos_oracle.so")

_i64 = ctypes.c_int64
_dbl = ctypes.c_double
_pd = ctypes.POINTER(ctypes.c_double)
_pu16 = ctypes.POINTER(ctypes.c_uint16)
_pi64 = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the .so path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-D_GNU_SOURCE",
             "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.lo_bf16_to_f64.restype = _dbl
        _lib.lo_bf16_to_f64.argtypes = [ctypes.c_uint16]
        _lib.lo_f64_to_bf16.restype = ctypes.c_uint16
        _lib.lo_f64_to_bf16.argtypes = [_dbl]
        _lib.lo_gelu.restype = _dbl
        _lib.lo_gelu.argtypes = [_dbl]
        _lib.lo_num_threads.restype = ctypes.c_int
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_pd)


def _u(a):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return a, a.ctypes.data_as(_pu16)


def num_threads() -> int:
    return int(lib().lo_num_threads())


# ------------------------------------------------------------------ bf16 ---

def bf16_to_f64(bits) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp64 values (exact)."""
    b, pb = _u(bits)
    out = np.empty(b.shape, dtype=np.float64)
    lib().lo_bf16_to_f64_array(pb, out.ctypes.data_as(_pd), ctypes.c_size_t(b.size))
    return out


def f64_to_bf16(x) -> np.ndarray:
    """Round fp64 values to bf16 bit patterns (nearest, ties to even)."""
    a, pa = _d(x)
    out = np.empty(a.shape, dtype=np.uint16)
    lib().lo_f64_to_bf16_array(pa, out.ctypes.data_as(_pu16), ctypes.c_size_t(a.size))
    return out


def round_bf16(x) -> np.ndarray:
    """Value-level bf16 rounding: nearest bf16 of each element, as fp64."""
    a, pa = _d(x)
    out = np.empty(a.shape, dtype=np.float64)
    lib().lo_round_bf16_array(pa, out.ctypes.data_as(_pd), ctypes.c_size_t(a.size))
    return out


def round_bf16x2(x) -> np.ndarray:
    """Value of a split-bf16 pair: hi + lo with hi = bf16(x), lo = bf16(x - hi)."""
    a = np.asarray(x, dtype=np.float64)
    hi = round_bf16(a)
    return hi + round_bf16(a - hi)


# ------------------------------------------------------------------ GEMM ---

def gemm(a, b_bits, ta: bool = False, tb: bool = False, fast: bool = True) -> np.ndarray:
    """fp64 C = op(A) @ op(B), ascending-k sums.

    ``a`` is [M,K] (or [K,M] when ``ta``): bf16 bit patterns (uint16) or the
    activations' values as floats (for kernels that read fp32 activations).
    ``b_bits`` is [K,N] (or [N,K] when ``tb``), bf16 bit patterns.  ``fast``
    picks the (i,k,j) loop order for non-transposed B; each element's
    summation order is unchanged, so the result is bit-equal.
    """
    a = np.asarray(a)
    A, pA = _d(bf16_to_f64(a) if a.dtype == np.uint16 else a)
    B, pB = _u(b_bits)
    if A.ndim != 2 or B.ndim != 2:
        raise ValueError("gemm expects 2-D operands")
    M, K = (A.shape[1], A.shape[0]) if ta else A.shape
    Kb, N = (B.shape[1], B.shape[0]) if tb else B.shape
    if K != Kb:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, Kb))
    C = np.empty((M, N), dtype=np.float64)
    if fast and not tb:
        rc = lib().lo_gemm_rowsweep(int(ta), _i64(M), _i64(N), _i64(K), pA, _i64(A.shape[1]),
                                    pB, _i64(B.shape[1]), C.ctypes.data_as(_pd), _i64(N))
    else:
        rc = lib().lo_gemm(int(ta), int(tb), _i64(M), _i64(N), _i64(K), pA, _i64(A.shape[1]),
                           pB, _i64(B.shape[1]), C.ctypes.data_as(_pd), _i64(N))
    if rc != 0:
        raise ValueError("lo_gemm rejected its arguments")
    return C


# ------------------------------------------------------------- row ops -----

def gelu(u: float) -> float:
    return float(lib().lo_gelu(_dbl(u)))


def k_slice_bounds(k: int, slices: int, ktile: int = 64):
    """Balanced cut of K into ``slices`` ranges of whole ``ktile``-wide steps:
    range z holds the steps [z*KT/S, (z+1)*KT/S) of the KT = ceil(K/ktile) steps."""
    kt = -(-k // ktile)
    return [(min(k, (z * kt // slices) * ktile), min(k, ((z + 1) * kt // slices) * ktile)) for z in range(slices)]


def sum_slices(planes) -> np.ndarray:
    """Sum of the partial products of a GEMM whose K was cut into ranges, plane 0 first."""
    p, pp = _d(planes)
    out = np.empty(p.shape[1:], dtype=np.float64)
    rc = lib().lo_sum_slices(_i64(p.shape[0]), _i64(out.size), pp, out.ctypes.data_as(_pd))
    assert rc == 0
    return out


def bias_act(x, bias=None, gelu: bool = True) -> np.ndarray:
    """y = g(x + bias) (g = erf-GELU, or identity when ``gelu`` is False)."""
    a, pa = _d(x)
    rows, cols = a.reshape(-1, a.shape[-1]).shape
    if bias is not None:
        b, pb = _d(bias)
        if b.shape != (cols,):
            raise ValueError("bias shape")
    else:
        pb = None
    y = np.empty_like(a)
    rc = lib().lo_bias_act(_i64(rows), _i64(cols), pa, pb, int(gelu), y.ctypes.data_as(_pd))
    assert rc == 0
    return y


def layernorm(x, gamma, beta, eps: float = 1e-5) -> np.ndarray:
    a, pa = _d(x)
    H = a.shape[-1]
    g, pg = _d(gamma)
    b, pb = _d(beta)
    if g.shape != (H,) or b.shape != (H,):
        raise ValueError("gamma/beta shape")
    y = np.empty_like(a)
    rc = lib().lo_layernorm(_i64(a.size // H), _i64(H), pa, pg, pb, _dbl(eps), y.ctypes.data_as(_pd))
    assert rc == 0
    return y


def rmsnorm(x, w, eps: float = 1e-5) -> np.ndarray:
    a, pa = _d(x)
    H = a.shape[-1]
    g, pg = _d(w)
    if g.shape != (H,):
        raise ValueError("weight shape")
    y = np.empty_like(a)
    rc = lib().lo_rmsnorm(_i64(a.size // H), _i64(H), pa, pg, _dbl(eps), y.ctypes.data_as(_pd))
    assert rc == 0
    return y


def softmax(s) -> np.ndarray:
    a, pa = _d(s)
    n = a.shape[-1]
    p = np.empty_like(a)
    rc = lib().lo_softmax(_i64(a.size // n), _i64(n), pa, p.ctypes.data_as(_pd))
    assert rc == 0
    return p


def attention(q, k, v, scale: float) -> np.ndarray:
    """q [B,Sq,Hq,d], k/v [B,Sk,Hkv,d] (any strides) -> o [B,Sq,Hq,d] fp64.

    Query head h reads key/value head h // (Hq/Hkv); no mask.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    Bn, Sq, Hq, d = q.shape
    _, Sk, Hkv, _ = k.shape
    if k.shape != v.shape or k.shape[0] != Bn or k.shape[3] != d:
        raise ValueError("attention operand shapes")
    for t in (q, k, v):
        if t.strides[-1] != 8:
            raise ValueError("innermost dimension must be contiguous")
    o = np.empty((Bn, Sq, Hq, d), dtype=np.float64)

    def st(t):
        return [_i64(t.strides[0] // 8), _i64(t.strides[1] // 8), _i64(t.strides[2] // 8)]

    rc = lib().lo_attention(_i64(Bn), _i64(Hq), _i64(Hkv), _i64(Sq), _i64(Sk), _i64(d),
                            q.ctypes.data_as(_pd), *st(q),
                            k.ctypes.data_as(_pd), *st(k),
                            v.ctypes.data_as(_pd), *st(v),
                            _dbl(scale),
                            o.ctypes.data_as(_pd), *st(o))
    if rc != 0:
        raise ValueError("lo_attention rejected its arguments")
    return o


def attention_causal(q, k, v, scale: float) -> np.ndarray:
    """Causal self-attention over a prompt: q [B,S,Hq,d], k/v [B,S,Hkv,d] -> o [B,S,Hq,d] fp64;
    query i sees keys 0..i.  Grouped-query rule as in ``attention``."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    Bn, S, Hq, d = q.shape
    if k.shape != v.shape or k.shape[0] != Bn or k.shape[1] != S or k.shape[3] != d:
        raise ValueError("attention operand shapes")
    Hkv = k.shape[2]
    for t in (q, k, v):
        if t.strides[-1] != 8:
            raise ValueError("innermost dimension must be contiguous")
    o = np.empty((Bn, S, Hq, d), dtype=np.float64)

    def st(t):
        return [_i64(t.strides[0] // 8), _i64(t.strides[1] // 8), _i64(t.strides[2] // 8)]

    rc = lib().lo_attention_causal(_i64(Bn), _i64(Hq), _i64(Hkv), _i64(S), _i64(d),
                                   q.ctypes.data_as(_pd), *st(q), k.ctypes.data_as(_pd), *st(k),
                                   v.ctypes.data_as(_pd), *st(v), _dbl(scale), o.ctypes.data_as(_pd), *st(o))
    if rc != 0:
        raise ValueError("lo_attention_causal rejected its arguments")
    return o


def rope(x, pos, theta: float = 10000.0) -> np.ndarray:
    """x [rows, heads, d]; pos [rows] int; rotate-half pairing."""
    a, pa = _d(x)
    rows, heads, d = a.shape
    p = np.ascontiguousarray(pos, dtype=np.int64)
    if p.shape != (rows,):
        raise ValueError("pos shape")
    y = np.empty_like(a)
    rc = lib().lo_rope(_i64(rows), _i64(heads), _i64(d), pa, p.ctypes.data_as(_pi64),
                       _dbl(theta), y.ctypes.data_as(_pd))
    if rc != 0:
        raise ValueError("lo_rope rejected its arguments")
    return y


def silu_mul(g, u) -> np.ndarray:
    a, pa = _d(g)
    b, pb = _d(u)
    if a.shape != b.shape:
        raise ValueError("shape mismatch")
    y = np.empty_like(a)
    lib().lo_silu_mul(ctypes.c_size_t(a.size), pa, pb, y.ctypes.data_as(_pd))
    return y
