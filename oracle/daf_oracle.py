"""ctypes + numpy face of the C++ oracle (oracle/daf_oracle.cpp).

TEST INFRASTRUCTURE.  Arrays in, arrays out.  The quantize / pack / unpack / dequantize path, the
plan, the random numbers, the reductions and the width rule are thin calls into the C++ code,
which is where the method is written down.  Three plain definitions that the fused GPU calls
are checked against are written out here in numpy instead: `relu` (max(z, +0) on the element
format), `relu_backward` (grad where xhat > 0) and `grad_weight` (the matrix product in double
precision).  16-bit inputs travel as uint16 bit patterns (numpy has no bfloat16).
"""
import ctypes
import os

import numpy as np

from . import build as _build

F32, F16, BF16 = 0, 1, 2
_NP = {F32: np.float32, F16: np.uint16, BF16: np.uint16}

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        c = ctypes
        vp, i64, i32, u64 = c.c_void_p, c.c_int64, c.c_int32, c.c_uint64
        L.daf_oracle_rand_bits.restype = c.c_int
        L.daf_oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.daf_oracle_rand.argtypes = [u64, u64]
        L.daf_oracle_rand.restype = c.c_uint32
        L.daf_oracle_widen.argtypes = [vp, c.c_int, i64, vp]
        L.daf_oracle_narrow.argtypes = [vp, c.c_int, i64, vp]
        L.daf_oracle_minmax.argtypes = [vp, c.c_int, i64, vp]
        L.daf_oracle_group_metrics.argtypes = [vp, c.c_int, i64, i32, vp, vp, vp, vp]
        L.daf_oracle_group_variance.argtypes = [vp, c.c_int, i64, i32, vp, i64, vp]
        L.daf_oracle_group_variance.restype = None
        L.daf_oracle_group_minmax.argtypes = [vp, c.c_int, i64, i32, vp, vp]
        L.daf_oracle_select_bits.argtypes = [vp, vp, i64, vp, i32, vp]
        L.daf_oracle_select_bits.restype = c.c_int
        L.daf_oracle_plan.argtypes = [i64, i32, vp, i64, vp]
        L.daf_oracle_plan.restype = i64
        L.daf_oracle_quantize_pack.argtypes = [vp, c.c_int, i64, i32, vp, i64, u64, vp, vp, vp, vp]
        L.daf_oracle_quantize_pack.restype = c.c_int
        L.daf_oracle_quantize_pack_range.argtypes = [vp, c.c_int, i64, i32, vp, i64, vp, u64, i64, i64,
                                                     vp, vp, vp, vp]
        L.daf_oracle_quantize_pack_range.restype = c.c_int
        L.daf_oracle_unpack_dequantize.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, c.c_int, vp]
        L.daf_oracle_unpack_dequantize.restype = c.c_int
        L.daf_oracle_unpack_dequantize_range.argtypes = [vp, vp, vp, vp, i64, vp, i64, i32, i64, i64,
                                                         vp, c.c_int, vp]
        L.daf_oracle_unpack_dequantize_range.restype = c.c_int
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _bits_arr(bits, G):
    b = np.ascontiguousarray(np.atleast_1d(np.asarray(bits)).astype(np.uint8))
    if b.size not in (1, G):
        raise ValueError("bits must have 1 or G entries")
    return b


def rand_bits() -> int:
    return int(lib().daf_oracle_rand_bits())


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    o = np.zeros(4, dtype=np.uint32)
    lib().daf_oracle_philox4x32_10(_p(c), _p(k), _p(o))
    return o


def rand(seed: int, i: int) -> int:
    return int(lib().daf_oracle_rand(seed, i))


def widen(x: np.ndarray, dtype: int) -> np.ndarray:
    x = np.ascontiguousarray(x.reshape(-1), dtype=_NP[dtype])
    out = np.empty(x.size, dtype=np.float32)
    lib().daf_oracle_widen(_p(x), dtype, x.size, _p(out))
    return out


def narrow(x: np.ndarray, dtype: int) -> np.ndarray:
    x = np.ascontiguousarray(x.reshape(-1), dtype=np.float32)
    out = np.empty(x.size, dtype=_NP[dtype])
    lib().daf_oracle_narrow(_p(x), dtype, x.size, _p(out))
    return out


def relu(x: np.ndarray, dtype: int) -> np.ndarray:
    """y = x if x > 0 else +0, element by element, in the element format (x: float32 values, or
    uint16 bit patterns for F16/BF16; same representation returned).  The activation function
    whose output the fused producer call stores and quantizes (Sec. 3.2.3)."""
    x = np.ascontiguousarray(x.reshape(-1), dtype=_NP[dtype])
    v = widen(x, dtype)                     # exact
    return np.where(v > 0, x, np.zeros_like(x))


def relu_backward(xhat: np.ndarray, grad_y: np.ndarray, dtype: int) -> np.ndarray:
    """grad_z = grad_y where xhat > 0, else +0 (backward of y = max(z, 0) seen through the
    dequantized y); all arrays in the element format (float32, or uint16 bit patterns)."""
    xhat = np.ascontiguousarray(xhat.reshape(-1), dtype=_NP[dtype])
    grad_y = np.ascontiguousarray(grad_y.reshape(-1), dtype=_NP[dtype])
    return np.where(widen(xhat, dtype) > 0, grad_y, np.zeros_like(grad_y))


def grad_weight(xhat: np.ndarray, grad_y: np.ndarray, m: int, k: int, n: int, dtype: int) -> np.ndarray:
    """Weight gradient of y = x W^T seen through the dequantized activation:
    dW[j, c] = sum_i grad_y[i, j] * xhat[i, c], float64[n, k].  xhat is [m, k] and grad_y is [m, n],
    both in the element format (float32, or uint16 bit patterns); the products and the sum are
    evaluated in double precision (each product of two 16-bit-format values is exact in it)."""
    xh = widen(xhat, dtype).astype(np.float64).reshape(m, k)
    gy = widen(grad_y, dtype).astype(np.float64).reshape(m, n)
    return gy.T @ xh


def linear_forward(x: np.ndarray, w: np.ndarray, m: int, k: int, n: int, dtype: int) -> np.ndarray:
    """Forward pass of a linear layer, y = x W^T: y[i, j] = sum_c x[i, c] * w[j, c], x [m, k] and
    w [n, k] in the element format (float32, or uint16 bit patterns).  Products and sum are
    evaluated in double precision (each product of two 16-bit-format values is exact in it), the
    sum is rounded to binary32 and then to the element format with `narrow` (nearest even).
    Returned flat, [m * n], in the element format.  Where the double-precision sum is itself a
    binary32 value (small-integer inputs, as the bit-exact GPU tests use) the result is the
    correctly rounded product; in general the two roundings can differ from a single one in the
    last place, and from a binary32 accumulation by its rounding errors: tests on general
    inputs compare with a tolerance."""
    xd = widen(x, dtype).astype(np.float64).reshape(m, k)
    wd = widen(w, dtype).astype(np.float64).reshape(n, k)
    return narrow((xd @ wd.T).astype(np.float32).reshape(-1), dtype)


def minmax(x: np.ndarray, dtype: int) -> np.ndarray:
    """Whole-tensor (min, max) as float32[2]."""
    x = np.ascontiguousarray(x.reshape(-1), dtype=_NP[dtype])
    out = np.empty(2, dtype=np.float32)
    lib().daf_oracle_minmax(_p(x), dtype, x.size, _p(out))
    return out


def group_metrics(x: np.ndarray, dtype: int, gs: int, codes, mn, sc) -> np.ndarray:
    """float64[G, 2]: per group, sum (x - xhat)^2 and sum x^2."""
    x = np.ascontiguousarray(x.reshape(-1), dtype=_NP[dtype])
    G = (x.size + gs - 1) // gs
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    mn = np.ascontiguousarray(mn, dtype=np.float32)
    sc = np.ascontiguousarray(sc, dtype=np.float32)
    out = np.empty((G, 2), dtype=np.float64)
    lib().daf_oracle_group_metrics(_p(x), dtype, x.size, gs, _p(codes), _p(mn), _p(sc), _p(out))
    return out


def group_variance(x: np.ndarray, dtype: int, gs: int, bits) -> np.ndarray:
    """float64[G]: per group, the variance of xhat under the stochastic rounding."""
    x = np.ascontiguousarray(x.reshape(-1), dtype=_NP[dtype])
    G = (x.size + gs - 1) // gs
    b = _bits_arr(bits, G)
    out = np.empty(G, dtype=np.float64)
    lib().daf_oracle_group_variance(_p(x), dtype, x.size, gs, _p(b), b.size, _p(out))
    return out


def group_minmax(x: np.ndarray, dtype: int, gs: int):
    """Per-group (min[G], max[G]) as float32."""
    x = np.ascontiguousarray(x.reshape(-1), dtype=_NP[dtype])
    G = (x.size + gs - 1) // gs
    mn = np.empty(G, dtype=np.float32)
    mx = np.empty(G, dtype=np.float32)
    lib().daf_oracle_group_minmax(_p(x), dtype, x.size, gs, _p(mn), _p(mx))
    return mn, mx


def select_bits(gmin: np.ndarray, gmax: np.ndarray, classes) -> np.ndarray:
    """Width per group by rank quantiles of the range (smallest range -> classes[0])."""
    gmin = np.ascontiguousarray(gmin, dtype=np.float32)
    gmax = np.ascontiguousarray(gmax, dtype=np.float32)
    cl = np.ascontiguousarray(classes, dtype=np.uint8)
    out = np.empty(gmin.size, dtype=np.uint8)
    if lib().daf_oracle_select_bits(_p(gmin), _p(gmax), gmin.size, _p(cl), cl.size, _p(out)) != 0:
        raise ValueError("daf_oracle_select_bits rejected the arguments")
    return out


def num_groups(n: int, gs: int) -> int:
    return (n + gs - 1) // gs


def plan(n: int, gs: int, bits):
    """Returns (off[G] uint32, total_words)."""
    G = num_groups(n, gs)
    b = _bits_arr(bits, G)
    off = np.empty(G, dtype=np.uint32)
    total = lib().daf_oracle_plan(n, gs, _p(b), b.size, _p(off))
    if total < 0:
        raise ValueError("daf_oracle_plan rejected the arguments")
    return off, int(total)


def quantize_pack(x: np.ndarray, dtype: int, gs: int, bits, seed: int, want_codes: bool = False):
    """x: flat float32 array, or uint16 bit patterns for F16/BF16.
    Returns (words uint32[total], min float32[G], scale float32[G], codes uint8[N] or None)."""
    x = np.ascontiguousarray(x.reshape(-1), dtype=_NP[dtype])
    n = x.size
    G = num_groups(n, gs)
    b = _bits_arr(bits, G)
    _, total = plan(n, gs, b)
    words = np.empty(total, dtype=np.uint32)
    mn = np.empty(G, dtype=np.float32)
    sc = np.empty(G, dtype=np.float32)
    codes = np.empty(n, dtype=np.uint8) if want_codes else None
    rc = lib().daf_oracle_quantize_pack(_p(x), dtype, n, gs, _p(b), b.size, seed,
                                        _p(words), _p(mn), _p(sc), _p(codes))
    if rc != 0:
        raise ValueError("daf_oracle_quantize_pack failed")
    return words, mn, sc, codes


def quantize_pack_range(x, dtype, gs, bits, off, seed, g_begin, g_end, words, mn, sc):
    """Groups [g_begin, g_end) only, into caller-provided arrays (used to time the oracle
    from several threads over disjoint ranges; ctypes drops the GIL during the call)."""
    n = x.size
    b = _bits_arr(bits, num_groups(n, gs))
    return lib().daf_oracle_quantize_pack_range(_p(x), dtype, n, gs, _p(b), b.size, _p(off), seed,
                                                g_begin, g_end, _p(words), _p(mn), _p(sc), None)


def unpack_dequantize(words, mn, sc, bits, n: int, gs: int, dtype: int, want_codes: bool = False):
    """Returns (xhat as float32 or uint16 bit patterns, codes or None)."""
    G = num_groups(n, gs)
    b = _bits_arr(bits, G)
    words = np.ascontiguousarray(words, dtype=np.uint32)
    mn = np.ascontiguousarray(mn, dtype=np.float32)
    sc = np.ascontiguousarray(sc, dtype=np.float32)
    out = np.empty(n, dtype=_NP[dtype])
    codes = np.empty(n, dtype=np.uint8) if want_codes else None
    rc = lib().daf_oracle_unpack_dequantize(_p(words), _p(mn), _p(sc), _p(b), b.size, n, gs,
                                            _p(out), dtype, _p(codes))
    if rc != 0:
        raise ValueError("daf_oracle_unpack_dequantize failed")
    return out, codes


def unpack_dequantize_range(words, mn, sc, bits, off, n, gs, g_begin, g_end, out, dtype):
    b = _bits_arr(bits, num_groups(n, gs))
    return lib().daf_oracle_unpack_dequantize_range(_p(words), _p(mn), _p(sc), _p(b), b.size, _p(off),
                                                    n, gs, g_begin, g_end, _p(out), dtype, None)
