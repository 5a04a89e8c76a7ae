"""ctypes front end of ``ffn_oracle.c`` -- TEST INFRASTRUCTURE ONLY (see package docstring).

Operand arrays are passed as their stored bit patterns:
  * bf16  -> ``numpy.uint16`` holding the upper 16 bits of the binary32 pattern
  * fp16  -> ``numpy.float16``
  * fp32  -> ``numpy.float32``
and are widened exactly to double inside the C code.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import numpy as np

ACT_IDENTITY, ACT_RELU, ACT_GELU_TANH, ACT_SILU = 0, 1, 2, 3
_DT_BF16, _DT_F16, _DT_F32 = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ffn_oracle.c")
_LIB = os.path.join(_HERE, "libffn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only).  Returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=native", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.orc_ffn_rows.restype = ctypes.c_int
        lib.orc_ffn_rows.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int, ctypes.c_int] + \
            [ctypes.c_int64] * 4 + [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        lib.orc_conv_chain.restype = ctypes.c_int
        lib.orc_conv_chain.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int, ctypes.c_int] + [ctypes.c_int64] * 8 + \
            [ctypes.c_void_p, ctypes.c_void_p]
        lib.orc_act.restype = ctypes.c_double
        lib.orc_act.argtypes = [ctypes.c_int, ctypes.c_double]
        lib.orc_widen.restype = None
        lib.orc_widen.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_void_p]
        lib.orc_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _dtype_code(a: np.ndarray, bf16: bool) -> int:
    if a.dtype == np.uint16:
        if not bf16:
            raise TypeError("uint16 arrays are bf16 bit patterns; pass bf16=True")
        return _DT_BF16
    if bf16:
        raise TypeError("bf16=True needs uint16 bit patterns")
    if a.dtype == np.float16:
        return _DT_F16
    if a.dtype == np.float32:
        return _DT_F32
    raise TypeError(f"unsupported operand dtype {a.dtype}")


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().orc_num_threads())


def act(kind: int, x: float) -> float:
    return float(_load().orc_act(int(kind), float(x)))


def widen(a: np.ndarray, bf16: bool = False) -> np.ndarray:
    a = np.ascontiguousarray(a)
    out = np.empty(a.shape, dtype=np.float64)
    _load().orc_widen(_ptr(a), _dtype_code(a, bf16), a.size, _ptr(out))
    return out


def ffn_rows(X, W1, W3, W2, act_kind: int, rows=None, bf16: bool = False, want_h: bool = False):
    """Rows ``rows`` (default: all) of ``Y = act(X W1) [* (X W3)] W2`` in double.

    Returns ``Y`` (len(rows) x N2 float64), or ``(Y, H)`` if ``want_h``.
    """
    X = np.ascontiguousarray(X)
    W1 = np.ascontiguousarray(W1)
    W2 = np.ascontiguousarray(W2)
    if W3 is not None:
        W3 = np.ascontiguousarray(W3)
    M, K = X.shape
    K1, N1 = W1.shape
    N1b, N2 = W2.shape
    if K1 != K or N1b != N1 or (W3 is not None and W3.shape != W1.shape):
        raise ValueError("shape mismatch")
    dt = _dtype_code(X, bf16)
    for w in (W1, W2) + ((W3,) if W3 is not None else ()):
        if _dtype_code(w, bf16) != dt:
            raise TypeError("operands must share one dtype")
    if rows is None:
        rows_arr, nrows, rows_p = None, M, None
    else:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        nrows, rows_p = rows_arr.size, _ptr(rows_arr)
    Y = np.empty((nrows, N2), dtype=np.float64)
    H = np.empty((nrows, N1), dtype=np.float64) if want_h else None
    rc = _load().orc_ffn_rows(_ptr(X), _ptr(W1), _ptr(W3) if W3 is not None else None, _ptr(W2),
                              dt, int(act_kind), M, K, N1, N2, rows_p, nrows, _ptr(Y),
                              _ptr(H) if want_h else None)
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return (Y, H) if want_h else Y


def ffn(X, W1, W3, W2, act_kind: int, bf16: bool = False):
    return ffn_rows(X, W1, W3, W2, act_kind, None, bf16)


def conv_chain(X, W1, W2, act_kind: int, bf16: bool = False, want_a: bool = False):
    """``Y = conv_k2(act(conv_k1(X, W1)), W2)`` in double: stride 1, zero padding k/2,
    cross-correlation, no bias.  X is [B][H][W][IC], W1 [k1][k1][IC][OC1], W2 [k2][k2][OC1][OC2];
    returns Y [B][H][W][OC2] float64, or ``(Y, A)`` with the activated intermediate."""
    X = np.ascontiguousarray(X)
    W1 = np.ascontiguousarray(W1)
    W2 = np.ascontiguousarray(W2)
    B, H, W, IC = X.shape
    k1, k1b, ICb, OC1 = W1.shape
    k2, k2b, OC1b, OC2 = W2.shape
    if k1 != k1b or k2 != k2b or ICb != IC or OC1b != OC1:
        raise ValueError("shape mismatch")
    dt = _dtype_code(X, bf16)
    if _dtype_code(W1, bf16) != dt or _dtype_code(W2, bf16) != dt:
        raise TypeError("operands must share one dtype")
    Y = np.empty((B, H, W, OC2), dtype=np.float64)
    A = np.empty((B, H, W, OC1), dtype=np.float64) if want_a else None
    rc = _load().orc_conv_chain(_ptr(X), _ptr(W1), _ptr(W2), dt, int(act_kind), B, H, W, IC, OC1, OC2, k1, k2,
                                _ptr(Y), _ptr(A) if want_a else None)
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return (Y, A) if want_a else Y
