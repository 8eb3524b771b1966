"""ctypes front end of the fp64 definition oracle (oracle/bb_oracle.c).

TEST INFRASTRUCTURE ONLY: importable from tests/, from the smoke check and
from the bench's cpu_baseline leg.  Nothing here touches the GPU library and
nothing in the GPU library touches this.

Arrays are numpy ``uint16`` holding bf16 bit patterns (a CPU torch bf16 tensor
is accepted and reinterpreted); results are numpy ``float64``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bb_oracle.c")
_LIB = os.path.join(_HERE, "libbb_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp).  Returns the library path."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
           "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i64p = ctypes.POINTER(ctypes.c_int64)
        i64 = ctypes.c_int64
        lib.bb_oracle_rmsnorm_swiglu_ffn.argtypes = [
            u16p, u16p, u16p, u16p, u16p, f64p, i64, i64, i64,
            ctypes.c_double, i64p, i64]
        lib.bb_oracle_rmsnorm_swiglu_ffn.restype = ctypes.c_int
        lib.bb_oracle_layernorm_matmul.argtypes = [
            u16p, u16p, u16p, u16p, f64p, i64, i64, i64,
            ctypes.c_double, i64p, i64]
        lib.bb_oracle_layernorm_matmul.restype = ctypes.c_int
        lib.bb_oracle_attention.argtypes = [
            u16p, u16p, u16p, f64p, i64, i64, i64, i64, i64, i64p, i64]
        lib.bb_oracle_attention.restype = ctypes.c_int
        lib.bb_oracle_num_threads.restype = ctypes.c_int
        lib.bb_oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _bits(a, shape) -> np.ndarray:
    """bf16 bit patterns as a C-contiguous uint16 array of the given shape."""
    if hasattr(a, "detach"):          # torch tensor
        import torch
        if a.dtype != torch.bfloat16:
            raise TypeError("torch inputs must be bfloat16")
        a = a.detach().cpu().contiguous().view(torch.uint16).numpy()
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("inputs must be uint16 bf16 bit patterns")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"shape {a.shape} != expected {tuple(shape)}")
    return a


def _p16(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _rows(rows: Optional[Sequence[int]], M: int):
    if rows is None:
        return None, None, M
    r = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    return r, r.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), int(r.size)


def num_threads() -> int:
    return int(_load().bb_oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().bb_oracle_set_num_threads(int(n))


def float32_eps(eps: float) -> float:
    """The GPU entry points take eps as a C float; the oracle uses that value."""
    return float(np.float32(eps))


def rmsnorm_swiglu_ffn(X, g, W1, W3, W2, eps: float,
                       rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Definition of Example 3's array program with mean/eps/gain (see the C
    file).  X [M,D], g [D], W1,W3 [D,F], W2 [F,D]  ->  float64 [nrows, D]."""
    lib = _load()
    M, D = (int(s) for s in X.shape)
    F = int(W1.shape[1])
    Xb, gb = _bits(X, (M, D)), _bits(g, (D,))
    W1b, W3b, W2b = _bits(W1, (D, F)), _bits(W3, (D, F)), _bits(W2, (F, D))
    keep, rp, n = _rows(rows, M)
    Y = np.empty((n, D), dtype=np.float64)
    rc = lib.bb_oracle_rmsnorm_swiglu_ffn(
        _p16(Xb), _p16(gb), _p16(W1b), _p16(W3b), _p16(W2b),
        Y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        M, D, F, float32_eps(eps), rp, n)
    del keep
    if rc != 0:
        raise RuntimeError("bb_oracle_rmsnorm_swiglu_ffn failed")
    return Y


def rmsnorm_swiglu_ffn_residual(X, g, W1, W3, W2, R, eps: float,
                                rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """The operator above followed by the residual connection of a decoder
    block: R + FFN(X), R [M,D] (bf16 values, added in float64)."""
    Y = rmsnorm_swiglu_ffn(X, g, W1, W3, W2, eps, rows)
    M, D = (int(s) for s in X.shape)
    Rf = R.reshape(M, D).to(dtype=__import__("torch").float64).numpy()
    return Y + (Rf if rows is None else Rf[np.asarray(list(rows), dtype=np.int64)])


def layernorm_matmul(X, gamma, beta, W, eps: float,
                     rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Definition of Example 2's array program with gamma/beta/eps.
    X [M,D], gamma,beta [D], W [D,N]  ->  float64 [nrows, N]."""
    lib = _load()
    M, D = (int(s) for s in X.shape)
    N = int(W.shape[1])
    Xb = _bits(X, (M, D))
    gb, bb = _bits(gamma, (D,)), _bits(beta, (D,))
    Wb = _bits(W, (D, N))
    keep, rp, n = _rows(rows, M)
    Y = np.empty((n, N), dtype=np.float64)
    rc = lib.bb_oracle_layernorm_matmul(
        _p16(Xb), _p16(gb), _p16(bb), _p16(Wb),
        Y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        M, D, N, float32_eps(eps), rp, n)
    del keep
    if rc != 0:
        raise RuntimeError("bb_oracle_layernorm_matmul failed")
    return Y


def attention(Q, K, V, rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Definition of Example 1's array program, softmax(Q K^T / sqrt(d)) V, per
    batch entry.  Q [B,M,d], K [B,N,d], V [B,N,dv]  ->  float64 [nrows, dv];
    rows index the B*M flattened query rows (None = all, in order)."""
    lib = _load()
    B, M, d = (int(s) for s in Q.shape)
    N, dv = int(K.shape[1]), int(V.shape[2])
    Qb, Kb, Vb = _bits(Q, (B, M, d)), _bits(K, (B, N, d)), _bits(V, (B, N, dv))
    keep, rp, n = _rows(rows, B * M)
    O = np.empty((n, dv), dtype=np.float64)
    rc = lib.bb_oracle_attention(
        _p16(Qb), _p16(Kb), _p16(Vb), O.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        B, M, N, d, dv, rp, n)
    del keep
    if rc != 0:
        raise RuntimeError("bb_oracle_attention failed")
    return O
