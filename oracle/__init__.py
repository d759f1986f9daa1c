"""ctypes loader for the CPU oracle (oracle/ubp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg, never by the product package.  Compiles the C file with gcc on first
use if the shared object is missing or older than the source.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ubp_oracle.c")
_SO = os.path.join(_HERE, "libubp_oracle.so")

ORC_OK, ORC_BAD_ARG, ORC_OUT_OF_BOUNDS, ORC_OVERLAP, ORC_NOMEM = range(5)
_NAMES = {0: "ok", 1: "bad argument", 2: "block out of bounds", 3: "blocks overlap", 4: "out of memory"}


class OracleError(ValueError):
    def __init__(self, code):
        super().__init__(_NAMES.get(code, str(code)))
        self.code = code


def build(force=False):
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", tmp, _SRC])
        os.replace(tmp, _SO)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        L.ubp_oracle_validate.argtypes = [i32, i32, i32, i32, vp, i64, ctypes.POINTER(i64)]
        L.ubp_oracle_densify.argtypes = [vp, i64, i32, i32, i32, i32, vp, i64, vp]
        L.ubp_oracle_gemm_rows.argtypes = [vp, vp, i64, i32, i32, i32, vp, i32, vp, vp]
        L.ubp_oracle_spmm.argtypes = [vp, i64, i32, i32, i32, i32, vp, i64, vp, i64, i32, vp, i32, vp, vp]
        L.ubp_oracle_pack.argtypes = [vp, i64, i64, i32, i32, i32, i32, vp, i64, vp, vp, vp]
        for f in (L.ubp_oracle_validate, L.ubp_oracle_densify, L.ubp_oracle_gemm_rows,
                  L.ubp_oracle_spmm, L.ubp_oracle_pack):
            f.restype = ctypes.c_int
        _lib = L
    return _lib


def _blocks(blocks):
    b = np.ascontiguousarray(np.asarray(blocks, dtype=np.int32).reshape(-1, 2))
    return b, b.shape[0]


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def validate(M, K, bh, bw, blocks):
    """Number of kept cells; raises OracleError on an invalid list."""
    b, nb = _blocks(blocks)
    painted = ctypes.c_int64(0)
    rc = lib().ubp_oracle_validate(M, K, bh, bw, _p(b), nb, ctypes.byref(painted))
    if rc:
        raise OracleError(rc)
    return painted.value


def densify(W64, bh, bw, blocks):
    W64 = np.ascontiguousarray(W64, dtype=np.float64)
    M, K = W64.shape
    b, nb = _blocks(blocks)
    Wd = np.empty((M, K), dtype=np.float64)
    rc = lib().ubp_oracle_densify(_p(W64), K, M, K, bh, bw, _p(b), nb, _p(Wd))
    if rc:
        raise OracleError(rc)
    return Wd


def spmm(W64, bh, bw, blocks, X64, rows=None, want_abs=False):
    """Y (float64) = densified(W) @ X for all rows, or for the listed rows only."""
    W64 = np.ascontiguousarray(W64, dtype=np.float64)
    X64 = np.ascontiguousarray(X64, dtype=np.float64)
    M, K = W64.shape
    K2, N = X64.shape
    if K2 != K:
        raise ValueError("shape mismatch")
    b, nb = _blocks(blocks)
    r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    nrows = M if r is None else r.shape[0]
    Y = np.empty((nrows, N), dtype=np.float64)
    Ya = np.empty((nrows, N), dtype=np.float64) if want_abs else None
    rc = lib().ubp_oracle_spmm(_p(W64), K, M, K, bh, bw, _p(b), nb, _p(X64), N, N, _p(r), nrows, _p(Y), _p(Ya))
    if rc:
        raise OracleError(rc)
    return (Y, Ya) if want_abs else Y


def pack(W_enc, bh, bw, blocks):
    """(indptr int32[M-bh+2], indices int32[nb], values[nb*bw*bh] of W's element type)."""
    W_enc = np.ascontiguousarray(W_enc)
    M, K = W_enc.shape
    b, nb = _blocks(blocks)
    indptr = np.zeros(M - bh + 2, dtype=np.int32)
    indices = np.zeros(nb, dtype=np.int32)
    values = np.zeros(nb * bw * bh, dtype=W_enc.dtype)
    rc = lib().ubp_oracle_pack(_p(W_enc), W_enc.dtype.itemsize, K, M, K, bh, bw, _p(b), nb,
                               _p(indptr), _p(indices), _p(values))
    if rc:
        raise OracleError(rc)
    return indptr, indices, values


def fused(Y64, bias=None, activation=None, lo=0.0, hi=0.0, rows=None):
    """The epilogue of a pruned convolution applied to the exact product, in float64:
    act(Y[i][j] + bias[i]) with act = identity (None), max(v, 0) ("relu") or min(max(v, lo), hi)
    ("clamp"); max / min ignore a NaN operand, so a NaN becomes the lower bound.  `rows`: the
    output rows Y64 holds when it is not the whole of Y (then bias[rows] is added)."""
    Y = np.array(Y64, dtype=np.float64)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64)
        if rows is not None:
            b = b[np.asarray(rows)]
        Y = Y + b[:, None]
    if activation in (None, "none"):
        return Y
    if activation == "relu":
        return np.fmax(Y, 0.0)
    if activation == "clamp":
        if not lo <= hi:
            raise ValueError("clamp needs lo <= hi")
        return np.fmin(np.fmax(Y, lo), hi)
    raise ValueError(activation)
