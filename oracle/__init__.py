"""CPU oracle for edge-sampled SpMM -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``es_oracle.c`` (plain C, fp64 accumulation).  Only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package; the product path never does and shares no code with it.

The arithmetic lives in the C file; this module only marshals NumPy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

FULL, BUCKET, FASTRAND = 0, 1, 2
MODES = {"full": FULL, "bucket": BUCKET, "fastrand": FASTRAND}
NORMS = {"none": 0, "mean": 1, "rsqrt": 2, "rescale": 3, "inv_degree": 4}

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "es_oracle.c")
_LIB = os.path.join(_HERE, "libes_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile es_oracle.c with gcc into oracle/libes_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    # ES_ORACLE_LIBRARY: a build of es_oracle.c made elsewhere (the sanitizer
    # test points the pin suite at an ASan/UBSan-instrumented one)
    lib = ctypes.CDLL(os.environ.get("ES_ORACLE_LIBRARY") or build())
    i32p = ctypes.POINTER(ctypes.c_int32)
    i64p = ctypes.POINTER(ctypes.c_int64)
    f32p = ctypes.POINTER(ctypes.c_float)
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.es_oracle_kept.restype = ctypes.c_int
    lib.es_oracle_kept.argtypes = [i32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                   ctypes.c_uint64, i64p, ctypes.c_int64, i32p,
                                   ctypes.c_int64, i32p]
    lib.es_oracle_spmm.restype = ctypes.c_int
    lib.es_oracle_spmm.argtypes = [i32p, i32p, f32p, f32p, ctypes.c_int64, ctypes.c_int64,
                                   ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                   ctypes.c_uint64, ctypes.c_int32, i64p, ctypes.c_int64, f64p, f64p]
    lib.es_oracle_spmm_backward.restype = ctypes.c_int
    lib.es_oracle_spmm_backward.argtypes = [i32p, i32p, f32p, f32p, ctypes.c_int64, ctypes.c_int64,
                                            ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                            ctypes.c_uint64, ctypes.c_int32, f64p, f64p]
    lib.es_oracle_row_factor.restype = ctypes.c_double
    lib.es_oracle_row_factor.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64]
    lib.es_oracle_sample_index.restype = ctypes.c_int64
    lib.es_oracle_sample_index.argtypes = [ctypes.c_int32, ctypes.c_uint64, ctypes.c_int64,
                                           ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
    lib.es_oracle_kept_count.restype = ctypes.c_int64
    lib.es_oracle_kept_count.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64]
    lib.es_oracle_multiplier.restype = ctypes.c_uint32
    lib.es_oracle_multiplier.argtypes = [ctypes.c_int64]
    lib.es_oracle_offset.restype = ctypes.c_uint64
    lib.es_oracle_offset.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64]
    lib.es_oracle_splitmix64_next.restype = ctypes.c_uint64
    lib.es_oracle_splitmix64_next.argtypes = [ctypes.POINTER(ctypes.c_uint64)]
    lib.es_oracle_threads.restype = ctypes.c_int
    lib.es_oracle_threads.argtypes = []
    lib.es_oracle_set_threads.restype = ctypes.c_int
    lib.es_oracle_set_threads.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def _mode(mode) -> int:
    return MODES[mode] if isinstance(mode, str) else int(mode)


def _ptr(a: Optional[np.ndarray], ctype):
    if a is None:
        return ctypes.cast(None, ctypes.POINTER(ctype))
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _c(a, dtype) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype != dtype or not a.flags.c_contiguous:
        a = np.ascontiguousarray(a, dtype=dtype)
    return a


def threads() -> int:
    return int(_load().es_oracle_threads())


def set_threads(n: int) -> int:
    """Thread count of the row loop (timing harness only); returns the count in use."""
    return int(_load().es_oracle_set_threads(int(n)))


def sample_index(mode, seed: int, row: int, i: int, n: int, W: int) -> int:
    return int(_load().es_oracle_sample_index(_mode(mode), seed, row, i, n, W))


def kept_count(mode, n: int, W: int) -> int:
    return int(_load().es_oracle_kept_count(_mode(mode), n, W))


def multiplier(n: int) -> int:
    return int(_load().es_oracle_multiplier(n))


def offset(seed: int, row: int, n: int) -> int:
    return int(_load().es_oracle_offset(seed, row, n))


def splitmix64_stream(seed: int, count: int):
    lib = _load()
    st = ctypes.c_uint64(seed)
    return [int(lib.es_oracle_splitmix64_next(ctypes.byref(st))) for _ in range(count)]


def kept(rowptr, W: int, mode, seed: int = 0, rows: Optional[Sequence[int]] = None,
         stride: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """(pos [nrows x stride] int32 with -1 padding, cnt [nrows] int32)."""
    rowptr = _c(rowptr, np.int32)
    N = rowptr.shape[0] - 1
    m = _mode(mode)
    rows_a = None if rows is None else _c(rows, np.int64)
    nrows = N if rows_a is None else rows_a.shape[0]
    if stride is None:
        if m == FULL:
            stride = int(np.diff(rowptr).max()) if N else 0
        else:
            stride = int(W)
    pos = np.empty((nrows, stride), dtype=np.int32)
    cnt = np.empty((nrows,), dtype=np.int32)
    rc = _load().es_oracle_kept(_ptr(rowptr, ctypes.c_int32), N, int(W), m, int(seed),
                                _ptr(rows_a, ctypes.c_int64), nrows,
                                _ptr(pos, ctypes.c_int32), stride, _ptr(cnt, ctypes.c_int32))
    if rc != 0:
        raise ValueError("es_oracle_kept: bad argument")
    return pos, cnt


def row_factor(norm, n: int, k: int) -> float:
    return float(_load().es_oracle_row_factor(_norm(norm), n, k))


def _norm(norm) -> int:
    return NORMS[norm] if isinstance(norm, str) else int(norm)


def spmm(rowptr, colidx, vals, X, F: int, W: int, mode, seed: int = 0,
         rows: Optional[Sequence[int]] = None, want_denom: bool = True, norm="none"):
    """(Yref [nrows x F] float64, denom [nrows x F] float64 or None)."""
    rowptr = _c(rowptr, np.int32)
    colidx = _c(colidx, np.int32)
    vals_a = None if vals is None else _c(vals, np.float32)
    X = _c(X, np.float32)
    N = rowptr.shape[0] - 1
    ldx = X.shape[1] if X.ndim == 2 else F
    rows_a = None if rows is None else _c(rows, np.int64)
    nrows = N if rows_a is None else rows_a.shape[0]
    Y = np.empty((nrows, F), dtype=np.float64)
    D = np.empty((nrows, F), dtype=np.float64) if want_denom else None
    rc = _load().es_oracle_spmm(_ptr(rowptr, ctypes.c_int32), _ptr(colidx, ctypes.c_int32),
                                _ptr(vals_a, ctypes.c_float), _ptr(X, ctypes.c_float),
                                ldx, N, int(F), int(W), _mode(mode), int(seed), _norm(norm),
                                _ptr(rows_a, ctypes.c_int64), nrows,
                                _ptr(Y, ctypes.c_double), _ptr(D, ctypes.c_double))
    if rc != 0:
        raise ValueError("es_oracle_spmm: bad argument")
    return Y, D


def spmm_backward(rowptr, colidx, vals, dY, F: int, W: int, mode, seed: int = 0, norm="none",
                  want_denom: bool = True):
    """(dX [N x F] float64, denom [N x F] float64 or None): transposed sampled product."""
    rowptr = _c(rowptr, np.int32)
    colidx = _c(colidx, np.int32)
    vals_a = None if vals is None else _c(vals, np.float32)
    dY = _c(dY, np.float32)
    N = rowptr.shape[0] - 1
    ldy = dY.shape[1] if dY.ndim == 2 else F
    dX = np.empty((N, F), dtype=np.float64)
    D = np.empty((N, F), dtype=np.float64) if want_denom else None
    rc = _load().es_oracle_spmm_backward(_ptr(rowptr, ctypes.c_int32), _ptr(colidx, ctypes.c_int32),
                                         _ptr(vals_a, ctypes.c_float), _ptr(dY, ctypes.c_float),
                                         ldy, N, int(F), int(W), _mode(mode), int(seed), _norm(norm),
                                         _ptr(dX, ctypes.c_double), _ptr(D, ctypes.c_double))
    if rc != 0:
        raise ValueError("es_oracle_spmm_backward: bad argument")
    return dX, D
