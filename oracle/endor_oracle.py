"""numpy-facing loader for the CPU oracle (``endor_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this module; the product package never does.  It marshals numpy arrays into the
plain-C oracle and holds no arithmetic of its own: every loop of Algorithms 1
and 2 (Section 4.1) lives in the C file.

The C file is compiled with gcc into ``oracle/liboracle.so`` on first use (or
by ``build_oracle()``); compiling the checker is not using it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "endor_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lock = threading.Lock()
_lib = None

_i64 = ctypes.c_int64
_p = ctypes.c_void_p


def build_oracle(force: bool = False) -> str:
    """Compile endor_oracle.c with gcc.  Returns the path of the shared object."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build_oracle())
            lib.oracle_bitmap_bytes.restype = _i64
            lib.oracle_bitmap_bytes.argtypes = [_i64, _i64]
            lib.oracle_compress.restype = _i64
            lib.oracle_compress.argtypes = [_p, ctypes.c_int, _i64, _i64, _p, _p, _p]
            lib.oracle_decompress.restype = _i64
            lib.oracle_decompress.argtypes = [ctypes.c_int, _i64, _i64, _p, _p, _p]
            lib.oracle_decompress_rows.restype = _i64
            lib.oracle_decompress_rows.argtypes = [ctypes.c_int, _i64, _i64, _i64, _i64, _p, _p, _p]
            lib.oracle_row_offsets.restype = None
            lib.oracle_row_offsets.argtypes = [_i64, _i64, _p, _p]
            lib.oracle_tile_offsets.restype = None
            lib.oracle_tile_offsets.argtypes = [_i64, _i64, _p, _p]
            lib.oracle_decompress_selected_rows.restype = None
            lib.oracle_decompress_selected_rows.argtypes = [ctypes.c_int, _i64, _p, _i64, _p, _p, _p, _p]
            lib.oracle_half_to_double_array.restype = None
            lib.oracle_half_to_double_array.argtypes = [_p, _i64, _p]
            lib.oracle_gemv_f16.restype = None
            lib.oracle_gemv_f16.argtypes = [_i64, _i64, _p, _p, _p, _p]
            lib.oracle_gemm_f16_rows.restype = None
            lib.oracle_gemm_f16_rows.argtypes = [_i64, _i64, _i64, _i64, _p, _p, _i64, _p]
            _lib = lib
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _elem_dtype(elem_bytes: int):
    return {1: np.uint8, 2: np.uint16}[elem_bytes]


def _as_patterns(dense: np.ndarray) -> np.ndarray:
    """View a 2-d float16 / int8 / uint8 / uint16 matrix as its raw bit patterns."""
    if dense.ndim != 2:
        raise ValueError("dense must be 2-d")
    if dense.dtype.itemsize not in (1, 2):
        raise ValueError("elements must be 1 or 2 bytes wide")
    return np.ascontiguousarray(dense).view(_elem_dtype(dense.dtype.itemsize))


def bitmap_bytes(rows: int, cols: int) -> int:
    return int(_load().oracle_bitmap_bytes(rows, cols))


def compress(dense: np.ndarray):
    """Algorithm 1.  Returns (bitmap uint8[ceil(N/8)], values, row_offsets int64[rows+1])."""
    lib = _load()
    W = _as_patterns(dense)
    rows, cols = W.shape
    eb = W.dtype.itemsize
    bitmap = np.empty(bitmap_bytes(rows, cols), dtype=np.uint8)
    values = np.empty(rows * cols, dtype=W.dtype)
    row_offsets = np.empty(rows + 1, dtype=np.int64)
    nnz = lib.oracle_compress(_ptr(W), eb, rows, cols, _ptr(bitmap), _ptr(values), _ptr(row_offsets))
    return bitmap, values[:nnz].copy(), row_offsets


def decompress(rows: int, cols: int, bitmap: np.ndarray, values: np.ndarray) -> np.ndarray:
    """Algorithm 2.  Returns the dense matrix as raw patterns (dtype of ``values``)."""
    lib = _load()
    bitmap = np.ascontiguousarray(bitmap, dtype=np.uint8)
    values = np.ascontiguousarray(values)
    eb = values.dtype.itemsize
    if bitmap.size < bitmap_bytes(rows, cols):
        raise ValueError("bitmap too short")
    out = np.empty((rows, cols), dtype=_elem_dtype(eb))
    # Alg. 2 reads v[k] for k < popcount(b); refuse a v that is too short
    # before the C loop could read past it.
    need = int(row_offsets(rows, cols, bitmap)[-1])
    if values.size < need:
        raise ValueError("values shorter than the number of 1 bits")
    k = lib.oracle_decompress(eb, rows, cols, _ptr(bitmap), _ptr(values), _ptr(out))
    assert k == need
    return out


def row_offsets(rows: int, cols: int, bitmap: np.ndarray) -> np.ndarray:
    lib = _load()
    bitmap = np.ascontiguousarray(bitmap, dtype=np.uint8)
    out = np.empty(rows + 1, dtype=np.int64)
    lib.oracle_row_offsets(rows, cols, _ptr(bitmap), _ptr(out))
    return out


def tile_offsets(n: int, tile: int, bitmap: np.ndarray) -> np.ndarray:
    lib = _load()
    bitmap = np.ascontiguousarray(bitmap, dtype=np.uint8)
    ntiles = (n + tile - 1) // tile
    out = np.empty(ntiles + 1, dtype=np.int64)
    lib.oracle_tile_offsets(n, tile, _ptr(bitmap), _ptr(out))
    return out


def decompress_selected_rows(cols: int, sel: np.ndarray, row_offs: np.ndarray,
                             bitmap: np.ndarray, values: np.ndarray) -> np.ndarray:
    lib = _load()
    sel = np.ascontiguousarray(sel, dtype=np.int64)
    row_offs = np.ascontiguousarray(row_offs, dtype=np.int64)
    bitmap = np.ascontiguousarray(bitmap, dtype=np.uint8)
    values = np.ascontiguousarray(values)
    eb = values.dtype.itemsize
    out = np.empty((sel.size, cols), dtype=_elem_dtype(eb))
    lib.oracle_decompress_selected_rows(eb, cols, _ptr(sel), sel.size, _ptr(row_offs),
                                        _ptr(bitmap), _ptr(values), _ptr(out))
    return out


def decompress_threaded(rows: int, cols: int, bitmap: np.ndarray, values: np.ndarray,
                        row_offs: np.ndarray, threads: int, out: np.ndarray | None = None) -> np.ndarray:
    """The same Algorithm 2, rows split into `threads` contiguous blocks, one OS
    thread per block, each starting its counter at row_offs[first row of block]
    (the analogue of the multi-core CPU decompression of Section 5.1).  Used only
    to time the oracle on all host cores; the per-block loop is the C oracle's."""
    lib = _load()
    bitmap = np.ascontiguousarray(bitmap, dtype=np.uint8)
    values = np.ascontiguousarray(values)
    eb = values.dtype.itemsize
    if out is None:
        out = np.empty((rows, cols), dtype=_elem_dtype(eb))
    threads = max(1, min(threads, rows))
    bounds = [rows * t // threads for t in range(threads + 1)]

    def work(t):
        r0, r1 = bounds[t], bounds[t + 1]
        return lib.oracle_decompress_rows(eb, cols, r0, r1, int(row_offs[r0]),
                                          _ptr(bitmap), _ptr(values), _ptr(out))

    with ThreadPoolExecutor(max_workers=threads) as ex:
        ends = list(ex.map(work, range(threads)))
    for t in range(threads):
        assert ends[t] == int(row_offs[bounds[t + 1]])
    return out


def half_to_double(h: np.ndarray) -> np.ndarray:
    lib = _load()
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float64)
    lib.oracle_half_to_double_array(_ptr(h), h.size, _ptr(out))
    return out


def gemv_f16(rows: int, cols: int, bitmap: np.ndarray, values: np.ndarray, x: np.ndarray) -> np.ndarray:
    """y = W x in double, W the Algorithm-2 output of (bitmap, values), x fp16 patterns."""
    lib = _load()
    bitmap = np.ascontiguousarray(bitmap, dtype=np.uint8)
    values = np.ascontiguousarray(values, dtype=np.uint16)
    x = np.ascontiguousarray(x).view(np.uint16)
    if x.size != cols or bitmap.size < bitmap_bytes(rows, cols):
        raise ValueError("bad sizes")
    if values.size < int(row_offsets(rows, cols, bitmap)[-1]):
        raise ValueError("values shorter than the number of 1 bits")
    y = np.empty(rows, dtype=np.float64)
    lib.oracle_gemv_f16(rows, cols, _ptr(bitmap), _ptr(values), _ptr(x), _ptr(y))
    return y


def gemm_f16(rows: int, cols: int, bitmap: np.ndarray, values: np.ndarray, X: np.ndarray,
             threads: int = 1) -> np.ndarray:
    """Y[b][i] = sum_j W[i][j] X[b][j] in double: W is first decompressed with Algorithm 2
    (decompress above), then the C triple loop runs on the dense matrix.  X: (nb, cols) fp16
    patterns.  `threads` > 1 only splits the rows into blocks, one OS thread each."""
    lib = _load()
    X = np.ascontiguousarray(X).view(np.uint16)
    if X.ndim != 2 or X.shape[1] != cols:
        raise ValueError("X must be (nb, cols)")
    nb = X.shape[0]
    dense = decompress(rows, cols, bitmap, np.ascontiguousarray(values, dtype=np.uint16))
    y = np.empty((nb, rows), dtype=np.float64)
    threads = max(1, min(threads, rows))
    bounds = [rows * t // threads for t in range(threads + 1)]

    def work(t):
        lib.oracle_gemm_f16_rows(rows, cols, bounds[t], bounds[t + 1], _ptr(dense), _ptr(X), nb, _ptr(y))

    if threads == 1:
        work(0)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(threads)))
    return y
