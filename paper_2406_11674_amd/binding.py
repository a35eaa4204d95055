"""Thin ctypes binding over the C-ABI library of include/endor.h.

Argument marshalling only: every step of the path (Algorithm 1 on the host,
Algorithm 2 and its offset table on the GPU; Section 4.1) runs inside
libendor.so.  torch is used for device memory and streams and nothing else.
There is no fallback: if the library has not been built, every call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

__all__ = [
    "EndorError", "Compressed", "DeviceMatrix", "lib", "library_path", "TILE_ELEMS", "MAX_BATCH",
    "bitmap_bytes", "workspace_bytes", "batch_workspace_bytes", "compress", "to_device",
    "build_offsets", "build_offsets_host", "decompress", "decompress_with_offsets",
    "decompress_batch", "decompress_batch_static", "build_offsets_batch", "decompress_batch_with_offsets",
    "decompress_rows", "decompress_cols", "compress_device", "gemv_f16", "HostBlob", "pin", "row_blocks", "stage_bytes", "h2d_decompress_pipeline",
]

TILE_ELEMS = 4096
MAX_BATCH = 16
STATIC_SCRATCH_BYTES = 4 << 20
_HERE = os.path.dirname(os.path.abspath(__file__))
# ENDOR_LIBRARY points at another build of the same library (kernel tuning experiments)
_LIB_PATH = os.environ.get("ENDOR_LIBRARY") or os.path.join(_HERE, "libendor.so")
_lib = None

_i64 = ctypes.c_int64
_p = ctypes.c_void_p
_sz = ctypes.c_size_t


class EndorError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = lib().endor_status_string(status).decode()
        super().__init__(f"{where}: {name} (status {status})")


class _Matrix(ctypes.Structure):
    _fields_ = [("rows", _i64), ("cols", _i64), ("d_bitmap", _p), ("d_values", _p),
                ("nnz", _i64), ("d_dense", _p)]


def library_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2406_11674_amd.build` "
                "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(_LIB_PATH)
        L.endor_status_string.restype = ctypes.c_char_p
        L.endor_status_string.argtypes = [ctypes.c_int]
        L.endor_bitmap_bytes.restype = _sz
        L.endor_bitmap_bytes.argtypes = [_i64, _i64]
        L.endor_workspace_bytes.restype = _sz
        L.endor_workspace_bytes.argtypes = [_i64, _i64]
        L.endor_batch_workspace_bytes.restype = _sz
        L.endor_batch_workspace_bytes.argtypes = [_p, ctypes.c_int]
        for name in ("endor_compress", "endor_compress_u8"):
            f = getattr(L, name)
            f.restype = ctypes.c_int
            f.argtypes = [_p, _i64, _i64, _p, _p, _i64, _p, _p]
        L.endor_build_offsets_host.restype = ctypes.c_int
        L.endor_build_offsets_host.argtypes = [_i64, _i64, _p, _p, _sz]
        L.endor_build_offsets.restype = ctypes.c_int
        L.endor_build_offsets.argtypes = [_i64, _i64, _p, _p, _sz, _p, _p]
        for name in ("endor_decompress", "endor_decompress_with_offsets",
                     "endor_decompress_u8", "endor_decompress_u8_with_offsets"):
            f = getattr(L, name)
            f.restype = ctypes.c_int
            f.argtypes = [_i64, _i64, _p, _p, _i64, _p, _sz, _p, _p]
        for name in ("endor_decompress_batch", "endor_build_offsets_batch",
                     "endor_decompress_batch_with_offsets", "endor_decompress_batch_u8",
                     "endor_decompress_batch_u8_with_offsets"):
            f = getattr(L, name)
            f.restype = ctypes.c_int
            f.argtypes = [_p, ctypes.c_int, _p, _sz, _p]
        for name in ("endor_decompress_rows", "endor_decompress_rows_u8",
                     "endor_decompress_cols", "endor_decompress_cols_u8"):
            f = getattr(L, name)
            f.restype = ctypes.c_int
            f.argtypes = [_i64, _i64, _p, _p, _i64, _p, _p, _i64, _p, _p]
        for name in ("endor_compress_device", "endor_compress_device_u8"):
            f = getattr(L, name)
            f.restype = ctypes.c_int
            f.argtypes = [_i64, _i64, _p, _p, _p, _i64, _p, _sz, _p, _p, _p]
        L.endor_decompress_batch_static.restype = ctypes.c_int
        L.endor_decompress_batch_static.argtypes = [_p, ctypes.c_int, _p]
        L.endor_gemv_f16.restype = ctypes.c_int
        L.endor_gemv_f16.argtypes = [_i64, _i64, _p, _p, _i64, _p, _p, _p, _p]
        L.endor_stage_bytes.restype = _sz
        L.endor_stage_bytes.argtypes = [_i64, _i64, _i64]
        L.endor_h2d_decompress_pipeline.restype = ctypes.c_int
        L.endor_h2d_decompress_pipeline.argtypes = [_p, ctypes.c_int, _p, _sz, _p, _sz, _p, _p]
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != 0:
        raise EndorError(status, where)


def bitmap_bytes(rows: int, cols: int) -> int:
    return int(lib().endor_bitmap_bytes(rows, cols))


def workspace_bytes(rows: int, cols: int) -> int:
    return int(lib().endor_workspace_bytes(rows, cols))


# ------------------------------------------------------------------ host: compression

@dataclass
class Compressed:
    """One matrix in the bitmap format, in host memory."""
    rows: int
    cols: int
    bitmap: np.ndarray       # uint8[bitmap_bytes(rows, cols)]
    values: np.ndarray       # uint16[nnz], or uint8[nnz] for the 8-bit variant
    row_offsets: np.ndarray  # int64[rows + 1]

    @property
    def nnz(self) -> int:
        return int(self.values.size)


def compress(dense: np.ndarray, want_row_offsets: bool = True) -> Compressed:
    """endor_compress / endor_compress_u8 on a 2-d array of 16-bit (float16 / int16 /
    uint16) or 8-bit (int8 / uint8) elements."""
    if dense.ndim != 2 or dense.dtype.itemsize not in (1, 2):
        raise ValueError("dense must be a 2-d array of 8- or 16-bit elements")
    wide = dense.dtype.itemsize == 2
    W = np.ascontiguousarray(dense).view(np.uint16 if wide else np.uint8)
    rows, cols = W.shape
    L = lib()
    fn = L.endor_compress if wide else L.endor_compress_u8
    bitmap = np.empty(bitmap_bytes(rows, cols), dtype=np.uint8)
    row_offsets = np.empty(rows + 1, dtype=np.int64) if want_row_offsets else None
    nnz = _i64(0)
    ro = row_offsets.ctypes.data if want_row_offsets else None
    # counting pass, then the packing pass into an exactly sized buffer
    _check(fn(W.ctypes.data, rows, cols, bitmap.ctypes.data, None, 0, ro, ctypes.byref(nnz)),
           "endor_compress(count)")
    values = np.empty(nnz.value, dtype=W.dtype)
    _check(fn(W.ctypes.data, rows, cols, bitmap.ctypes.data, values.ctypes.data, values.size, ro,
              ctypes.byref(nnz)), "endor_compress")
    return Compressed(rows, cols, bitmap, values, row_offsets)


def build_offsets_host(c: Compressed) -> np.ndarray:
    """endor_build_offsets_host: the tile offset table as a host byte array, ready to be
    copied to the device and passed as `workspace` to the *_with_offsets calls."""
    ws = np.zeros(max(workspace_bytes(c.rows, c.cols), 256), dtype=np.uint8)
    _check(lib().endor_build_offsets_host(c.rows, c.cols, c.bitmap.ctypes.data, ws.ctypes.data, ws.size),
           "endor_build_offsets_host")
    return ws


# ------------------------------------------------------------------ device side

def _torch():
    import torch
    return torch


def _stream_handle(stream) -> int:
    torch = _torch()
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


@dataclass
class DeviceMatrix:
    """One compressed matrix resident in device memory (torch tensors own the memory)."""
    rows: int
    cols: int
    bitmap: object   # torch.uint8[bitmap_bytes]
    values: object   # torch.int16[nnz] (16-bit elements) or torch.uint8[nnz] (8-bit)
    nnz: int

    @property
    def elem_bytes(self) -> int:
        return int(self.values.element_size())


def to_device(c: Compressed, device="cuda") -> DeviceMatrix:
    torch = _torch()
    bm = torch.from_numpy(c.bitmap).to(device)
    vals = torch.from_numpy(c.values.view(np.int16 if c.values.dtype.itemsize == 2 else np.uint8)).to(device)
    return DeviceMatrix(c.rows, c.cols, bm, vals, c.nnz)


def _new_workspace(nbytes: int, device):
    torch = _torch()
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _new_dense(rows, cols, device, elem_bytes=2):
    torch = _torch()
    return torch.empty((rows, cols), dtype=torch.int16 if elem_bytes == 2 else torch.uint8, device=device)


def build_offsets(m: DeviceMatrix, workspace=None, row_offsets: bool = False, stream=None):
    """endor_build_offsets.  Returns (workspace, row_offsets tensor or None)."""
    torch = _torch()
    if workspace is None:
        workspace = _new_workspace(workspace_bytes(m.rows, m.cols), m.bitmap.device)
    ro = torch.empty(m.rows + 1, dtype=torch.int64, device=m.bitmap.device) if row_offsets else None
    _check(lib().endor_build_offsets(m.rows, m.cols, _dptr(m.bitmap), _dptr(workspace),
                                     workspace.numel(), _dptr(ro), _stream_handle(stream)),
           "endor_build_offsets")
    return workspace, ro


def decompress(m: DeviceMatrix, out=None, workspace=None, stream=None):
    """endor_decompress.  `out`: any 2-byte-element tensor of rows*cols elements."""
    if out is None:
        out = _new_dense(m.rows, m.cols, m.bitmap.device, m.elem_bytes)
    if workspace is None:
        workspace = _new_workspace(workspace_bytes(m.rows, m.cols), m.bitmap.device)
    if out.element_size() != m.elem_bytes:
        raise ValueError("output element width differs from the values'")
    fn = lib().endor_decompress if m.elem_bytes == 2 else lib().endor_decompress_u8
    _check(fn(m.rows, m.cols, _dptr(m.bitmap), _dptr(m.values), m.nnz, _dptr(workspace),
              workspace.numel(), _dptr(out), _stream_handle(stream)), "endor_decompress")
    return out


def decompress_with_offsets(m: DeviceMatrix, workspace, out=None, stream=None):
    if out is None:
        out = _new_dense(m.rows, m.cols, m.bitmap.device, m.elem_bytes)
    if out.element_size() != m.elem_bytes:
        raise ValueError("output element width differs from the values'")
    fn = lib().endor_decompress_with_offsets if m.elem_bytes == 2 else lib().endor_decompress_u8_with_offsets
    _check(fn(m.rows, m.cols, _dptr(m.bitmap), _dptr(m.values), m.nnz, _dptr(workspace),
              workspace.numel(), _dptr(out), _stream_handle(stream)), "endor_decompress_with_offsets")
    return out


def _descs(mats, outs):
    arr = (_Matrix * len(mats))()
    for i, m in enumerate(mats):
        arr[i].rows, arr[i].cols = m.rows, m.cols
        arr[i].d_bitmap = _dptr(m.bitmap)
        arr[i].d_values = _dptr(m.values)
        arr[i].nnz = m.nnz
        arr[i].d_dense = _dptr(outs[i]) if outs is not None else 0
    return arr


def batch_workspace_bytes(mats) -> int:
    arr = _descs(mats, None)
    return int(lib().endor_batch_workspace_bytes(ctypes.addressof(arr), len(mats)))


def _batch(fn_name, mats, outs, workspace, stream):
    arr = _descs(mats, outs)
    _check(getattr(lib(), fn_name)(ctypes.addressof(arr), len(mats), _dptr(workspace),
                                   0 if workspace is None else workspace.numel(),
                                   _stream_handle(stream)), fn_name)


def decompress_batch(mats, outs=None, workspace=None, stream=None):
    """endor_decompress_batch over a list of DeviceMatrix.  Returns (outs, workspace)."""
    if not mats:
        return [], workspace
    dev = mats[0].bitmap.device
    eb = mats[0].elem_bytes
    if any(m.elem_bytes != eb for m in mats):
        raise ValueError("one batch holds one element width")
    if outs is None:
        outs = [_new_dense(m.rows, m.cols, dev, eb) for m in mats]
    if workspace is None:
        workspace = _new_workspace(batch_workspace_bytes(mats), dev)
    _batch("endor_decompress_batch" if eb == 2 else "endor_decompress_batch_u8", mats, outs, workspace, stream)
    return outs, workspace


def decompress_batch_static(mats, outs, stream=None):
    """endor_decompress_batch_static: the batch call that takes no workspace and allocates
    nothing (its tables live in a fixed device array inside the library).  `outs` is required."""
    if not mats:
        return outs
    eb = mats[0].elem_bytes
    if eb != 2 or any(m.elem_bytes != eb for m in mats):
        raise ValueError("decompress_batch_static takes 16-bit values")
    if len(outs) != len(mats):
        raise ValueError("one output per matrix")
    arr = _descs(mats, outs)
    _check(lib().endor_decompress_batch_static(ctypes.addressof(arr), len(mats), _stream_handle(stream)),
           "endor_decompress_batch_static")
    return outs


def build_offsets_batch(mats, workspace=None, stream=None):
    if workspace is None:
        workspace = _new_workspace(batch_workspace_bytes(mats), mats[0].bitmap.device)
    _batch("endor_build_offsets_batch", mats, None, workspace, stream)
    return workspace


def decompress_batch_with_offsets(mats, workspace, outs=None, stream=None):
    eb = mats[0].elem_bytes
    if any(m.elem_bytes != eb for m in mats):
        raise ValueError("one batch holds one element width")
    if outs is None:
        outs = [_new_dense(m.rows, m.cols, mats[0].bitmap.device, eb) for m in mats]
    _batch("endor_decompress_batch_with_offsets" if eb == 2 else "endor_decompress_batch_u8_with_offsets",
           mats, outs, workspace, stream)
    return outs


def decompress_rows(m: DeviceMatrix, row_offsets, sel, out=None, stream=None):
    """endor_decompress_rows[_u8]: out[r] = row sel[r].  row_offsets, sel: int64 device tensors."""
    torch = _torch()
    if row_offsets.dtype != torch.int64 or sel.dtype != torch.int64:
        raise ValueError("row_offsets and sel must be int64 tensors")
    nsel = int(sel.numel())
    if out is None:
        out = _new_dense(nsel, m.cols, m.bitmap.device, m.elem_bytes)
    fn = lib().endor_decompress_rows if m.elem_bytes == 2 else lib().endor_decompress_rows_u8
    _check(fn(m.rows, m.cols, _dptr(m.bitmap), _dptr(m.values), m.nnz, _dptr(row_offsets), _dptr(sel),
              nsel, _dptr(out), _stream_handle(stream)), "endor_decompress_rows")
    return out


def decompress_cols(m: DeviceMatrix, row_offsets, sel, out=None, stream=None):
    """endor_decompress_cols[_u8]: out[i][q] = W[i][sel[q]].  row_offsets, sel: int64 device tensors."""
    torch = _torch()
    if row_offsets.dtype != torch.int64 or sel.dtype != torch.int64:
        raise ValueError("row_offsets and sel must be int64 tensors")
    nsel = int(sel.numel())
    if out is None:
        out = _new_dense(m.rows, nsel, m.bitmap.device, m.elem_bytes)
    fn = lib().endor_decompress_cols if m.elem_bytes == 2 else lib().endor_decompress_cols_u8
    _check(fn(m.rows, m.cols, _dptr(m.bitmap), _dptr(m.values), m.nnz, _dptr(row_offsets), _dptr(sel),
              nsel, _dptr(out), _stream_handle(stream)), "endor_decompress_cols")
    return out


def compress_device(dense, values=None, row_offsets: bool = False, stream=None):
    """endor_compress_device[_u8] on a 2-d device tensor of 2- or 1-byte elements.
    Returns (DeviceMatrix, workspace, row_offsets or None).  `values`: preallocated
    buffer (its length is the capacity); default rows*cols elements.  Synchronises once
    to read the number of non-zeros back."""
    torch = _torch()
    rows, cols = dense.shape
    eb = dense.element_size()
    if eb not in (1, 2) or not dense.is_contiguous():
        raise ValueError("dense must be a contiguous 2-d tensor of 1- or 2-byte elements")
    dev = dense.device
    bitmap = torch.empty(bitmap_bytes(rows, cols), dtype=torch.uint8, device=dev)
    if values is None:
        values = torch.empty(rows * cols, dtype=torch.int16 if eb == 2 else torch.uint8, device=dev)
    ws = _new_workspace(workspace_bytes(rows, cols), dev)
    ro = torch.empty(rows + 1, dtype=torch.int64, device=dev) if row_offsets else None
    nnz = torch.zeros(1, dtype=torch.int64, device=dev)
    fn = lib().endor_compress_device if eb == 2 else lib().endor_compress_device_u8
    _check(fn(rows, cols, _dptr(dense), _dptr(bitmap), _dptr(values), values.numel(), _dptr(ws), ws.numel(),
              _dptr(ro), _dptr(nnz), _stream_handle(stream)), "endor_compress_device")
    n = int(nnz.item())
    if n > values.numel():
        raise EndorError(2, f"endor_compress_device: {n} non-zeros, capacity {values.numel()}")
    return DeviceMatrix(rows, cols, bitmap, values[:n], n), ws, ro


def gemv_f16(m: DeviceMatrix, row_offsets, x, y=None, stream=None):
    """endor_gemv_f16: y (fp32, rows) = W x with W in compressed form, x fp16 (cols)."""
    torch = _torch()
    if m.elem_bytes != 2 or x.element_size() != 2 or x.numel() != m.cols:
        raise ValueError("gemv_f16 needs 16-bit values and an fp16 x of length cols")
    if y is None:
        y = torch.empty(m.rows, dtype=torch.float32, device=m.bitmap.device)
    _check(lib().endor_gemv_f16(m.rows, m.cols, _dptr(m.bitmap), _dptr(m.values), m.nnz, _dptr(row_offsets),
                                _dptr(x), _dptr(y), _stream_handle(stream)), "endor_gemv_f16")
    return y


# ------------------------------------------------------------------ host -> device pipeline

class _HostBlob(ctypes.Structure):
    _fields_ = [("rows", _i64), ("cols", _i64), ("h_bitmap", _p), ("h_values", _p),
                ("nnz", _i64), ("d_dense", _p)]


@dataclass
class HostBlob:
    """A compressed matrix, or a block of whole rows of one, in (pinned) host tensors."""
    rows: int
    cols: int
    bitmap: object      # torch.uint8, host
    values: object      # torch.int16, host
    nnz: int
    row_begin: int = 0  # first row of the block inside its matrix


def stage_bytes(rows: int, cols: int, nnz: int) -> int:
    return int(lib().endor_stage_bytes(rows, cols, nnz))


def pin(c: Compressed):
    """Copy a Compressed into pinned host tensors (allocated pinned, not registered)."""
    torch = _torch()
    bm = torch.empty(c.bitmap.size, dtype=torch.uint8, pin_memory=True)
    bm.numpy()[:] = c.bitmap
    if c.values.dtype.itemsize != 2:
        raise ValueError("the host-to-device pipeline takes 16-bit values")
    vals = torch.empty(c.values.size, dtype=torch.int16, pin_memory=True)
    vals.numpy()[:] = c.values.view(np.int16)
    return bm, vals


def row_blocks(c: Compressed, pinned, nblocks: int):
    """Split one matrix into up to `nblocks` HostBlobs of whole rows.  Block starts are
    rounded so that r0*cols is a multiple of 64 (a bitmap word boundary); the block's
    values start at row_offsets[r0]."""
    bm, vals = pinned
    if c.row_offsets is None:
        raise ValueError("row_blocks needs the compressor's row offsets")
    rows, cols = c.rows, c.cols
    step = 64 // int(np.gcd(cols, 64)) if cols else 1   # smallest r with r*cols % 64 == 0
    cuts = sorted({min(rows, (rows * i // nblocks) // step * step) for i in range(nblocks)} | {rows})
    if cuts[0] != 0:
        cuts.insert(0, 0)
    out = []
    for r0, r1 in zip(cuts[:-1], cuts[1:]):
        if r1 <= r0:
            continue
        k0, k1 = int(c.row_offsets[r0]), int(c.row_offsets[r1])
        out.append(HostBlob(r1 - r0, cols, bm[r0 * cols // 8:], vals[k0:k1], k1 - k0, r0))
    return out


def h2d_decompress_pipeline(blobs, outs, stages, workspaces, copy_stream, compute_stream):
    """endor_h2d_decompress_pipeline.  `outs[k]`: device tensor (or view) that receives blob k."""
    arr = (_HostBlob * len(blobs))()
    for i, b in enumerate(blobs):
        arr[i].rows, arr[i].cols, arr[i].nnz = b.rows, b.cols, b.nnz
        arr[i].h_bitmap = _dptr(b.bitmap)
        arr[i].h_values = _dptr(b.values)
        arr[i].d_dense = _dptr(outs[i])
    st = (_p * 2)(_dptr(stages[0]), _dptr(stages[1]))
    ws = (_p * 2)(_dptr(workspaces[0]), _dptr(workspaces[1]))
    _check(lib().endor_h2d_decompress_pipeline(
        ctypes.addressof(arr), len(blobs), ctypes.addressof(st), min(s.numel() for s in stages),
        ctypes.addressof(ws), min(w.numel() for w in workspaces),
        int(copy_stream.cuda_stream), int(compute_stream.cuda_stream)), "endor_h2d_decompress_pipeline")
