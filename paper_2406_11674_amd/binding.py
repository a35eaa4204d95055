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
    "decompress_rows", "decompress_cols", "compress_device", "gemv_f16", "gemm_f16", "gemm_scratch_bytes", "HostBlob", "pin", "row_blocks", "row_block_cuts", "stage_bytes", "Pipeline", "PIPELINE_SLOTS", "check_batch",
]

TILE_ELEMS = 4096
MAX_BATCH = 16
STATIC_SCRATCH_BYTES = 4 << 20
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libendor.so")
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
        L.endor_gemm_scratch_bytes.restype = _sz
        L.endor_gemm_scratch_bytes.argtypes = [_i64, _i64, ctypes.c_int]
        L.endor_gemm_f16.restype = ctypes.c_int
        L.endor_gemm_f16.argtypes = [_i64, _i64, _p, _p, _i64, _p, _sz, _p, _i64, ctypes.c_int, _p, _p, _sz, _p]
        L.endor_stage_bytes.restype = _sz
        L.endor_stage_bytes.argtypes = [_i64, _i64, _i64, ctypes.c_int]
        L.endor_row_block_cuts.restype = ctypes.c_int
        L.endor_row_block_cuts.argtypes = [_i64, _i64, ctypes.c_int, _p]
        L.endor_row_block.restype = ctypes.c_int
        L.endor_row_block.argtypes = [_i64, _i64, ctypes.c_int, _p, _p, _p, _i64, _i64, _p, _p]
        L.endor_pipeline_init.restype = ctypes.c_int
        L.endor_pipeline_init.argtypes = [_p, _p, _sz, _p, _sz, _p, _p, _p]
        L.endor_pipeline_destroy.restype = ctypes.c_int
        L.endor_pipeline_destroy.argtypes = [_p]
        L.endor_h2d_decompress_pipeline.restype = ctypes.c_int
        L.endor_h2d_decompress_pipeline.argtypes = [_p, _p, ctypes.c_int]
        L.endor_check_batch.restype = ctypes.c_int
        L.endor_check_batch.argtypes = [_p, ctypes.c_int, _p, _sz, _p, _p]
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
    if out.element_size() != m.elem_bytes or out.numel() != m.rows * m.cols:
        raise ValueError("output must hold rows*cols elements of the values' width")
    fn = lib().endor_decompress if m.elem_bytes == 2 else lib().endor_decompress_u8
    _check(fn(m.rows, m.cols, _dptr(m.bitmap), _dptr(m.values), m.nnz, _dptr(workspace),
              workspace.numel(), _dptr(out), _stream_handle(stream)), "endor_decompress")
    return out


def decompress_with_offsets(m: DeviceMatrix, workspace, out=None, stream=None):
    if out is None:
        out = _new_dense(m.rows, m.cols, m.bitmap.device, m.elem_bytes)
    if out.element_size() != m.elem_bytes or out.numel() != m.rows * m.cols:
        raise ValueError("output must hold rows*cols elements of the values' width")
    fn = lib().endor_decompress_with_offsets if m.elem_bytes == 2 else lib().endor_decompress_u8_with_offsets
    _check(fn(m.rows, m.cols, _dptr(m.bitmap), _dptr(m.values), m.nnz, _dptr(workspace),
              workspace.numel(), _dptr(out), _stream_handle(stream)), "endor_decompress_with_offsets")
    return out


def _descs(mats, outs):
    arr = (_Matrix * len(mats))()
    for i, m in enumerate(mats):
        if outs is not None and (outs[i].numel() != m.rows * m.cols or outs[i].element_size() != m.elem_bytes):
            raise ValueError("output %d does not have rows*cols elements of the values' width" % i)
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


def check_batch(mats, workspace, status=None, stream=None):
    """endor_check_batch: status[i] = 0 if matrix i's nnz equals the number of 1 bits its table
    records, else ENDOR_ERR_NNZ_MISMATCH (6).  Device int32 tensor; no synchronisation."""
    torch = _torch()
    if status is None:
        status = torch.full((len(mats),), -1, dtype=torch.int32, device=mats[0].bitmap.device)
    arr = _descs(mats, None)
    _check(lib().endor_check_batch(ctypes.addressof(arr), len(mats), _dptr(workspace), workspace.numel(),
                                   _dptr(status), _stream_handle(stream)), "endor_check_batch")
    return status


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


def gemm_scratch_bytes(rows: int, cols: int, nb: int) -> int:
    return int(lib().endor_gemm_scratch_bytes(rows, cols, nb))


def gemm_f16(m: DeviceMatrix, workspace, X, Y=None, scratch=None, stream=None):
    """endor_gemm_f16: Y (fp32, nb x rows) = X W^T with W in compressed form; X: (nb, cols) fp16
    device tensor (row stride = ldx), workspace: the matrix's tile offset table."""
    torch = _torch()
    if m.elem_bytes != 2 or X.element_size() != 2 or X.dim() != 2 or X.shape[1] != m.cols or X.stride(1) != 1:
        raise ValueError("gemm_f16 needs 16-bit values and an fp16 X of shape (nb, cols)")
    nb = int(X.shape[0])
    if Y is None:
        Y = torch.empty((nb, m.rows), dtype=torch.float32, device=m.bitmap.device)
    if Y.dtype != torch.float32 or Y.numel() != nb * m.rows or not Y.is_contiguous():
        raise ValueError("Y must be a contiguous fp32 tensor of nb*rows elements")
    need = gemm_scratch_bytes(m.rows, m.cols, nb) if nb and m.rows and m.cols else 0
    if scratch is None and need:
        scratch = torch.empty(need, dtype=torch.uint8, device=m.bitmap.device)
    _check(lib().endor_gemm_f16(m.rows, m.cols, _dptr(m.bitmap), _dptr(m.values), m.nnz, _dptr(workspace),
                                0 if workspace is None else workspace.numel(), _dptr(X),
                                int(X.stride(0)) if nb > 1 else max(m.cols, int(X.stride(0))), nb, _dptr(Y),
                                _dptr(scratch), 0 if scratch is None else scratch.numel(), _stream_handle(stream)),
           "endor_gemm_f16")
    return Y


# ------------------------------------------------------------------ host -> device pipeline

PIPELINE_SLOTS = 3


class _HostBlob(ctypes.Structure):
    _fields_ = [("rows", _i64), ("cols", _i64), ("h_bitmap", _p), ("h_values", _p),
                ("nnz", _i64), ("d_dense", _p), ("elem_bytes", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class _Pipeline(ctypes.Structure):
    _fields_ = [("d_stage", _p * PIPELINE_SLOTS), ("d_workspace", _p * PIPELINE_SLOTS),
                ("stage_bytes", _sz), ("workspace_bytes", _sz), ("copy_stream", _p), ("copy_stream2", _p),
                ("compute_stream", _p), ("copied", _p * PIPELINE_SLOTS), ("freed", _p * PIPELINE_SLOTS),
                ("next_slot", ctypes.c_uint32), ("slots_used", ctypes.c_uint32), ("blobs_done", ctypes.c_uint64)]


@dataclass
class HostBlob:
    """A compressed matrix, or a block of whole rows of one, inside a pinned host buffer."""
    rows: int
    cols: int
    nnz: int
    elem_bytes: int
    bitmap_ptr: int     # host address of the block's bitmap
    values_ptr: int     # host address of the block's values
    row_begin: int = 0  # first row of the block inside its matrix
    keep: object = None  # the pinned tensor(s) that own the memory


def stage_bytes(rows: int, cols: int, nnz: int, elem_bytes: int = 2) -> int:
    return int(lib().endor_stage_bytes(rows, cols, nnz, elem_bytes))


def _align256(x: int) -> int:
    return (x + 255) & ~255


def pin(c: Compressed, pinned: bool = True):
    """Copy a Compressed into ONE pinned host tensor (allocated pinned, not registered), the
    values starting at the next multiple of 256 bytes after the bitmap, so that the pipeline
    moves the blob in a single copy.  Returns a HostBlob.  pinned=False: ordinary host memory
    (for use without a GPU)."""
    torch = _torch()
    eb = c.values.dtype.itemsize
    bm_bytes = c.bitmap.size
    buf = torch.empty(_align256(bm_bytes) + eb * c.values.size, dtype=torch.uint8, pin_memory=pinned)
    flat = buf.numpy()
    flat[:bm_bytes] = c.bitmap
    flat[_align256(bm_bytes):] = c.values.view(np.uint8)
    base = int(buf.data_ptr())
    return HostBlob(c.rows, c.cols, c.nnz, eb, base, base + _align256(bm_bytes), 0, buf)


def row_block_cuts(rows: int, cols: int, nblocks: int):
    """endor_row_block_cuts: nblocks + 1 row indices at bitmap word boundaries."""
    cuts = (_i64 * (nblocks + 1))()
    _check(lib().endor_row_block_cuts(rows, cols, nblocks, cuts), "endor_row_block_cuts")
    return list(cuts)


def row_blocks(c: Compressed, nblocks: int, pinned: bool = True):
    """Split one matrix into HostBlobs of whole rows (endor_row_block_cuts / endor_row_block
    decide where a block's bitmap and values start); each block is copied into a pinned
    tensor of its own, bitmap and values adjacent as in pin()."""
    torch = _torch()
    if c.row_offsets is None:
        raise ValueError("row_blocks needs the compressor's row offsets")
    eb = c.values.dtype.itemsize
    bm8 = np.ascontiguousarray(c.bitmap)
    v8 = np.ascontiguousarray(c.values).view(np.uint8)
    ro = np.ascontiguousarray(c.row_offsets, dtype=np.int64)
    cuts = row_block_cuts(c.rows, c.cols, nblocks)
    out = []
    for r0, r1 in zip(cuts[:-1], cuts[1:]):
        if r1 <= r0:
            continue
        blob = _HostBlob()
        _check(lib().endor_row_block(c.rows, c.cols, eb, bm8.ctypes.data, v8.ctypes.data, ro.ctypes.data,
                                     r0, r1, None, ctypes.byref(blob)), "endor_row_block")
        bm_bytes = bitmap_bytes(blob.rows, blob.cols)
        b_off = blob.h_bitmap - bm8.ctypes.data
        v_off = (blob.h_values or v8.ctypes.data) - v8.ctypes.data
        buf = torch.empty(_align256(bm_bytes) + eb * blob.nnz, dtype=torch.uint8, pin_memory=pinned)
        flat = buf.numpy()
        flat[:bm_bytes] = bm8[b_off:b_off + bm_bytes]
        flat[_align256(bm_bytes):] = v8[v_off:v_off + eb * blob.nnz]
        base = int(buf.data_ptr())
        out.append(HostBlob(blob.rows, blob.cols, blob.nnz, eb, base, base + _align256(bm_bytes), r0, buf))
    return out


class Pipeline:
    """endor_pipeline: three staging slots and workspaces (torch tensors own the memory), two
    torch streams, events created by endor_pipeline_init and destroyed with the object."""

    def __init__(self, stage_bytes_: int, workspace_bytes_: int, copy_stream, compute_stream, device="cuda",
                 copy_stream2=None):
        torch = _torch()
        self.stages = [torch.empty(max(256, stage_bytes_), dtype=torch.uint8, device=device)
                       for _ in range(PIPELINE_SLOTS)]
        self.workspaces = [torch.empty(max(256, workspace_bytes_), dtype=torch.uint8, device=device)
                           for _ in range(PIPELINE_SLOTS)]
        self.copy_stream, self.copy_stream2, self.compute_stream = copy_stream, copy_stream2, compute_stream
        self._p = _Pipeline()
        st = (_p * PIPELINE_SLOTS)(*[_dptr(t) for t in self.stages])
        ws = (_p * PIPELINE_SLOTS)(*[_dptr(t) for t in self.workspaces])
        _check(lib().endor_pipeline_init(ctypes.byref(self._p), st, self.stages[0].numel(), ws,
                                         self.workspaces[0].numel(), int(copy_stream.cuda_stream),
                                         int(copy_stream2.cuda_stream) if copy_stream2 is not None else None,
                                         int(compute_stream.cuda_stream)), "endor_pipeline_init")
        self._live = True

    @classmethod
    def for_blobs(cls, blobs, copy_stream, compute_stream, device="cuda", copy_stream2=None):
        sb = max(stage_bytes(b.rows, b.cols, b.nnz, b.elem_bytes) for b in blobs)
        wb = max(workspace_bytes(b.rows, b.cols) for b in blobs)
        return cls(sb, wb, copy_stream, compute_stream, device, copy_stream2)

    def run(self, blobs, outs):
        """endor_h2d_decompress_pipeline.  `outs[k]`: device tensor (or view) that receives blob k."""
        arr = (_HostBlob * len(blobs))()
        for i, b in enumerate(blobs):
            if outs[i].numel() != b.rows * b.cols or outs[i].element_size() != b.elem_bytes:
                raise ValueError("output %d does not match its blob" % i)
            arr[i].rows, arr[i].cols, arr[i].nnz = b.rows, b.cols, b.nnz
            arr[i].h_bitmap, arr[i].h_values = b.bitmap_ptr, b.values_ptr
            arr[i].d_dense = _dptr(outs[i])
            arr[i].elem_bytes, arr[i].reserved = b.elem_bytes, 0
        _check(lib().endor_h2d_decompress_pipeline(ctypes.byref(self._p), arr, len(blobs)),
               "endor_h2d_decompress_pipeline")

    def close(self):
        if self._live:
            self._live = False
            _check(lib().endor_pipeline_destroy(ctypes.byref(self._p)), "endor_pipeline_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
