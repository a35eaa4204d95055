"""The C-ABI library loads without a GPU, exports every symbol include/endor.h
declares, and rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2406_11674_amd as endor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "endor.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(endor_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared_functions()
    assert "endor_compress" in names and "endor_decompress" in names and len(names) >= 10
    L = endor.lib()
    for n in names:
        assert hasattr(L, n), n


def test_size_helpers():
    assert endor.bitmap_bytes(9216, 36864) == 42_467_328          # Section 4.1's bitmap size
    assert endor.bitmap_bytes(3, 5) == 8 and endor.bitmap_bytes(0, 7) == 0
    assert endor.bitmap_bytes(-1, 5) == 0
    assert endor.workspace_bytes(1, 1) % 256 == 0 and endor.workspace_bytes(1, 1) > 0
    assert endor.workspace_bytes(0, 5) == 0
    n_tiles = 8192 * 28672 // 4096
    assert endor.workspace_bytes(8192, 28672) < 5 * n_tiles      # about one word per tile
    assert endor.workspace_bytes(1 << 20, 1 << 20) == 0          # >= 2^34 elements


def test_device_entry_points_reject_bad_arguments_without_launching():
    L = endor.lib()
    ws = 1 << 20
    fake = 0x1000  # never dereferenced: every call below fails validation first
    # NULL bitmap
    assert L.endor_decompress(4, 64, None, fake, 10, fake, ws, fake, None) == 1
    # misaligned bitmap / workspace / dense
    assert L.endor_decompress(4, 64, fake + 4, fake, 10, fake, ws, fake, None) == 1
    assert L.endor_decompress(4, 64, fake, fake, 10, fake + 8, ws, fake, None) == 1
    assert L.endor_decompress(4, 64, fake, fake, 10, fake, ws, fake + 1, None) == 1
    # nnz out of range, NULL values with nnz > 0, NULL dense
    assert L.endor_decompress(4, 64, fake, fake, 4 * 64 + 1, fake, ws, fake, None) == 1
    assert L.endor_decompress(4, 64, fake, None, 10, fake, ws, fake, None) == 1
    assert L.endor_decompress(4, 64, fake, fake, 10, fake, ws, None, None) == 1
    # workspace too small / missing
    assert L.endor_decompress(4, 64, fake, fake, 10, fake, 16, fake, None) == 2
    assert L.endor_decompress(4, 64, fake, fake, 10, None, 0, fake, None) == 1
    # negative and oversized dims
    assert L.endor_decompress(-4, 64, fake, fake, 10, fake, ws, fake, None) == 1
    assert L.endor_decompress(1 << 20, 1 << 20, fake, fake, 10, fake, ws, fake, None) == 3
    assert L.endor_build_offsets(4, 64, None, fake, ws, None, None) == 1
    assert L.endor_build_offsets(4, 64, fake, fake, ws, fake + 4, None) == 1
    assert L.endor_decompress_batch(None, 2, fake, ws, None) == 1
    assert L.endor_decompress_batch(None, -1, fake, ws, None) == 1
    # empty work is accepted and launches nothing
    assert L.endor_decompress(0, 64, None, None, 0, None, 0, None, None) == 0
    assert L.endor_decompress_batch(None, 0, None, 0, None) == 0


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2406_11674_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libendor.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.lib()


def test_header_is_valid_c99_and_cxx17(tmp_path):
    """include/endor.h is a C header: it must compile on its own as C99 and as C++17."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None or shutil.which("g++") is None:
        pytest.skip("needs gcc and g++")
    src_c = tmp_path / "use.c"
    src_c.write_text('#include "endor.h"\nint main(void) { return (int)endor_bitmap_bytes(1, 1) == 8 ? 0 : 1; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, "-c",
                           str(src_c), "-o", str(tmp_path / "use_c.o")])
    src_cpp = tmp_path / "use.cpp"
    src_cpp.write_text(src_c.read_text())
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, "-c",
                           str(src_cpp), "-o", str(tmp_path / "use_cpp.o")])


def test_widened_entry_points_reject_bad_arguments_without_launching():
    L = endor.lib()
    fake, ws = 0x1000, 1 << 20
    # row subset
    assert L.endor_decompress_rows(4, 64, None, fake, 10, fake, fake, 2, fake, None) == 1
    assert L.endor_decompress_rows(4, 64, fake, fake, 10, None, fake, 2, fake, None) == 1
    assert L.endor_decompress_rows(4, 64, fake, fake, 10, fake, None, 2, fake, None) == 1
    assert L.endor_decompress_rows(4, 64, fake, fake, 10, fake, fake, 2, None, None) == 1
    assert L.endor_decompress_rows(4, 64, fake, fake, 10, fake + 4, fake, 2, fake, None) == 1
    assert L.endor_decompress_rows(4, 64, fake, fake, 10, fake, fake, -1, fake, None) == 1
    assert L.endor_decompress_rows(4, 64, fake, fake, 4 * 64 + 1, fake, fake, 2, fake, None) == 1
    assert L.endor_decompress_rows(4, 64, fake, fake, 10, fake, fake, 0, None, None) == 0       # nothing selected
    assert L.endor_decompress_rows_u8(4, 64, fake, fake + 1, 10, fake, fake + 4, 2, fake + 3, None) == 1   # misaligned sel
    # column subset
    assert L.endor_decompress_cols(4, 64, None, fake, 10, fake, fake, 2, fake, None) == 1
    assert L.endor_decompress_cols(4, 64, fake, fake, 10, fake, None, 2, fake, None) == 1
    assert L.endor_decompress_cols(4, 64, fake, fake, 10, fake, fake, 2, None, None) == 1
    assert L.endor_decompress_cols(4, 1 << 20, fake, fake, 10, fake, fake, 2, fake, None) == 3   # row too long for LDS
    assert L.endor_decompress_cols(4, 64, fake, fake, 10, fake, fake, 0, None, None) == 0
    # fused product
    assert L.endor_gemv_f16(4, 64, None, fake, 10, fake, fake, fake, None) == 1
    assert L.endor_gemv_f16(4, 64, fake, fake, 10, None, fake, fake, None) == 1
    assert L.endor_gemv_f16(4, 64, fake, fake, 10, fake, None, fake, None) == 1
    assert L.endor_gemv_f16(4, 64, fake, fake, 10, fake, fake, None, None) == 1
    assert L.endor_gemv_f16(4, 64, fake, fake, 10, fake, fake, fake + 2, None) == 1
    assert L.endor_gemv_f16(0, 64, None, None, 0, None, None, None, None) == 0
    # small-batch product
    assert L.endor_gemm_f16(4, 64, None, fake, 10, fake, ws, fake, 64, 2, fake, None, 0, None) == 1
    assert L.endor_gemm_f16(4, 64, fake, fake, 10, None, ws, fake, 64, 2, fake, None, 0, None) == 1
    assert L.endor_gemm_f16(4, 64, fake, fake, 10, fake, 16, fake, 64, 2, fake, None, 0, None) == 2
    assert L.endor_gemm_f16(4, 64, fake, fake, 10, fake, ws, fake, 63, 2, fake, None, 0, None) == 1     # ldx < cols
    assert L.endor_gemm_f16(4, 64, fake, fake, 10, fake, ws, fake, 64, 17, fake, None, 0, None) == 1    # batch too large
    assert L.endor_gemm_f16(4, 64, fake, fake, 10, fake, ws, fake, 64, 2, None, None, 0, None) == 1
    assert L.endor_gemm_f16(64, 4096, fake, fake, 10, fake, ws, fake, 4096, 2, fake, None, 0, None) == 1  # scratch missing
    assert L.endor_gemm_f16(0, 64, None, None, 0, None, 0, None, 64, 2, None, None, 0, None) == 0
    assert endor.gemm_scratch_bytes(4, 64, 2) == 0 and endor.gemm_scratch_bytes(64, 4096, 2) > 0
    assert endor.gemm_scratch_bytes(64, 4096, 17) == 0
    # device compressor
    assert L.endor_compress_device(4, 64, None, fake, fake, 256, fake, ws, None, fake, None) == 1
    assert L.endor_compress_device(4, 64, fake, None, fake, 256, fake, ws, None, fake, None) == 1
    assert L.endor_compress_device(4, 64, fake, fake, fake, 256, fake, ws, None, None, None) == 1
    assert L.endor_compress_device(4, 64, fake, fake, None, 256, fake, ws, None, fake, None) == 1
    assert L.endor_compress_device(4, 64, fake, fake, fake, 256, fake, 16, None, fake, None) == 2
    assert L.endor_compress_device(4, 64, fake, fake, fake, -1, fake, ws, None, fake, None) == 1
    assert L.endor_compress_device(1 << 20, 1 << 20, fake, fake, fake, 256, fake, ws, None, fake, None) == 3
    # host table builder
    assert L.endor_build_offsets_host(4, 64, None, fake, ws) == 1
    assert L.endor_build_offsets_host(-1, 64, fake, fake, ws) == 1
    assert L.endor_build_offsets_host(0, 64, None, None, 0) == 0
    # pipeline
    assert L.endor_h2d_decompress_pipeline(None, None, 2) == 1
    assert L.endor_pipeline_init(None, None, 0, None, 0, None, None, None) == 1
    assert L.endor_pipeline_destroy(None) == 1
    pipe = (ctypes.c_byte * 256)()      # zeroed: never initialised, so it holds no events
    blob = (ctypes.c_byte * 64)()
    assert L.endor_h2d_decompress_pipeline(pipe, blob, 1) == 1
    assert L.endor_h2d_decompress_pipeline(pipe, None, 0) == 0
    three = (ctypes.c_void_p * 3)(fake, fake + 256, fake + 512)
    same = (ctypes.c_void_p * 3)(fake, fake, fake + 512)
    assert L.endor_pipeline_init(pipe, three, ws, three, ws, fake, None, fake) == 1           # one stream for both
    assert L.endor_pipeline_init(pipe, three, ws, three, ws, fake, fake, fake + 8) == 1       # second copy stream = first
    assert L.endor_pipeline_init(pipe, same, ws, three, ws, fake, None, fake + 8) == 1        # a slot given twice
    assert endor.stage_bytes(4, 64, 10) == 256 + 256 and endor.stage_bytes(4, 64, 257) == 0
    assert endor.stage_bytes(4, 64, 256, 1) == 256 + 256 and endor.stage_bytes(4, 64, 10, 3) == 0
    # check mode
    assert L.endor_check_batch(None, 1, fake, ws, fake, None) == 1
    assert L.endor_check_batch(None, 0, None, 0, None, None) == 0
