"""GPU parity: the HIP decompression path (through the C ABI) against the CPU
oracle, element by element and bit for bit, on the same seeded host buffers.

Integer / byte work throughout, so the bar is exact equality.
"""
import numpy as np
import pytest

import paper_2406_11674_amd as endor
from oracle import endor_oracle as orc
from paper_2406_11674_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

POISON = 0x7FFF  # int16 view of 0x7FFF; never produced by zero fill


def _say(msg):
    print(msg, flush=True)


def _random_compressed(rows, cols, keep, seed, zero_values=True):
    """A compressed matrix built directly in the compressed domain: random bits,
    arbitrary 16-bit patterns as values (the zero pattern included)."""
    n = rows * cols
    g = np.random.default_rng(seed)
    bits = g.random(n) < keep
    bitmap = np.zeros(endor.bitmap_bytes(rows, cols), np.uint8)
    packed = np.packbits(bits, bitorder="little")
    bitmap[: packed.size] = packed
    values = g.integers(0, 1 << 16, size=int(bits.sum()), dtype=np.uint32).astype(np.uint16)
    if zero_values and values.size:
        values[:: 7] = 0
    return endor.Compressed(rows, cols, bitmap, values, None)


def _gpu_decompress(c, poison=True):
    m = endor.to_device(c)
    out = torch.full((c.rows, c.cols), POISON, dtype=torch.int16, device="cuda")
    endor.decompress(m, out=out)
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16)


SHAPES = [
    (1, 1), (1, 7), (1, 8), (1, 9), (3, 5), (1, 63), (1, 64), (1, 65), (1, 511), (1, 512), (1, 513),
    (1, 4095), (1, 4096), (1, 4097), (2, 4096), (3, 4097), (7, 9001),
    (16, 4096), (17, 4095),                      # one workgroup's 16 tiles, ragged neighbour
    (255, 4096), (256, 4096), (257, 4096),       # around one 256-tile chunk
    (1031, 2053),                                # > 2 chunks, nothing aligned
    (1024, 1024),                                # config 1 shape
]


@pytest.mark.parametrize("shape", SHAPES, ids=str)
@pytest.mark.parametrize("keep", [0.0, 0.1, 0.5, 0.9, 1.0])
def test_decompress_matches_oracle(shape, keep):
    rows, cols = shape
    _say(f"case shape={shape} keep={keep}")
    c = _random_compressed(rows, cols, keep, seed=rows * 31 + cols)
    expect = orc.decompress(rows, cols, c.bitmap, c.values)
    got = _gpu_decompress(c)
    assert np.array_equal(got, expect)


def test_pad_bits_are_ignored():
    rows, cols = 3, 1365  # N = 4095: one pad bit in the last byte, 7 more bytes of pad in the word
    c = _random_compressed(rows, cols, 0.5, seed=2)
    expect = orc.decompress(rows, cols, c.bitmap, c.values)
    c.bitmap[rows * cols // 8] |= 0x80
    c.bitmap[rows * cols // 8 + 1:] = 0xFF
    got = _gpu_decompress(c)
    assert np.array_equal(got, expect)


def test_output_is_fully_overwritten_and_nothing_else():
    rows, cols = 37, 4099
    n = rows * cols
    c = _random_compressed(rows, cols, 0.5, seed=3)
    expect = orc.decompress(rows, cols, c.bitmap, c.values).reshape(-1)
    m = endor.to_device(c)
    guard = 4096
    buf = torch.full((guard + n + guard,), POISON, dtype=torch.int16, device="cuda")
    out = buf[guard:guard + n]                      # 16-byte aligned (guard*2 bytes)
    for _ in range(2):                              # twice into the same buffer
        endor.decompress(m, out=out)
    torch.cuda.synchronize()
    host = buf.cpu().numpy().view(np.uint16)
    assert np.all(host[:guard] == POISON) and np.all(host[guard + n:] == POISON)
    assert np.array_equal(host[guard:guard + n], expect)


@pytest.mark.parametrize("voff", [1, 3, 7])
@pytest.mark.parametrize("ooff", [0, 1, 4])
def test_unaligned_values_and_output(voff, ooff):
    """values only 2-byte aligned, dense output only 2-/8-byte aligned."""
    rows, cols = 9, 5000
    n = rows * cols
    c = _random_compressed(rows, cols, 0.5, seed=voff * 10 + ooff)
    expect = orc.decompress(rows, cols, c.bitmap, c.values).reshape(-1)
    bm = torch.from_numpy(c.bitmap).cuda()
    vbuf = torch.full((voff + c.nnz + 9,), 0x5555, dtype=torch.int16, device="cuda")
    vbuf[voff:voff + c.nnz] = torch.from_numpy(c.values.view(np.int16)).cuda()
    m = endor.DeviceMatrix(rows, cols, bm, vbuf[voff:voff + c.nnz], c.nnz)
    obuf = torch.full((ooff + n + 16,), POISON, dtype=torch.int16, device="cuda")
    endor.decompress(m, out=obuf[ooff:ooff + n])
    torch.cuda.synchronize()
    host = obuf.cpu().numpy().view(np.uint16)
    assert np.array_equal(host[ooff:ooff + n], expect)
    assert np.all(host[:ooff] == POISON) and np.all(host[ooff + n:] == POISON)


def test_bitmap_only_8_byte_aligned():
    rows, cols = 300, 4096
    c = _random_compressed(rows, cols, 0.5, seed=8)
    expect = orc.decompress(rows, cols, c.bitmap, c.values)
    buf = torch.zeros(8 + c.bitmap.size, dtype=torch.uint8, device="cuda")
    buf[8:] = torch.from_numpy(c.bitmap).cuda()
    m = endor.DeviceMatrix(rows, cols, buf[8:], torch.from_numpy(c.values.view(np.int16)).cuda(), c.nnz)
    out = endor.decompress(m)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint16), expect)


def test_row_offsets_and_reuse_of_the_table():
    rows, cols = 523, 4111
    w = synth.pruned_fp16(rows, cols, 0.5, seed=11, row_skew=True)
    c = endor.compress(w)
    m = endor.to_device(c)
    ws, ro = endor.build_offsets(m, row_offsets=True)
    out = endor.decompress_with_offsets(m, ws)
    torch.cuda.synchronize()
    assert np.array_equal(ro.cpu().numpy(), orc.row_offsets(rows, cols, c.bitmap))
    assert np.array_equal(ro.cpu().numpy(), c.row_offsets)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), orc.decompress(rows, cols, c.bitmap, c.values))
    assert np.array_equal(out.cpu().numpy().view(np.uint16), w)


def test_row_offsets_tile_aligned_total():
    rows, cols = 64, 4096   # position rows*cols is a tile boundary
    c = _random_compressed(rows, cols, 0.3, seed=12)
    m = endor.to_device(c)
    _, ro = endor.build_offsets(m, row_offsets=True)
    torch.cuda.synchronize()
    assert np.array_equal(ro.cpu().numpy(), orc.row_offsets(rows, cols, c.bitmap))


def test_empty_matrices():
    for rows, cols in [(0, 5), (5, 0), (0, 0)]:
        c = endor.Compressed(rows, cols, np.zeros(0, np.uint8), np.zeros(0, np.uint16), None)
        m = endor.to_device(c)
        out = endor.decompress(m)
        torch.cuda.synchronize()
        assert out.numel() == 0
        _, ro = endor.build_offsets(m, row_offsets=True)
        torch.cuda.synchronize()
        assert not ro.cpu().numpy().any()


def test_batch_of_mixed_shapes_matches_oracle():
    shapes = [(1, 1), (64, 4096), (0, 9), (300, 4099), (17, 33), (1031, 2053)] + [(5, 777)] * 14
    cs = [_random_compressed(r, c, 0.5, seed=100 + i) for i, (r, c) in enumerate(shapes)]
    assert len(cs) > endor.MAX_BATCH                       # exercises the split into launch groups
    mats = [endor.to_device(c) for c in cs]
    outs = [torch.full((c.rows, c.cols), POISON, dtype=torch.int16, device="cuda") for c in cs]
    endor.decompress_batch(mats, outs=outs)
    torch.cuda.synchronize()
    for c, o in zip(cs, outs):
        assert np.array_equal(o.cpu().numpy().view(np.uint16), orc.decompress(c.rows, c.cols, c.bitmap, c.values))
    # table reuse in batch form
    ws = endor.build_offsets_batch(mats)
    outs2 = endor.decompress_batch_with_offsets(mats, ws)
    torch.cuda.synchronize()
    for a, b in zip(outs, outs2):
        assert torch.equal(a, b)


def test_round_trip_special_patterns_through_host_compress():
    w = synth.pruned_fp16(300, 5001, 0.5, seed=21)
    g = np.random.default_rng(1)
    idx = g.integers(0, w.size, size=5000)
    w.reshape(-1)[idx] = np.array([0x8000, 0x0001, 0x7C00, 0xFC00, 0x7E01, 0xFFFF], np.uint16)[g.integers(0, 6, 5000)]
    c = endor.compress(w)
    assert np.array_equal(_gpu_decompress(c), w)


# ---------------------------------------------------------------------------
# the benchmark configurations at full size, in the batched launch bench.py times
# ---------------------------------------------------------------------------
def _full_config(config, keep=0.5, row_skew=False, variant=0):
    shapes = synth.CONFIGS[config]
    cs, dense = [], []
    for i, (name, rows, cols) in enumerate(shapes):
        _say(f"  generating {name} {rows}x{cols} keep={keep} skew={row_skew}")
        w = synth.pruned_fp16(rows, cols, keep, seed=synth.seed_for(config, i, variant), row_skew=row_skew)
        cs.append(endor.compress(w, want_row_offsets=False))
        dense.append(w)
    return cs, dense


def _check_full(cs, dense):
    mats = [endor.to_device(c) for c in cs]
    outs = [torch.full((c.rows, c.cols), POISON, dtype=torch.int16, device="cuda") for c in cs]
    endor.decompress_batch(mats, outs=outs)
    torch.cuda.synchronize()
    for c, w, o in zip(cs, dense, outs):
        _say(f"  oracle {c.rows}x{c.cols}")
        expect = orc.decompress(c.rows, c.cols, c.bitmap, c.values)     # Algorithm 2 on the CPU
        assert np.array_equal(expect, w)                                # and the round trip is lossless
        got = o.cpu().numpy().view(np.uint16)
        assert np.array_equal(got, expect)
        # size law of Section 4.1 on the real buffers
        assert c.bitmap.nbytes + c.values.nbytes == (c.rows * c.cols) // 8 + 2 * c.nnz


@pytest.mark.parametrize("config", [0, 1, 2, 3], ids=["1024sq", "opt66b_attn", "opt66b_ffn", "llama2_70b_layer"])
def test_full_size_configs(config):
    _say(f"full-size config {config}")
    cs, dense = _full_config(config)
    _check_full(cs, dense)


@pytest.mark.parametrize("keep", [0.1, 0.3, 0.7])
def test_down_proj_keep_sweep(keep):
    _say(f"down_proj keep={keep}")
    cs, dense = _full_config(4, keep=keep, variant=int(keep * 10))
    assert abs(cs[0].nnz / (8192 * 28672) - keep) < 1e-3
    _check_full(cs, dense)


def test_down_proj_row_skew():
    _say("down_proj Beta(2,2) row skew")
    cs, dense = _full_config(4, row_skew=True, variant=9)
    _check_full(cs, dense)


# ---------------------------------------------------------------------------
# pinned host -> device copy overlapped with decompression (two streams)
# ---------------------------------------------------------------------------
def _expect(c):
    return orc.decompress(c.rows, c.cols, c.bitmap, c.values)


def test_h2d_pipeline_whole_matrices_matches_oracle():
    shapes = [(300, 4099), (1031, 2053), (64, 4096), (1, 1), (777, 1000), (0, 7)]
    cs = [endor.compress(synth.pruned_fp16(r, c, 0.5, seed=40 + i)) for i, (r, c) in enumerate(shapes)]
    blobs = [endor.pin(c) for c in cs]
    outs = [torch.full((c.rows, c.cols), POISON, dtype=torch.int16, device="cuda") for c in cs]
    s_copy, s_comp = torch.cuda.Stream(), torch.cuda.Stream()
    pipe = endor.Pipeline.for_blobs(blobs, s_copy, s_comp)
    torch.cuda.synchronize()
    pipe.run(blobs, outs)
    torch.cuda.synchronize()
    for c, o in zip(cs, outs):
        assert np.array_equal(o.cpu().numpy().view(np.uint16), _expect(c))
    pipe.close()


def test_h2d_pipeline_back_to_back_calls_keep_their_slots_apart():
    """Two calls with different blobs and outputs of their own, no synchronisation between
    them: the second call's copies reuse the staging slots of the first, whose decompressions
    may still be running, so the events kept in the pipeline object must order them."""
    shapes = [(900, 4099), (1031, 2053), (640, 4096), (1500, 3000), (777, 1000), (2048, 2048), (333, 4100)]
    first = [endor.compress(synth.pruned_fp16(r, c, 0.5, seed=300 + i)) for i, (r, c) in enumerate(shapes)]
    second = [endor.compress(synth.pruned_fp16(r, c, 0.5, seed=400 + i)) for i, (r, c) in enumerate(shapes)]
    b1, b2 = [endor.pin(c) for c in first], [endor.pin(c) for c in second]
    o1 = [torch.full((c.rows, c.cols), POISON, dtype=torch.int16, device="cuda") for c in first]
    o2 = [torch.full((c.rows, c.cols), POISON, dtype=torch.int16, device="cuda") for c in second]
    s_copy, s_comp = torch.cuda.Stream(), torch.cuda.Stream()
    pipe = endor.Pipeline.for_blobs(b1 + b2, s_copy, s_comp)
    torch.cuda.synchronize()
    for _ in range(3):
        pipe.run(b1, o1)
        pipe.run(b2, o2)
    torch.cuda.synchronize()
    for c, o in zip(first + second, o1 + o2):
        assert np.array_equal(o.cpu().numpy().view(np.uint16), _expect(c))
    pipe.close()


@pytest.mark.parametrize("shape,nblocks", [((2048, 4096), 8), ((1031, 2053), 5), ((96, 24), 3), ((333, 64), 50)])
@pytest.mark.parametrize("wide", [True, False], ids=["fp16", "u8"])
def test_h2d_pipeline_row_blocks_matches_oracle(shape, nblocks, wide):
    rows, cols = shape
    w = synth.pruned_fp16(rows, cols, 0.5, seed=50, row_skew=True) if wide else synth.pruned_int8(rows, cols, 0.4, seed=51)
    c = endor.compress(w)
    blobs = endor.row_blocks(c, nblocks)
    assert sum(b.rows for b in blobs) == rows and sum(b.nnz for b in blobs) == c.nnz
    out = torch.full((rows, cols), POISON & 0x7F, dtype=torch.int16 if wide else torch.uint8, device="cuda")
    outs = [out[b.row_begin:b.row_begin + b.rows] for b in blobs]
    s_copy, s_comp = torch.cuda.Stream(), torch.cuda.Stream()
    pipe = endor.Pipeline.for_blobs(blobs, s_copy, s_comp)
    torch.cuda.synchronize()
    pipe.run(blobs, outs)
    torch.cuda.synchronize()
    expect = _expect(c)
    assert np.array_equal(out.cpu().numpy().view(w.dtype), expect) and np.array_equal(expect, w)
    pipe.close()


def test_h2d_pipeline_u8_whole_matrices():
    """The 8-bit variant through the transfer pipeline (Section 4.2: same bitmap, one byte per value)."""
    shapes = [(300, 4099), (1031, 2053), (64, 4096), (1, 1)]
    cs = [endor.compress(synth.pruned_int8(r, c, 0.5, seed=60 + i)) for i, (r, c) in enumerate(shapes)]
    blobs = [endor.pin(c) for c in cs]
    assert all(b.elem_bytes == 1 for b in blobs)
    outs = [torch.full((c.rows, c.cols), 0x7F, dtype=torch.uint8, device="cuda") for c in cs]
    s_copy, s_comp = torch.cuda.Stream(), torch.cuda.Stream()
    pipe = endor.Pipeline.for_blobs(blobs, s_copy, s_comp)
    torch.cuda.synchronize()
    pipe.run(blobs, outs)
    pipe.run(blobs, outs)
    torch.cuda.synchronize()
    for c, o in zip(cs, outs):
        assert np.array_equal(o.cpu().numpy(), _expect(c))
    pipe.close()


def test_h2d_pipeline_refuses_a_blob_larger_than_its_slots():
    small = endor.pin(endor.compress(synth.pruned_fp16(8, 64, 0.5, seed=1)))
    big = endor.pin(endor.compress(synth.pruned_fp16(512, 4096, 0.5, seed=2)))
    s_copy, s_comp = torch.cuda.Stream(), torch.cuda.Stream()
    pipe = endor.Pipeline.for_blobs([small], s_copy, s_comp)
    out = torch.empty((512, 4096), dtype=torch.int16, device="cuda")
    with pytest.raises(endor.EndorError) as e:
        pipe.run([big], [out])
    assert e.value.status == 2
    pipe.close()


# ---------------------------------------------------------------------------
# 8-bit elements (Section 4.2): same bitmap, one byte per value
# ---------------------------------------------------------------------------
def _random_compressed_u8(rows, cols, keep, seed):
    n = rows * cols
    g = np.random.default_rng(seed)
    bits = g.random(n) < keep
    bitmap = np.zeros(endor.bitmap_bytes(rows, cols), np.uint8)
    packed = np.packbits(bits, bitorder="little")
    bitmap[: packed.size] = packed
    values = g.integers(0, 256, size=int(bits.sum()), dtype=np.uint16).astype(np.uint8)   # zero bytes allowed
    return endor.Compressed(rows, cols, bitmap, values, None)


@pytest.mark.parametrize("shape", SHAPES, ids=str)
@pytest.mark.parametrize("keep", [0.0, 0.1, 0.5, 0.9, 1.0])
def test_decompress_u8_matches_oracle(shape, keep):
    rows, cols = shape
    _say(f"u8 case shape={shape} keep={keep}")
    c = _random_compressed_u8(rows, cols, keep, seed=rows * 17 + cols)
    expect = orc.decompress(rows, cols, c.bitmap, c.values)
    assert expect.dtype == np.uint8
    m = endor.to_device(c)
    out = torch.full((rows, cols), 0xA5, dtype=torch.uint8, device="cuda")
    endor.decompress(m, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), expect)


@pytest.mark.parametrize("wide", [True, False], ids=["fp16", "u8"])
def test_dense_tiles_inside_a_sparse_matrix(wide):
    """A matrix sparse enough overall for the small-staging expander that still holds tiles with
    more 1 bits than that staging area takes: all 4096 set, 1025 (one over), exactly 1024 (the
    limit), a dense run across a tile boundary, and a dense ragged last tile."""
    rows, cols = 64, 4099
    n = rows * cols
    _say(f"dense tiles in a sparse matrix wide={wide}")
    g = np.random.default_rng(77 + wide)
    bits = g.random(n) < 0.05
    bits[3 * 4096:4 * 4096] = True
    for tile, ones in ((7, 1025), (9, 1024), (12, 2500), (13, 4095)):
        t = np.zeros(4096, bool)
        t[g.choice(4096, ones, replace=False)] = True
        bits[tile * 4096:(tile + 1) * 4096] = t
    bits[20 * 4096 - 700:20 * 4096 + 900] = True
    bits[(n // 4096) * 4096:] = True
    assert bits.sum() * 5 < n
    bitmap = np.zeros(endor.bitmap_bytes(rows, cols), np.uint8)
    packed = np.packbits(bits, bitorder="little")
    bitmap[: packed.size] = packed
    nnz = int(bits.sum())
    if wide:
        values = g.integers(0, 1 << 16, size=nnz, dtype=np.uint32).astype(np.uint16)
    else:
        values = g.integers(0, 256, size=nnz, dtype=np.uint16).astype(np.uint8)
    c = endor.Compressed(rows, cols, bitmap, values, None)
    expect = orc.decompress(rows, cols, c.bitmap, c.values)
    m = endor.to_device(c)
    out = torch.full((rows, cols), 0x5A, dtype=torch.int16 if wide else torch.uint8, device="cuda")
    for _ in range(2):
        endor.decompress(m, out=out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got.view(np.uint16) if wide else got, expect)


@pytest.mark.parametrize("voff", [1, 5, 15])
@pytest.mark.parametrize("ooff", [0, 1, 8])
def test_u8_unaligned_values_and_output(voff, ooff):
    rows, cols = 9, 5000
    n = rows * cols
    c = _random_compressed_u8(rows, cols, 0.5, seed=voff * 10 + ooff)
    expect = orc.decompress(rows, cols, c.bitmap, c.values).reshape(-1)
    bm = torch.from_numpy(c.bitmap).cuda()
    vbuf = torch.full((voff + c.nnz + 17,), 0x55, dtype=torch.uint8, device="cuda")
    vbuf[voff:voff + c.nnz] = torch.from_numpy(c.values).cuda()
    m = endor.DeviceMatrix(rows, cols, bm, vbuf[voff:voff + c.nnz], c.nnz)
    obuf = torch.full((ooff + n + 32,), 0xA5, dtype=torch.uint8, device="cuda")
    endor.decompress(m, out=obuf[ooff:ooff + n])
    torch.cuda.synchronize()
    host = obuf.cpu().numpy()
    assert np.array_equal(host[ooff:ooff + n], expect)
    assert np.all(host[:ooff] == 0xA5) and np.all(host[ooff + n:] == 0xA5)


def test_u8_batch_and_table_reuse_full_size():
    """The paper's 8-bit example shape (9216 x 36864, half kept) plus its transpose shape, batched."""
    _say("u8 full size")
    cs, dense = [], []
    for i, (rows, cols) in enumerate([(9216, 36864), (36864, 9216)]):
        w = synth.pruned_int8(rows, cols, 0.5, seed=synth.seed_for(2, i, 8))
        cs.append(endor.compress(w, want_row_offsets=False))
        dense.append(w)
    c0 = cs[0]
    # size law of Section 4.2 on real buffers: 1/8 + nnz/N of the dense size (62 % printed for one half kept)
    ratio = (c0.rows * c0.cols // 8 + c0.nnz) / (c0.rows * c0.cols)
    assert abs(ratio - 0.625) < 1e-3
    mats = [endor.to_device(c) for c in cs]
    outs = [torch.full((c.rows, c.cols), 0xA5, dtype=torch.uint8, device="cuda") for c in cs]
    _, ws = endor.decompress_batch(mats, outs=outs)
    torch.cuda.synchronize()
    for c, w, o in zip(cs, dense, outs):
        expect = orc.decompress(c.rows, c.cols, c.bitmap, c.values)
        assert np.array_equal(expect, w)
        assert np.array_equal(o.cpu().numpy(), expect)
    again = endor.decompress_with_offsets(mats[0], ws)   # matrix 0's table sits at the start of the batch workspace
    both = endor.decompress_batch_with_offsets(mats, ws)
    torch.cuda.synchronize()
    assert torch.equal(again, outs[0])
    assert all(torch.equal(a, b) for a, b in zip(both, outs))


# ---------------------------------------------------------------------------
# row-subset decompression (the selective load of Section 4.2)
# ---------------------------------------------------------------------------
ROW_SHAPES = [(40, 77), (5, 3), (64, 64), (33, 4096), (17, 4097), (9, 12345), (300, 8192), (50, 28672), (7, 28673)]


@pytest.mark.parametrize("shape", ROW_SHAPES, ids=str)
@pytest.mark.parametrize("wide", [True, False], ids=["fp16", "u8"])
def test_decompress_rows_matches_oracle(shape, wide):
    rows, cols = shape
    _say(f"rows case shape={shape} wide={wide}")
    if wide:
        w = synth.pruned_fp16(rows, cols, 0.5, seed=rows + cols, row_skew=True)
    else:
        w = synth.pruned_int8(rows, cols, 0.4, seed=rows + cols)
    c = endor.compress(w)
    m = endor.to_device(c)
    g = np.random.default_rng(rows)
    sel_np = np.concatenate([g.integers(0, rows, size=max(1, rows // 2)), [rows - 1, 0, 0]]).astype(np.int64)
    sel = torch.from_numpy(sel_np).cuda()
    ro_host = torch.from_numpy(c.row_offsets).cuda()
    _, ro_dev = endor.build_offsets(m, row_offsets=True)
    expect = orc.decompress_selected_rows(cols, sel_np, c.row_offsets, c.bitmap, c.values)
    assert np.array_equal(expect, w.view(expect.dtype)[sel_np])          # the oracle's own pin, on this input
    for ro in (ro_host, ro_dev):
        out = torch.full((sel_np.size, cols), 0x5A, dtype=torch.int16 if wide else torch.uint8, device="cuda")
        endor.decompress_rows(m, ro, sel, out=out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(expect.dtype), expect)


def test_decompress_rows_dense_rows_inside_a_sparse_matrix():
    """Overall sparse enough for the row kernel's smaller staging area (2304 values), with row
    segments that exceed it: all 4096 set, 2305 (one over), exactly 2304 (the limit), and a dense
    ragged last segment."""
    rows, cols = 12, 2 * 4096 + 37
    _say("rows: dense rows in a sparse matrix")
    g = np.random.default_rng(91)
    w = g.integers(1, 1 << 16, size=(rows, cols), dtype=np.uint32).astype(np.uint16)
    w[g.random((rows, cols)) >= 0.1] = 0
    w[2, :] = g.integers(1, 1 << 16, size=cols, dtype=np.uint32).astype(np.uint16)        # every segment full
    for row, ones in ((4, 2305), (5, 2304)):
        seg = np.zeros(4096, np.uint16)
        seg[g.choice(4096, ones, replace=False)] = g.integers(1, 1 << 16, size=ones, dtype=np.uint32).astype(np.uint16)
        w[row, 4096:8192] = seg
    w[7, 8192:] = 0x3C00
    assert np.count_nonzero(w) * 16 <= (rows * cols // 16) * 9 * 16
    c = endor.compress(w)
    m = endor.to_device(c)
    sel_np = np.array([2, 4, 5, 7, 0, 11, 2], np.int64)
    out = torch.full((sel_np.size, cols), POISON, dtype=torch.int16, device="cuda")
    for _ in range(2):
        endor.decompress_rows(m, torch.from_numpy(c.row_offsets).cuda(), torch.from_numpy(sel_np).cuda(), out=out)
    torch.cuda.synchronize()
    expect = orc.decompress_selected_rows(cols, sel_np, c.row_offsets, c.bitmap, c.values)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), expect)
    assert np.array_equal(expect, w[sel_np])


def test_decompress_rows_out_of_range_index_is_skipped():
    rows, cols = 12, 5000
    w = synth.pruned_fp16(rows, cols, 0.5, seed=77)
    c = endor.compress(w)
    m = endor.to_device(c)
    sel_np = np.array([3, -1, rows, 11], np.int64)
    out = torch.full((4, cols), POISON, dtype=torch.int16, device="cuda")
    endor.decompress_rows(m, torch.from_numpy(c.row_offsets).cuda(), torch.from_numpy(sel_np).cuda(), out=out)
    torch.cuda.synchronize()
    host = out.cpu().numpy().view(np.uint16)
    assert np.array_equal(host[0], w[3]) and np.array_equal(host[3], w[11])
    assert np.all(host[1] == POISON) and np.all(host[2] == POISON)


def test_decompress_rows_unaligned_output():
    rows, cols = 20, 4099   # odd row pitch: every output row starts 2-byte aligned only
    w = synth.pruned_fp16(rows, cols, 0.5, seed=78)
    c = endor.compress(w)
    m = endor.to_device(c)
    sel_np = np.arange(rows - 1, -1, -1, dtype=np.int64)
    buf = torch.full((1 + rows * cols + 8,), POISON, dtype=torch.int16, device="cuda")
    endor.decompress_rows(m, torch.from_numpy(c.row_offsets).cuda(), torch.from_numpy(sel_np).cuda(),
                          out=buf[1:1 + rows * cols])
    torch.cuda.synchronize()
    host = buf.cpu().numpy().view(np.uint16)
    assert np.array_equal(host[1:1 + rows * cols].reshape(rows, cols), w[sel_np])
    assert host[0] == POISON and np.all(host[1 + rows * cols:] == POISON)


def test_decompress_rows_full_size_gate_proj():
    """A tenth of the rows of a Llama2-70B gate projection (28672 x 8192)."""
    rows, cols = 28672, 8192
    _say("rows full size")
    w = synth.pruned_fp16(rows, cols, 0.5, seed=synth.seed_for(3, 4))
    c = endor.compress(w)
    m = endor.to_device(c)
    sel_np = np.sort(np.random.default_rng(5).choice(rows, size=rows // 10, replace=False)).astype(np.int64)
    out = endor.decompress_rows(m, torch.from_numpy(c.row_offsets).cuda(), torch.from_numpy(sel_np).cuda())
    torch.cuda.synchronize()
    expect = orc.decompress_selected_rows(cols, sel_np, c.row_offsets, c.bitmap, c.values)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), expect)
    assert np.array_equal(expect, w[sel_np])


# ---------------------------------------------------------------------------
# Algorithm 1 on the device (endor_compress_device) against the oracle's Algorithm 1
# ---------------------------------------------------------------------------
def _check_device_compress(w):
    rows, cols = w.shape
    dense = torch.from_numpy(w.view(np.int16) if w.dtype.itemsize == 2 else w).cuda()
    m, ws, ro = endor.compress_device(dense, row_offsets=True)
    torch.cuda.synchronize()
    b, v, r = orc.compress(w)
    bm = m.bitmap.cpu().numpy()
    assert np.array_equal(bm[: b.size], b) and not bm[b.size:].any()      # pad bits/bytes are zero
    assert m.nnz == v.size
    assert np.array_equal(m.values.cpu().numpy().view(v.dtype), v)
    assert np.array_equal(ro.cpu().numpy(), r)
    # and the table it leaves behind serves decompression: device round trip
    back = endor.decompress_with_offsets(m, ws)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy().view(w.dtype), w)


@pytest.mark.parametrize("shape", SHAPES, ids=str)
@pytest.mark.parametrize("keep", [0.0, 0.5, 1.0])
def test_compress_device_matches_oracle(shape, keep):
    rows, cols = shape
    _say(f"device compress shape={shape} keep={keep}")
    g = np.random.default_rng(rows * 3 + cols)
    w = g.integers(1, 1 << 16, size=(rows, cols), dtype=np.uint32).astype(np.uint16)
    w[g.random((rows, cols)) >= keep] = 0
    if w.size > 6:
        w.reshape(-1)[[1, 3, 5]] = [0x8000, 0x0001, 0x7E01]     # -0.0, subnormal, NaN are values
    _check_device_compress(w)


@pytest.mark.parametrize("shape", [(1, 1), (3, 5), (1, 4097), (33, 4099), (1031, 2053)], ids=str)
def test_compress_device_u8_matches_oracle(shape):
    _check_device_compress(synth.pruned_int8(shape[0], shape[1], 0.5, seed=sum(shape)))


def test_compress_device_counting_pass_and_capacity():
    w = synth.pruned_fp16(100, 4099, 0.5, seed=3)
    nnz_true = int(np.count_nonzero(w))
    dense = torch.from_numpy(w.view(np.int16)).cuda()
    # capacity 0: nothing is written to values, the count still comes back
    guard = torch.full((64,), POISON, dtype=torch.int16, device="cuda")
    with pytest.raises(endor.EndorError):
        endor.compress_device(dense, values=guard[:0])
    assert torch.all(guard == POISON)
    # capacity one short of nnz: the last value is not written, nothing past the buffer is touched
    buf = torch.full((nnz_true + 63,), POISON, dtype=torch.int16, device="cuda")
    with pytest.raises(endor.EndorError):
        endor.compress_device(dense, values=buf[: nnz_true - 1])
    torch.cuda.synchronize()
    host = buf.cpu().numpy().view(np.uint16)
    assert np.all(host[nnz_true - 1:] == POISON)
    assert np.array_equal(host[: nnz_true - 1], orc.compress(w)[1][: nnz_true - 1])


def test_compress_device_unaligned_dense_and_values():
    rows, cols = 31, 4101
    w = synth.pruned_fp16(rows, cols, 0.5, seed=4)
    big = torch.zeros(1 + rows * cols, dtype=torch.int16, device="cuda")
    big[1:] = torch.from_numpy(w.view(np.int16)).cuda().reshape(-1)
    dense = big[1:].view(rows, cols)                     # 2-byte aligned only
    vbuf = torch.full((3 + rows * cols,), POISON, dtype=torch.int16, device="cuda")
    m, ws, _ = endor.compress_device(dense, values=vbuf[3:])
    torch.cuda.synchronize()
    b, v, _ = orc.compress(w)
    assert np.array_equal(m.values.cpu().numpy().view(np.uint16), v)
    assert np.array_equal(m.bitmap.cpu().numpy()[: b.size], b)
    assert torch.all(vbuf[:3] == POISON) and torch.all(vbuf[3 + v.size:] == POISON)


def test_compress_device_many_chunks():
    """More chunks than lanes (so the sum of chunk totals takes several rounds) and a last
    chunk with a single tile."""
    _say("device compress, 66 chunks")
    rows, cols = 16897, 4096                                  # 16897 tiles = 66 chunks + 1 tile
    _check_device_compress(synth.pruned_fp16(rows, cols, 0.3, seed=21))


def test_compress_device_full_size_down_proj():
    _say("device compress full size")
    w = synth.pruned_fp16(8192, 28672, 0.5, seed=synth.seed_for(4, 0))
    _check_device_compress(w)


# ---------------------------------------------------------------------------
# fused consumer: y = W x straight from the compressed form (fp32 accumulation)
# ---------------------------------------------------------------------------
def _gemv_tolerance(w_bits, x16, cols):
    """fp16 products are exact in fp32; every fp32 addition on the longest chain (a lane adds
    cols/64 products one after the other, then 6 adds across lanes and one more) contributes
    at most 2^-24 of the running magnitude, so |err_i| <= (cols/64 + 8) * 2^-24 * sum_j |W_ij x_j|
    (plus one ulp of the smallest normal for underflow)."""
    absw = np.abs(w_bits.view(np.float16).astype(np.float64))
    absx = np.abs(x16.astype(np.float64))
    return (cols / 64 + 8) * 2.0 ** -24 * 1.01 * (absw @ absx) + 2.0 ** -126


GEMV_SHAPES = [(1, 1), (3, 5), (7, 13), (33, 65), (5, 4095), (5, 4096), (5, 4097), (40, 1000), (64, 8192),
               (16, 28672), (9, 12345)]


@pytest.mark.parametrize("shape", GEMV_SHAPES, ids=str)
def test_gemv_matches_oracle(shape):
    rows, cols = shape
    _say(f"gemv case shape={shape}")
    w = synth.pruned_fp16(rows, cols, 0.5, seed=rows * 5 + cols, row_skew=True)
    w.reshape(-1)[:: 97] = 0x0001                      # fp16 subnormals among the values
    x16 = np.random.default_rng(cols).standard_normal(cols).astype(np.float16)
    c = endor.compress(w)
    m = endor.to_device(c)
    ro = torch.from_numpy(c.row_offsets).cuda()
    y = endor.gemv_f16(m, ro, torch.from_numpy(x16).cuda())
    torch.cuda.synchronize()
    ref = orc.gemv_f16(rows, cols, c.bitmap, c.values, x16)
    err = np.abs(y.cpu().numpy().astype(np.float64) - ref)
    tol = _gemv_tolerance(w, x16, cols)
    assert np.all(err <= tol), (err.max(), tol[np.argmax(err)])


def test_gemv_unaligned_x_and_device_row_offsets():
    rows, cols = 50, 9001
    w = synth.pruned_fp16(rows, cols, 0.5, seed=3)
    x16 = np.random.default_rng(1).standard_normal(cols).astype(np.float16)
    c = endor.compress(w)
    m = endor.to_device(c)
    _, ro = endor.build_offsets(m, row_offsets=True)
    xbuf = torch.zeros(cols + 1, dtype=torch.float16, device="cuda")
    xbuf[1:] = torch.from_numpy(x16).cuda()
    y = endor.gemv_f16(m, ro, xbuf[1:])
    torch.cuda.synchronize()
    ref = orc.gemv_f16(rows, cols, c.bitmap, c.values, x16)
    assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - ref) <= _gemv_tolerance(w, x16, cols))


def test_gemv_nonfinite_x_like_the_dense_product():
    rows, cols = 4, 100
    w = synth.pruned_fp16(rows, cols, 0.5, seed=9)
    w[0, 7] = 0            # a zero element meets x = inf: 0 * inf = nan, as with the dense matrix
    w[1, 7] = 0x3C00       # 1.0 meets inf: +inf (unless other terms make it nan)
    x16 = np.random.default_rng(2).standard_normal(cols).astype(np.float16)
    x16[7] = np.inf
    c = endor.compress(w)
    m = endor.to_device(c)
    y = endor.gemv_f16(m, torch.from_numpy(c.row_offsets).cuda(), torch.from_numpy(x16).cuda())
    torch.cuda.synchronize()
    ref = orc.gemv_f16(rows, cols, c.bitmap, c.values, x16)
    got = y.cpu().numpy().astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref))


@pytest.mark.parametrize("shape", [(8192, 28672), (28672, 8192)], ids=["down_proj", "gate_proj"])
def test_gemv_full_size(shape):
    rows, cols = shape
    _say(f"gemv full size {shape}")
    w = synth.pruned_fp16(rows, cols, 0.5, seed=synth.seed_for(3, 6 if rows == 8192 else 4))
    x16 = np.random.default_rng(11).standard_normal(cols).astype(np.float16)
    c = endor.compress(w)
    m = endor.to_device(c)
    y = endor.gemv_f16(m, torch.from_numpy(c.row_offsets).cuda(), torch.from_numpy(x16).cuda())
    torch.cuda.synchronize()
    ref = orc.gemv_f16(rows, cols, c.bitmap, c.values, x16)          # every row
    err = np.abs(y.cpu().numpy().astype(np.float64) - ref)
    tol = np.concatenate([_gemv_tolerance(w[r0:r0 + 1024], x16, cols) for r0 in range(0, rows, 1024)])
    assert np.all(err <= tol)


# ---------------------------------------------------------------------------
# fused small-batch product on the matrix cores: Y = X W^T, nb <= 16
# ---------------------------------------------------------------------------
def _gemm_tolerance(w_bits, X16, cols):
    """fp16 products are exact in fp32.  A matrix instruction adds 32 of them to the fp32
    accumulator; its internal order is not documented, so each instruction is charged two
    roundings of the running magnitude (a probe on the device returned the correctly rounded
    exact sum, i.e. one), and the column ranges are added with one rounding each:
    |err| <= (2 * ceil(cols/32) + 16 + 8) * 2^-24 * sum_j |W_ij x_bj|, plus underflow."""
    absw = np.abs(w_bits.view(np.float16).astype(np.float64))
    absx = np.abs(X16.astype(np.float64))
    return (2 * ((cols + 31) // 32) + 24) * 2.0 ** -24 * 1.01 * (absx @ absw.T) + 2.0 ** -126


def _gpu_gemm(c, X16, **kw):
    m = endor.to_device(c)
    ws, _ = endor.build_offsets(m)
    Y = endor.gemm_f16(m, ws, torch.from_numpy(X16.view(np.int16)).cuda().view(torch.float16), **kw)
    torch.cuda.synchronize()
    return Y.cpu().numpy().astype(np.float64)


GEMM_SHAPES = [(1, 1), (3, 5), (7, 13), (16, 256), (17, 257), (33, 65), (5, 4095), (5, 4096), (5, 4097), (40, 1000),
               (64, 8192), (16, 28672), (9, 12345), (100, 2053), (300, 4099)]


@pytest.mark.parametrize("shape", GEMM_SHAPES, ids=str)
@pytest.mark.parametrize("nb", [1, 3, 16])
def test_gemm_matches_oracle(shape, nb):
    rows, cols = shape
    _say(f"gemm case shape={shape} nb={nb}")
    w = synth.pruned_fp16(rows, cols, 0.5, seed=rows * 5 + cols, row_skew=True)
    w.reshape(-1)[:: 97] = 0x0001                      # fp16 subnormals among the values
    X16 = np.random.default_rng(cols + nb).standard_normal((nb, cols)).astype(np.float16)
    c = endor.compress(w)
    got = _gpu_gemm(c, X16)
    ref = orc.gemm_f16(rows, cols, c.bitmap, c.values, X16)
    assert got.shape == ref.shape
    assert np.all(np.abs(got - ref) <= _gemm_tolerance(w, X16, cols))


@pytest.mark.parametrize("shape", [(33, 65), (100, 2053), (64, 8192), (300, 4099)], ids=str)
def test_gemm_is_exact_on_integer_valued_inputs(shape):
    """Small integers in W and X: every product and every partial sum is an integer below 2^24,
    exactly representable in fp32, so the result must equal the oracle's bit for bit whatever
    the order of addition - a dropped, doubled or misplaced term cannot hide in a tolerance."""
    rows, cols = shape
    g = np.random.default_rng(rows + cols)
    wi = (g.integers(-8, 9, (rows, cols)) * (g.random((rows, cols)) < 0.5)).astype(np.float16)
    X16 = g.integers(-8, 9, (16, cols)).astype(np.float16)
    c = endor.compress(wi)
    got = _gpu_gemm(c, X16)
    assert np.array_equal(got, orc.gemm_f16(rows, cols, c.bitmap, c.values, X16))


def test_gemm_subnormal_inputs_count_in_full():
    rows, cols = 20, 700
    g = np.random.default_rng(5)
    wi = (g.integers(1, 1024, (rows, cols)) * (g.random((rows, cols)) < 0.5)).astype(np.uint16)   # fp16 subnormals
    X16 = g.integers(-4, 5, (4, cols)).astype(np.float16)
    c = endor.compress(wi)
    got = _gpu_gemm(c, X16)
    ref = orc.gemm_f16(rows, cols, c.bitmap, c.values, X16)
    assert np.any(ref != 0) and np.array_equal(got, ref)          # integers * 2^-24: exact in fp32


def test_gemm_unaligned_x_and_padded_rows_of_x():
    rows, cols, nb = 40, 1000, 5
    w = synth.pruned_fp16(rows, cols, 0.5, seed=8)
    c = endor.compress(w)
    m = endor.to_device(c)
    ws, _ = endor.build_offsets(m)
    X16 = np.random.default_rng(1).standard_normal((nb, cols)).astype(np.float16)
    ref = orc.gemm_f16(rows, cols, c.bitmap, c.values, X16)
    tol = _gemm_tolerance(w, X16, cols)
    # rows of X 1003 elements apart, starting 2 bytes off a 16-byte boundary: the slow load path
    buf = torch.zeros(nb * 1003 + 9, dtype=torch.float16, device="cuda")
    Xd = torch.as_strided(buf, (nb, cols), (1003, 1), storage_offset=1)
    Xd.copy_(torch.from_numpy(X16.view(np.int16)).cuda().view(torch.float16))
    Y = endor.gemm_f16(m, ws, Xd)
    torch.cuda.synchronize()
    assert np.all(np.abs(Y.cpu().numpy().astype(np.float64) - ref) <= tol)
    # aligned, rows 1008 apart: the fast path with ldx > cols
    buf2 = torch.zeros(nb * 1008, dtype=torch.float16, device="cuda")
    Xe = torch.as_strided(buf2, (nb, cols), (1008, 1))
    Xe.copy_(Xd)
    Y2 = endor.gemm_f16(m, ws, Xe)
    torch.cuda.synchronize()
    assert np.all(np.abs(Y2.cpu().numpy().astype(np.float64) - ref) <= tol)


@pytest.mark.parametrize("voff", [1, 3, 6])
@pytest.mark.parametrize("shape", [(50, 9001), (200, 4096), (33, 700)], ids=str)
def test_products_with_values_at_2_byte_alignment(voff, shape):
    """`values` starting 2, 6 or 12 bytes off a 16-byte boundary, with guard patterns around it:
    the products read 20-byte windows from dword boundaries, and those at the two ends of the
    array must take the guarded path."""
    rows, cols = shape
    _say(f"products, values offset {voff} elements, shape {shape}")
    w = synth.pruned_fp16(rows, cols, 0.5, seed=21 + voff)
    c = endor.compress(w)
    vbuf = torch.full((voff + c.nnz + 24,), 0x7E00, dtype=torch.int16, device="cuda")   # NaN patterns around
    vbuf[voff:voff + c.nnz] = torch.from_numpy(c.values.view(np.int16)).cuda()
    bm = torch.from_numpy(c.bitmap).cuda()
    m = endor.DeviceMatrix(rows, cols, bm, vbuf[voff:voff + c.nnz], c.nnz)
    ws, ro = endor.build_offsets(m, row_offsets=True)
    x16 = np.random.default_rng(2).standard_normal(cols).astype(np.float16)
    y = endor.gemv_f16(m, ro, torch.from_numpy(x16.view(np.int16)).cuda().view(torch.float16))
    X16 = np.random.default_rng(3).standard_normal((3, cols)).astype(np.float16)
    Y = endor.gemm_f16(m, ws, torch.from_numpy(X16.view(np.int16)).cuda().view(torch.float16))
    torch.cuda.synchronize()
    ref = orc.gemv_f16(rows, cols, c.bitmap, c.values, x16)
    assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - ref) <= _gemv_tolerance(w, x16, cols))
    refm = orc.gemm_f16(rows, cols, c.bitmap, c.values, X16)
    assert np.all(np.abs(Y.cpu().numpy().astype(np.float64) - refm) <= _gemm_tolerance(w, X16, cols))


def test_gemm_nonfinite_x_like_the_dense_product():
    rows, cols = 4, 100
    w = synth.pruned_fp16(rows, cols, 0.5, seed=9)
    w[0, 7] = 0            # a zero element meets x = inf: 0 * inf = nan, as with the dense matrix
    w[1, 7] = 0x3C00
    X16 = np.random.default_rng(2).standard_normal((3, cols)).astype(np.float16)
    X16[1, 7] = np.inf
    c = endor.compress(w)
    got = _gpu_gemm(c, X16)
    ref = orc.gemm_f16(rows, cols, c.bitmap, c.values, X16)
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(np.isinf(got), np.isinf(ref))
    ok = np.isfinite(ref)
    assert np.all(np.abs(got - ref)[ok] <= _gemm_tolerance(w, X16, cols)[ok])


@pytest.mark.parametrize("shape", [(8192, 28672), (28672, 8192)], ids=["down_proj", "gate_proj"])
def test_gemm_full_size(shape):
    """Both orientations of the Llama2-70B FFN at full size, 16 right-hand sides, every output:
    random fp16 data within the derived bound, and integer-valued data exactly."""
    rows, cols = shape
    _say(f"gemm full size {shape}")
    w = synth.pruned_fp16(rows, cols, 0.5, seed=synth.seed_for(3, 6 if rows == 8192 else 4))
    X16 = np.random.default_rng(11).standard_normal((16, cols)).astype(np.float16)
    c = endor.compress(w)
    got = _gpu_gemm(c, X16)
    ref = orc.gemm_f16(rows, cols, c.bitmap, c.values, X16, threads=16)
    tol = np.concatenate([_gemm_tolerance(w[r0:r0 + 1024], X16, cols) for r0 in range(0, rows, 1024)], axis=1)
    assert np.all(np.abs(got - ref) <= tol)
    # the same bitmap with small integers as values, and integer right-hand sides: exact
    g = np.random.default_rng(12)
    vi = g.integers(1, 9, c.nnz).astype(np.float16).view(np.uint16)
    vi[g.random(c.nnz) < 0.5] |= 0x8000                                   # signs
    Xi = g.integers(-8, 9, (16, cols)).astype(np.float16)
    ci = endor.Compressed(rows, cols, c.bitmap, vi, c.row_offsets)
    got = _gpu_gemm(ci, Xi)
    assert np.array_equal(got, orc.gemm_f16(rows, cols, c.bitmap, vi, Xi, threads=16))


# ---------------------------------------------------------------------------
# precondition violations stay memory-safe; check mode reports them
# ---------------------------------------------------------------------------
def test_short_values_are_zero_extended_and_nothing_past_nnz_is_read():
    """A blob whose nnz is smaller than the number of 1 bits (truncated values): the output
    equals Algorithm 2 on the values extended with zeros, i.e. nothing at or past
    values + nnz was read (there sit non-zero guard patterns), and the guard zones around the
    output are intact."""
    rows, cols = 700, 4099
    c = _random_compressed(rows, cols, 0.5, seed=77, zero_values=False)
    for short in (c.nnz - 1, c.nnz - 4097, c.nnz // 2, 5, 0):
        _say(f"short values: nnz {c.nnz} -> {short}")
        vals = torch.full((c.nnz + 64,), 0x5A5A, dtype=torch.int16, device="cuda")     # guard patterns behind
        vals[:short] = torch.from_numpy(c.values[:short].view(np.int16)).cuda()
        guard = 4096
        buf = torch.full((rows * cols + 2 * guard,), POISON, dtype=torch.int16, device="cuda")
        out = buf[guard:guard + rows * cols].view(rows, cols)
        m = endor.DeviceMatrix(rows, cols, torch.from_numpy(c.bitmap).cuda(), vals[:short], short)
        endor.decompress(m, out=out)
        torch.cuda.synchronize()
        padded = np.zeros(c.nnz, np.uint16)
        padded[:short] = c.values[:short]
        assert np.array_equal(out.cpu().numpy().view(np.uint16), orc.decompress(rows, cols, c.bitmap, padded))
        assert bool((buf[:guard] == POISON).all()) and bool((buf[guard + rows * cols:] == POISON).all())


def test_foreign_offset_table_cannot_write_outside_the_output():
    """decompress_with_offsets with the table of ANOTHER bitmap of the same shape (a stale
    workspace): the result is meaningless but stays inside the output buffer, and a correct
    call afterwards is unaffected."""
    rows, cols = 1031, 2053
    a = _random_compressed(rows, cols, 0.9, seed=81)
    b = _random_compressed(rows, cols, 0.1, seed=82)
    ma, mb = endor.to_device(a), endor.to_device(b)
    ws_a, _ = endor.build_offsets(ma)
    ws_b, _ = endor.build_offsets(mb)
    guard = 8192
    for m, ws_wrong, ws_right, c in ((mb, ws_a, ws_b, b), (ma, ws_b, ws_a, a)):
        buf = torch.full((rows * cols + 2 * guard,), POISON, dtype=torch.int16, device="cuda")
        out = buf[guard:guard + rows * cols].view(rows, cols)
        endor.decompress_with_offsets(m, ws_wrong, out=out)
        torch.cuda.synchronize()
        assert bool((buf[:guard] == POISON).all()) and bool((buf[guard + rows * cols:] == POISON).all())
        endor.decompress_with_offsets(m, ws_right, out=out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint16), _expect(c))
        assert bool((buf[:guard] == POISON).all()) and bool((buf[guard + rows * cols:] == POISON).all())


def test_check_mode_reports_a_wrong_nnz_without_synchronising():
    shapes = [(64, 4096), (300, 4099), (0, 9), (1031, 2053), (5, 7)]
    cs = [_random_compressed(r, c, 0.5, seed=500 + i) for i, (r, c) in enumerate(shapes)]
    mats = [endor.to_device(c) for c in cs]
    outs, ws = endor.decompress_batch(mats)
    status = endor.check_batch(mats, ws)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0, 0, 0, 0]
    # the same bitmaps with one count off by one and one by many (values shortened accordingly)
    wrong = list(mats)
    wrong[1] = endor.DeviceMatrix(mats[1].rows, mats[1].cols, mats[1].bitmap, mats[1].values[:-1], mats[1].nnz - 1)
    wrong[3] = endor.DeviceMatrix(mats[3].rows, mats[3].cols, mats[3].bitmap, mats[3].values[:10], 10)
    outs, ws = endor.decompress_batch(wrong)
    status = endor.check_batch(wrong, ws)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 6, 0, 6, 0]
    # more matrices than one launch group
    many = [mats[4]] * 20 + [wrong[1]]
    ws = endor.build_offsets_batch(many)
    status = endor.check_batch(many, ws)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0] * 20 + [6]


def test_batch_mixing_aligned_and_unaligned_outputs():
    """One output of a batch that is not 16-byte aligned puts the whole launch group on the
    element-wise store path; every matrix must still be exact."""
    shapes = [(64, 4096), (300, 4099), (17, 33), (1031, 2053)]
    cs = [_random_compressed(r, c, 0.5, seed=600 + i) for i, (r, c) in enumerate(shapes)]
    mats = [endor.to_device(c) for c in cs]
    bufs, outs = [], []
    for i, c in enumerate(cs):
        off = [0, 1, 0, 3][i]                       # elements: 0 = aligned, 1 and 3 = 2 and 6 bytes off
        buf = torch.full((c.rows * c.cols + 16,), POISON, dtype=torch.int16, device="cuda")
        bufs.append((buf, off))
        outs.append(buf[off:off + c.rows * c.cols].view(c.rows, c.cols))
    endor.decompress_batch(mats, outs=outs)
    torch.cuda.synchronize()
    for c, o, (buf, off) in zip(cs, outs, bufs):
        assert np.array_equal(o.cpu().numpy().view(np.uint16), _expect(c))
        assert bool((buf[:off] == POISON).all()) and bool((buf[off + c.rows * c.cols:] == POISON).all())


def test_decompress_straight_from_pinned_host_memory():
    """Pinned host memory is addressable by the device, so the blob may stay on the host and
    the kernels fetch it across the link themselves (no staging copy)."""
    rows, cols = 1031, 2053
    c = endor.compress(synth.pruned_fp16(rows, cols, 0.5, seed=90))
    blob = endor.pin(c)
    nb = endor.bitmap_bytes(rows, cols)
    m = endor.DeviceMatrix(rows, cols, blob.keep[:nb], blob.keep[(nb + 255) // 256 * 256:].view(torch.int16), c.nnz)
    out = torch.full((rows, cols), POISON, dtype=torch.int16, device="cuda")
    ws = torch.empty(endor.workspace_bytes(rows, cols), dtype=torch.uint8, device="cuda")
    endor.decompress(m, out=out, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint16), _expect(c))


# ---------------------------------------------------------------------------
# the device entry points only enqueue kernels: they can be captured into a HIP graph
# ---------------------------------------------------------------------------
def test_decompress_batch_in_a_hip_graph_replays_correctly():
    shapes = [(300, 4099), (64, 4096), (1031, 2053)]
    cs = [endor.compress(synth.pruned_fp16(r, c, 0.5, seed=60 + i)) for i, (r, c) in enumerate(shapes)]
    mats = [endor.to_device(c) for c in cs]
    outs = [torch.full((c.rows, c.cols), POISON, dtype=torch.int16, device="cuda") for c in cs]
    ws = torch.empty(max(256, endor.batch_workspace_bytes(mats)), dtype=torch.uint8, device="cuda")
    expect = [orc.decompress(c.rows, c.cols, c.bitmap, c.values) for c in cs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        endor.decompress_batch(mats, outs=outs, workspace=ws, stream=side)     # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        endor.decompress_batch(mats, outs=outs, workspace=ws, stream=torch.cuda.current_stream())
    for rep in range(4):
        for o in outs:                      # eager work and a synchronisation between replays
            o.fill_(POISON)
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, expect):
            assert np.array_equal(o.cpu().numpy().view(np.uint16), e), f"replay {rep}"


def test_products_in_a_hip_graph_replay_correctly():
    """Both products captured into one graph (they allocate nothing and never synchronise) and
    replayed on fresh right-hand sides, with eager work and synchronisation between the replays."""
    rows, cols, nb = 300, 4099, 5
    w = synth.pruned_fp16(rows, cols, 0.5, seed=71)
    c = endor.compress(w)
    m = endor.to_device(c)
    tab, ro = endor.build_offsets(m, row_offsets=True)
    x = torch.zeros(cols, dtype=torch.float16, device="cuda")
    X = torch.zeros((nb, cols), dtype=torch.float16, device="cuda")
    y = torch.empty(rows, dtype=torch.float32, device="cuda")
    Y = torch.empty((nb, rows), dtype=torch.float32, device="cuda")
    sc = torch.empty(max(256, endor.gemm_scratch_bytes(rows, cols, nb)), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside capture
        endor.gemv_f16(m, ro, x, y=y, stream=side)
        endor.gemm_f16(m, tab, X, Y=Y, scratch=sc, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        endor.gemv_f16(m, ro, x, y=y, stream=torch.cuda.current_stream())
        endor.gemm_f16(m, tab, X, Y=Y, scratch=sc, stream=torch.cuda.current_stream())
    for rep in range(3):
        x16 = np.random.default_rng(100 + rep).standard_normal(cols).astype(np.float16)
        X16 = np.random.default_rng(200 + rep).standard_normal((nb, cols)).astype(np.float16)
        x.copy_(torch.from_numpy(x16.view(np.int16)).cuda().view(torch.float16))
        X.copy_(torch.from_numpy(X16.view(np.int16)).cuda().view(torch.float16))
        y.fill_(float("nan"))
        Y.fill_(float("nan"))
        sc.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref = orc.gemv_f16(rows, cols, c.bitmap, c.values, x16)
        assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - ref) <= _gemv_tolerance(w, x16, cols)), f"replay {rep}"
        refm = orc.gemm_f16(rows, cols, c.bitmap, c.values, X16)
        assert np.all(np.abs(Y.cpu().numpy().astype(np.float64) - refm) <= _gemm_tolerance(w, X16, cols)), f"replay {rep}"


# ---------------------------------------------------------------------------
# more than 2^32 elements / values: 64-bit indexing everywhere
# ---------------------------------------------------------------------------
def test_more_than_2_pow_32_values_all_bits_set():
    """Every bit 1 => the output is the value stream itself (the special case the oracle is
    pinned on), checked on the device.  N = nnz = 2^32 + 2^20."""
    rows, cols = 4097, 1 << 20
    n = rows * cols
    _say(f"2^32 test: all ones, n={n}")
    period = 65521                                     # prime, so no power-of-two shift goes unnoticed
    base = torch.arange(period, device="cuda").to(torch.int16)
    values = base.repeat((n + period - 1) // period)[:n].contiguous()
    bitmap = torch.full((endor.bitmap_bytes(rows, cols),), 0xFF, dtype=torch.uint8, device="cuda")
    m = endor.DeviceMatrix(rows, cols, bitmap, values, n)
    out = torch.full((rows, cols), POISON, dtype=torch.int16, device="cuda")
    endor.decompress(m, out=out)
    torch.cuda.synchronize()
    assert torch.equal(out.view(-1), values)
    _, ro = endor.build_offsets(m, row_offsets=True)
    torch.cuda.synchronize()
    assert torch.equal(ro, torch.arange(rows + 1, device="cuda", dtype=torch.int64) * cols)


def test_more_than_2_pow_32_elements_sparse_random():
    """N = 2^32 + 2^20, one element in eight kept at random.  Whole output against the oracle's
    Algorithm 2 and, slab by slab, against a mask-scatter built with torch on the device."""
    rows, cols = 4097, 1 << 20
    n = rows * cols
    _say(f"2^32 test: sparse random, n={n}")
    g = np.random.default_rng(2032)
    nbytes = n // 8
    bm = g.integers(0, 256, nbytes, dtype=np.uint8)
    bm &= g.integers(0, 256, nbytes, dtype=np.uint8)
    bm &= g.integers(0, 256, nbytes, dtype=np.uint8)
    per_row = np.bitwise_count(bm.view(np.uint64).reshape(rows, -1)).sum(axis=1, dtype=np.int64)
    row_offs = np.concatenate([[0], np.cumsum(per_row)]).astype(np.int64)
    nnz = int(row_offs[-1])
    values = g.integers(0, 1 << 16, nnz, dtype=np.uint16)
    c = endor.Compressed(rows, cols, bm, values, row_offs)
    m = endor.to_device(c)
    out = torch.full((rows, cols), POISON, dtype=torch.int16, device="cuda")
    endor.decompress(m, out=out)
    _, ro = endor.build_offsets(m, row_offsets=True)
    torch.cuda.synchronize()
    assert np.array_equal(ro.cpu().numpy(), row_offs)
    # the whole output, slab by slab, against torch's masked_scatter_
    shifts = torch.arange(8, device="cuda", dtype=torch.uint8)
    slab = 256
    for r0 in range(0, rows, slab):
        r1 = min(rows, r0 + slab)
        bytes_ = m.bitmap[r0 * cols // 8: r1 * cols // 8]
        mask = ((bytes_[:, None] >> shifts) & 1).bool().view(r1 - r0, cols)
        expect = torch.zeros((r1 - r0, cols), dtype=torch.int16, device="cuda")
        expect.masked_scatter_(mask, m.values[int(row_offs[r0]):int(row_offs[r1])])
        assert torch.equal(out[r0:r1], expect), f"rows {r0}..{r1}"
        del mask, expect
    # the whole output against the oracle's Algorithm 2 (rows split over the host threads)
    full = orc.decompress_threaded(rows, cols, bm, values, row_offs, 16)
    got_all = out.cpu().numpy().view(np.uint16)
    assert np.array_equal(got_all, full)
    del got_all
    sel = np.array([0, 1, 2047, 4094, 4095, 4096], np.int64)      # row 4096 starts at flat index 2^32
    expect = full[sel].copy()
    del full
    # and the row-subset entry point at the same offsets
    rsel = endor.decompress_rows(m, ro, torch.from_numpy(sel).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(rsel.cpu().numpy().view(np.uint16), expect)


def test_host_built_offset_table_serves_the_device():
    """The table built at compression time on the host, copied over, replaces the device pass."""
    rows, cols = 1031, 2053
    w = synth.pruned_fp16(rows, cols, 0.5, seed=91, row_skew=True)
    c = endor.compress(w)
    m = endor.to_device(c)
    host_ws = endor.build_offsets_host(c)
    dev_ws, _ = endor.build_offsets(m)
    torch.cuda.synchronize()
    nchunks = ((rows * cols + 4095) // 4096 + 255) // 256
    ct_bytes = (nchunks * 4 + 255) // 256 * 256
    dev = dev_ws.cpu().numpy()
    assert np.array_equal(dev[: nchunks * 4], host_ws[: nchunks * 4])
    assert np.array_equal(dev[ct_bytes: ct_bytes + nchunks * 257 * 4], host_ws[ct_bytes: ct_bytes + nchunks * 257 * 4])
    out = endor.decompress_with_offsets(m, torch.from_numpy(host_ws).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint16), orc.decompress(rows, cols, c.bitmap, c.values))


# ---------------------------------------------------------------------------
# column-subset decompression (the down-projection half of Section 4.2's selective load)
# ---------------------------------------------------------------------------
COL_SHAPES = [(40, 77), (5, 3), (64, 64), (33, 4096), (17, 4097), (9, 12345), (300, 8192), (50, 28672), (7, 28673),
              (3, 100000)]


@pytest.mark.parametrize("shape", COL_SHAPES, ids=str)
@pytest.mark.parametrize("wide", [True, False], ids=["fp16", "u8"])
def test_decompress_cols_matches_oracle(shape, wide):
    rows, cols = shape
    _say(f"cols case shape={shape} wide={wide}")
    if wide:
        w = synth.pruned_fp16(rows, cols, 0.5, seed=rows + cols, row_skew=True)
    else:
        w = synth.pruned_int8(rows, cols, 0.4, seed=rows + cols)
    c = endor.compress(w)
    m = endor.to_device(c)
    g = np.random.default_rng(cols)
    sel_np = np.concatenate([g.integers(0, cols, size=max(1, cols // 3)), [cols - 1, 0, 0]]).astype(np.int64)
    # the definition: Algorithm 2's output, then the selected columns of it
    expect = orc.decompress(rows, cols, c.bitmap, c.values)[:, sel_np]
    out = torch.full((rows, sel_np.size), 0x5A, dtype=torch.int16 if wide else torch.uint8, device="cuda")
    endor.decompress_cols(m, torch.from_numpy(c.row_offsets).cuda(), torch.from_numpy(sel_np).cuda(), out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(expect.dtype), expect)


def test_decompress_cols_out_of_range_index_is_skipped():
    rows, cols = 12, 5000
    w = synth.pruned_fp16(rows, cols, 0.5, seed=79)
    c = endor.compress(w)
    m = endor.to_device(c)
    sel_np = np.array([3, -1, cols, 4999], np.int64)
    out = torch.full((rows, 4), POISON, dtype=torch.int16, device="cuda")
    endor.decompress_cols(m, torch.from_numpy(c.row_offsets).cuda(), torch.from_numpy(sel_np).cuda(), out=out)
    torch.cuda.synchronize()
    host = out.cpu().numpy().view(np.uint16)
    assert np.array_equal(host[:, 0], w[:, 3]) and np.array_equal(host[:, 3], w[:, 4999])
    assert np.all(host[:, 1] == POISON) and np.all(host[:, 2] == POISON)


def test_decompress_cols_full_size_down_proj():
    """A tenth of the columns of a Llama2-70B down projection (8192 x 28672), device-built row offsets."""
    rows, cols = 8192, 28672
    _say("cols full size")
    w = synth.pruned_fp16(rows, cols, 0.5, seed=synth.seed_for(3, 6))
    c = endor.compress(w)
    m = endor.to_device(c)
    _, ro = endor.build_offsets(m, row_offsets=True)
    sel_np = np.sort(np.random.default_rng(6).choice(cols, size=cols // 10, replace=False)).astype(np.int64)
    out = endor.decompress_cols(m, ro, torch.from_numpy(sel_np).cuda())
    torch.cuda.synchronize()
    expect = orc.decompress(rows, cols, c.bitmap, c.values)
    assert np.array_equal(expect, w)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), expect[:, sel_np])


# ---------------------------------------------------------------------------
# seeded sweep: random shapes and densities through every entry point.  The densities sit on both
# sides of the points where the host switches kernels (one element in five for the store-dominated
# expander, nine in sixteen for the row kernel's staging area) and at the two ends.
# ---------------------------------------------------------------------------
SWEEP_KEEPS = [0.0, 0.02, 0.1, 0.19, 0.21, 0.5, 0.55, 0.58, 0.9, 1.0]


@pytest.mark.parametrize("case", range(100))
def test_seeded_sweep_through_every_entry_point(case):
    g = np.random.default_rng(1000 + case)
    rows = int(g.integers(1, 200))
    cols = int(g.choice([g.integers(1, 300), g.integers(4000, 4200), g.integers(8100, 8300), g.integers(1, 20000)]))
    keep = SWEEP_KEEPS[case % len(SWEEP_KEEPS)]
    wide = bool(g.integers(0, 2))
    _say(f"sweep case={case} shape=({rows}, {cols}) keep={keep} wide={wide}")
    if wide:
        w = g.integers(1, 1 << 16, size=(rows, cols), dtype=np.uint32).astype(np.uint16)
    else:
        w = g.integers(1, 256, size=(rows, cols), dtype=np.uint16).astype(np.uint8)
    w[g.random((rows, cols)) >= keep] = 0
    dt = torch.int16 if wide else torch.uint8
    c = endor.compress(w)
    b, v, r = orc.compress(w)
    assert np.array_equal(c.bitmap[: b.size], b) and np.array_equal(c.values, v) and np.array_equal(c.row_offsets, r)
    m = endor.to_device(c)
    ro = torch.from_numpy(c.row_offsets).cuda()

    # Algorithm 2
    expect = orc.decompress(rows, cols, c.bitmap, c.values)
    assert np.array_equal(expect, w.view(expect.dtype))
    out = torch.full((rows, cols), 0x5A, dtype=dt, device="cuda")
    endor.decompress(m, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(expect.dtype), expect)

    # selected rows and columns
    rsel = g.integers(0, rows, size=max(1, rows // 3)).astype(np.int64)
    got = endor.decompress_rows(m, ro, torch.from_numpy(rsel).cuda())
    csel = g.integers(0, cols, size=max(1, cols // 5)).astype(np.int64)
    gotc = torch.full((rows, csel.size), 0x5A, dtype=dt, device="cuda")
    endor.decompress_cols(m, ro, torch.from_numpy(csel).cuda(), out=gotc)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(expect.dtype), expect[rsel])
    assert np.array_equal(gotc.cpu().numpy().view(expect.dtype), expect[:, csel])

    # Algorithm 1 on the device
    dm, _, dro = endor.compress_device(torch.from_numpy(w.view(np.int16) if wide else w).cuda(), row_offsets=True)
    torch.cuda.synchronize()
    assert dm.nnz == v.size
    assert np.array_equal(dm.bitmap.cpu().numpy()[: b.size], b)
    assert np.array_equal(dm.values.cpu().numpy().view(v.dtype), v)
    assert np.array_equal(dro.cpu().numpy(), r)

    # the products (fp16 only): values reinterpreted as fp16, non-finite patterns cleared first
    if wide:
        wf = w.copy()
        wf[(wf & 0x7C00) == 0x7C00] = 0x3C00
        cf = endor.compress(wf)
        mf = endor.to_device(cf)
        rof = torch.from_numpy(cf.row_offsets).cuda()
        x16 = g.standard_normal(cols).astype(np.float16)
        y = endor.gemv_f16(mf, rof, torch.from_numpy(x16).cuda())
        torch.cuda.synchronize()
        ref = orc.gemv_f16(rows, cols, cf.bitmap, cf.values, x16)
        assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - ref) <= _gemv_tolerance(wf, x16, cols))
        nb = int(g.integers(1, 17))
        X16 = g.standard_normal((nb, cols)).astype(np.float16)
        gotY = _gpu_gemm(cf, X16)
        refY = orc.gemm_f16(rows, cols, cf.bitmap, cf.values, X16)
        assert np.all(np.abs(gotY - refY) <= _gemm_tolerance(wf, X16, cols))


def test_concurrent_calls_on_two_streams_with_distinct_workspaces():
    """The library keeps no state between calls: two host threads, two streams, two workspaces."""
    import threading
    cs = [endor.compress(synth.pruned_fp16(700, 4099, 0.5, seed=70 + i)) for i in range(2)]
    mats = [endor.to_device(c) for c in cs]
    outs = [torch.full((c.rows, c.cols), POISON, dtype=torch.int16, device="cuda") for c in cs]
    wss = [torch.empty(max(256, endor.workspace_bytes(c.rows, c.cols)), dtype=torch.uint8, device="cuda") for c in cs]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    errors = []

    def work(i):
        try:
            for _ in range(20):
                endor.decompress(mats[i], out=outs[i], workspace=wss[i], stream=streams[i])
        except Exception as e:  # pragma: no cover
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors
    for c, o in zip(cs, outs):
        assert np.array_equal(o.cpu().numpy().view(np.uint16), orc.decompress(c.rows, c.cols, c.bitmap, c.values))
