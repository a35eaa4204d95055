#!/usr/bin/env python3
"""Benchmark of the Endor decompression hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: build the
tile offset table from the bitmaps and expand every matrix of the workload into
its dense fp16 form (endor_decompress_batch), inputs already resident in HBM.

Prints ONE JSON line.  Its headline (`value`, `roofline`, `cpu_baseline`) is the
Llama2-70B decoder layer; beside it the same line carries
  configs   every other benchmark configuration, measured the same way: the OPT-66B
            attention projections and FFN pair, the FFN pair's host-to-device transfer
            alone and overlapped with decompression, the down_proj keep sweep and the
            row-skewed variant, the 1024x1024 case
  extras    the entry points beyond plain decompression (8-bit values, row / column
            subsets, device-side compressor, fused products), each against its own
            algorithmic byte count
  ceilings  plain streaming kernels (write, read, copy, the 1.125:2 mix, and the mixes of
            the other densities and of 8-bit values) on the same box: what the memory
            system delivers for traffic of this shape
`--workload X --only` restricts the run to one workload (the form the rocprofv3
summaries under profiles/ are made with).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak

WORKLOADS = {
    # name: (synth config index, description)
    "llama2_70b_layer": (3, "one Llama2-70B decoder layer: q,o 8192x8192; k,v 1024x8192; "
                            "gate,up 28672x8192; down 8192x28672; fp16, keep 0.5"),
    "opt66b_attn": (1, "OPT-66B attention projections: 4 x 9216x9216 fp16, keep 0.5"),
    "opt66b_ffn": (2, "OPT-66B FFN pair: 36864x9216 and 9216x36864 fp16, keep 0.5"),
    "down_proj": (4, "Llama2-70B down_proj 8192x28672 fp16"),
    "1024sq": (0, "single 1024x1024 fp16 matrix, keep 0.5"),
}


def _events(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def make_inputs(endor, synth, workload, keep, row_skew, variant=0):
    cfg, _ = WORKLOADS[workload]
    host = []
    for i, (_, rows, cols) in enumerate(synth.CONFIGS[cfg]):
        w = synth.pruned_fp16(rows, cols, keep, seed=synth.seed_for(cfg, i, variant), row_skew=row_skew)
        host.append(endor.compress(w, want_row_offsets=True))
        del w
    return host


class Resident:
    """A workload resident in HBM: `rotate` device copies of the compressed input (so that no
    step finds its input in a cache left by the step before), one set of outputs."""

    def __init__(self, endor, torch, host, rotate):
        self.endor, self.torch, self.host = endor, torch, host
        self.rotate = max(1, rotate)
        self.sets = [[endor.to_device(c) for c in host] for _ in range(self.rotate)]
        self.outs = [torch.empty((c.rows, c.cols), dtype=torch.int16, device="cuda") for c in host]
        ws_bytes = max(256, endor.batch_workspace_bytes(self.sets[0]))
        self.workspaces = [torch.empty(ws_bytes, dtype=torch.uint8, device="cuda") for _ in range(self.rotate)]
        self.stream = torch.cuda.current_stream()
        self.turn = 0
        self.elements = sum(c.rows * c.cols for c in host)
        self.nnz = sum(c.nnz for c in host)
        self.dense_bytes = 2 * self.elements
        self.alg_bytes = 2 * self.elements + sum((c.rows * c.cols + 7) // 8 for c in host) + 2 * self.nnz

    def step(self):
        k = self.turn = (self.turn + 1) % self.rotate
        self.endor.decompress_batch(self.sets[k], outs=self.outs, workspace=self.workspaces[k], stream=self.stream)

    def expand_only(self):
        k = self.turn = (self.turn + 1) % self.rotate
        self.endor.decompress_batch_with_offsets(self.sets[k], self.workspaces[k], outs=self.outs, stream=self.stream)

    def build_tables(self):
        for k in range(self.rotate):
            self.endor.build_offsets_batch(self.sets[k], workspace=self.workspaces[k], stream=self.stream)

    def time_steps(self, steps, warmup):
        """W warm-up steps, then exactly K timed steps.  Returns (wall ms/step, event ms/step)."""
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        ev0, ev1 = _events(torch)
        t0 = time.perf_counter()
        ev0.record(self.stream)
        for _ in range(steps):
            self.step()
        ev1.record(self.stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, ev0.elapsed_time(ev1) / steps

    def time_expand(self, reps, warmup):
        """The expand kernel alone, tables already in the workspaces (the *_with_offsets path: a
        table built once, or shipped with the blob).  Returns (average over back-to-back launches,
        sorted single-launch durations), HIP events on the launch stream."""
        torch = self.torch
        self.build_tables()
        for _ in range(max(2, warmup)):
            self.expand_only()
        torch.cuda.synchronize()
        evs = [_events(torch) for _ in range(reps)]
        for a, b in evs:
            a.record(self.stream)
            self.expand_only()
            b.record(self.stream)
        torch.cuda.synchronize()
        per = sorted(a.elapsed_time(b) for a, b in evs)
        a, b = _events(torch)
        a.record(self.stream)
        for _ in range(reps):
            self.expand_only()
        b.record(self.stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps, per


def config_entry(endor, synth, torch, workload, keep, row_skew, steps, warmup, rotate):
    host = make_inputs(endor, synth, workload, keep, row_skew)
    r = Resident(endor, torch, host, rotate)
    wall_ms, ev_ms = r.time_steps(steps, warmup)
    exp_ms, _ = r.time_expand(max(10, steps), warmup)
    entry = {
        "workload": workload, "keep": keep, "row_skew": row_skew,
        "ms_per_step": round(wall_ms, 4), "ms_per_step_events": round(ev_ms, 4),
        "dense_GBps": round(r.dense_bytes / wall_ms / 1e6, 1),
        "algorithmic_bytes": r.alg_bytes,
        "hbm_frac_whole_path": round(r.alg_bytes / wall_ms / 1e6 / HBM_PEAK_GBS, 4),
        "ms_expand_with_offsets": round(exp_ms, 4),
        "hbm_frac_with_offsets": round(r.alg_bytes / exp_ms / 1e6 / HBM_PEAK_GBS, 4),
    }
    return entry, host, r


def overlap_leg(endor, torch, host, outs, nblocks, reps=5):
    """Pinned host -> device copy of the compressed blobs, alone and overlapped with
    decompression (two streams, three staging slots).  Link-bound by design: these figures
    are reported beside `value`, never as it.  Every timed call is bracketed by a device
    synchronisation, so no call's tail hides under the next call's copies."""
    eb = host[0].values.dtype.itemsize
    whole = [endor.pin(c) for c in host]
    blocks, block_outs = [], []
    for c, o in zip(host, outs):
        for b in endor.row_blocks(c, nblocks):
            blocks.append(b)
            block_outs.append(o[b.row_begin:b.row_begin + b.rows])
    s_copy, s_copy2, s_comp = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    compressed_bytes = sum(c.bitmap.nbytes + c.values.nbytes for c in host)
    dense_bytes = sum(eb * c.rows * c.cols for c in host)
    pipe = endor.Pipeline.for_blobs(whole + blocks, s_copy, s_comp)
    pipe2 = endor.Pipeline.for_blobs(whole + blocks, s_copy, s_comp, copy_stream2=s_copy2)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        best, total = 1e9, 0.0
        for _ in range(reps):
            t = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t
            best, total = min(best, dt), total + dt
        return total / reps * 1e3, best * 1e3

    dev = [torch.empty(b.keep.numel(), dtype=torch.uint8, device="cuda") for b in whole]
    dense_pinned = [torch.empty((c.rows, c.cols), dtype=o.dtype, pin_memory=True) for c, o in zip(host, outs)]

    def copy_only():
        with torch.cuda.stream(s_copy):
            for d, b in zip(dev, whole):
                d.copy_(b.keep, non_blocking=True)

    def dense_copy():   # what the uncompressed baseline would move over the same link
        with torch.cuda.stream(s_copy):
            for o, hp in zip(outs, dense_pinned):
                o.copy_(hp, non_blocking=True)

    vdt = torch.int16 if eb == 2 else torch.uint8
    mats = []
    for c, d in zip(host, dev):
        nb = c.bitmap.size
        mats.append(endor.DeviceMatrix(c.rows, c.cols, d[:nb], d[(nb + 255) // 256 * 256:].view(vdt), c.nnz))
    ws = torch.empty(max(256, endor.batch_workspace_bytes(mats)), dtype=torch.uint8, device="cuda")
    copy_only()
    torch.cuda.synchronize()
    ms_copy, ms_copy_min = timed(copy_only)
    ms_dense_copy, _ = timed(dense_copy)
    ms_dec, _ = timed(lambda: endor.decompress_batch(mats, outs=outs, workspace=ws, stream=s_comp))
    one_block = max(blocks, key=lambda b: b.rows * b.cols)
    ms_pipe_whole, ms_pipe_whole_min = timed(lambda: pipe.run(whole, outs))
    ms_pipe_blocks, ms_pipe_blocks_min = timed(lambda: pipe.run(blocks, block_outs))
    ms_pipe2_whole, _ = timed(lambda: pipe2.run(whole, outs))
    ms_pipe2_blocks, ms_pipe2_blocks_min = timed(lambda: pipe2.run(blocks, block_outs))
    pipe.close()
    pipe2.close()
    return {
        "elem_bytes": eb, "compressed_bytes": compressed_bytes, "dense_bytes": dense_bytes,
        "ms_decompress_alone": round(ms_dec, 3),
        "ms_h2d_copy_compressed_alone": round(ms_copy, 3),
        "ms_h2d_copy_dense_alone": round(ms_dense_copy, 3),
        "h2d_GBps": round(compressed_bytes / ms_copy / 1e6, 1),
        "ms_pipeline_whole_matrices": round(ms_pipe_whole, 3),
        "ms_pipeline_row_blocks": round(ms_pipe_blocks, 3),
        "ms_pipeline_whole_matrices_two_copy_streams": round(ms_pipe2_whole, 3),
        "ms_pipeline_row_blocks_two_copy_streams": round(ms_pipe2_blocks, 3),
        "min_ms": {"copy": round(ms_copy_min, 3), "pipeline_whole": round(ms_pipe_whole_min, 3),
                   "pipeline_row_blocks": round(ms_pipe_blocks_min, 3),
                   "pipeline_row_blocks_two_copy_streams": round(ms_pipe2_blocks_min, 3)},
        "row_blocks_per_matrix": nblocks, "blobs": len(blocks),
        "largest_block_fraction": round(one_block.rows * one_block.cols * eb / dense_bytes, 4),
        "sum_copy_plus_decompress_ms": round(ms_copy + ms_dec, 3),
        "dense_GBps_pcie_inclusive": round(dense_bytes / min(ms_pipe_whole, ms_pipe_blocks, ms_pipe2_blocks) / 1e6, 1),
        "speedup_vs_dense_copy": round(ms_dense_copy / min(ms_pipe_whole, ms_pipe_blocks, ms_pipe2_blocks), 3),
    }


def extras_leg(endor, synth, torch, np, host, shapes, cfg, keep):
    """Timings of the entry points beyond plain decompression, each with its own
    algorithmic byte count (what the operation must move) against the 8 TB/s HBM peak."""
    big = max(range(len(host)), key=lambda i: host[i].rows * host[i].cols)
    c = host[big]
    rows, cols, n, nnz = c.rows, c.cols, c.rows * c.cols, c.nnz
    m = endor.to_device(c)
    ro = torch.from_numpy(c.row_offsets).cuda()
    stream = torch.cuda.current_stream()
    out = []

    def timed(name, fn, alg_bytes, reps=20, note="", matrix=None):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = _events(torch)
        a.record(stream)
        for _ in range(reps):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        gbs = alg_bytes / ms / 1e6
        out.append({"name": name, "matrix": matrix or [shapes[big][0], rows, cols], "ms": round(ms, 4),
                    "algorithmic_bytes": int(alg_bytes), "GB/s": round(gbs, 1),
                    "hbm_frac": round(gbs / HBM_PEAK_GBS, 4), "note": note})

    # 8-bit variant, whole path (same bitmap density, one byte per value)
    w8 = synth.pruned_int8(rows, cols, keep, seed=synth.seed_for(cfg, big, 8))
    c8 = endor.compress(w8, want_row_offsets=False)
    m8 = endor.to_device(c8)
    o8 = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
    ws8 = torch.empty(max(256, endor.workspace_bytes(rows, cols)), dtype=torch.uint8, device="cuda")
    timed("decompress_u8", lambda: endor.decompress(m8, out=o8, workspace=ws8), n + n // 8 + c8.nnz,
          note="endor_decompress_u8: offsets + expand, 1 + 1/8 + p bytes per element")
    endor.build_offsets(m8, workspace=ws8)
    timed("decompress_u8_with_offsets", lambda: endor.decompress_with_offsets(m8, ws8, out=o8), n + n // 8 + c8.nnz,
          note="endor_decompress_u8_with_offsets: the expand kernel alone (table built once or shipped with the blob)")
    del w8, c8, m8, o8

    # row subset: a tenth of the rows, sorted
    sel_np = np.sort(np.random.default_rng(5).choice(rows, size=max(1, rows // 10), replace=False)).astype(np.int64)
    sel = torch.from_numpy(sel_np).cuda()
    osel = torch.empty((sel_np.size, cols), dtype=torch.int16, device="cuda")
    nnz_sel = int((c.row_offsets[sel_np + 1] - c.row_offsets[sel_np]).sum())
    timed("decompress_rows_10pct", lambda: endor.decompress_rows(m, ro, sel, out=osel),
          2 * sel_np.size * cols + sel_np.size * cols // 8 + 2 * nnz_sel,
          note="endor_decompress_rows on a sorted random tenth of the rows; bytes of the selected rows only")

    # column subset on the widest matrix (the down projection): a tenth of the columns, sorted
    wide = max(range(len(host)), key=lambda i: (host[i].cols, host[i].rows))
    cw = host[wide]
    mw = endor.to_device(cw) if wide != big else m
    row = torch.from_numpy(cw.row_offsets).cuda()
    csel_np = np.sort(np.random.default_rng(6).choice(cw.cols, size=max(1, cw.cols // 10), replace=False)).astype(np.int64)
    csel = torch.from_numpy(csel_np).cuda()
    ocol = torch.empty((cw.rows, csel_np.size), dtype=torch.int16, device="cuda")
    frac_sel = csel_np.size / cw.cols
    lines_touched = 1.0 - (1.0 - frac_sel) ** 32      # a 64-byte line holds 32 values, each selected w.p. frac_sel
    timed("decompress_cols_10pct", lambda: endor.decompress_cols(mw, row, csel, out=ocol),
          cw.rows * cw.cols // 8 + int(2 * cw.nnz * lines_touched) + 2 * cw.rows * csel_np.size,
          matrix=[shapes[wide][0], cw.rows, cw.cols],
          note="endor_decompress_cols on a sorted random tenth of the columns; algorithmic = bitmap + the 64-byte "
               "lines of the value stream that hold a selected value (%.1f %% of them) + output" % (100 * lines_touched))
    del ocol

    # device-side compressor: dense -> bitmap + values (+ table)
    dense = endor.decompress(m)
    vals = torch.empty(n, dtype=torch.int16, device="cuda")
    bm = torch.empty(endor.bitmap_bytes(rows, cols), dtype=torch.uint8, device="cuda")
    ws = torch.empty(max(256, endor.workspace_bytes(rows, cols)), dtype=torch.uint8, device="cuda")
    nnz_dev = torch.zeros(1, dtype=torch.int64, device="cuda")
    L = endor.lib()

    def comp():
        st = L.endor_compress_device(rows, cols, dense.data_ptr(), bm.data_ptr(), vals.data_ptr(), n, ws.data_ptr(),
                                     ws.numel(), None, nnz_dev.data_ptr(), stream.cuda_stream)
        assert st == 0
    timed("compress_device", comp, 2 * n + n // 8 + 2 * nnz,
          note="endor_compress_device; algorithmic = one read of dense + bitmap + values written")
    assert int(nnz_dev.item()) == nnz
    del dense, vals, bm

    # fused consumers
    x = torch.randn(cols, device="cuda").to(torch.float16)
    y = torch.empty(rows, dtype=torch.float32, device="cuda")
    timed("gemv_f16", lambda: endor.gemv_f16(m, ro, x, y=y), n // 8 + 2 * nnz + 8 * (rows + 1) + 2 * cols + 4 * rows,
          note="endor_gemv_f16: bitmap + values + row offsets + x read, y written; a dense fp16 GEMV "
               "would read %d bytes" % (2 * n))
    # small-batch product on the matrix cores: one expansion of W shared by nb right-hand sides
    tab, _ = endor.build_offsets(m)
    for nb in (1, 16):
        X = torch.randn((nb, cols), device="cuda").to(torch.float16)
        Y = torch.empty((nb, rows), dtype=torch.float32, device="cuda")
        sc = torch.empty(max(256, endor.gemm_scratch_bytes(rows, cols, nb)), dtype=torch.uint8, device="cuda")
        timed("gemm_f16_nb%d" % nb, lambda: endor.gemm_f16(m, tab, X, Y=Y, scratch=sc),
              n // 8 + 2 * nnz + 2 * nb * cols + 4 * nb * rows,
              note="endor_gemm_f16 with %d right-hand side(s): bitmap + values + X read, Y written; %.1f GFLOP per call"
                   % (nb, 2e-9 * n * nb))
    # what the fused product replaces: decompress, then the library's dense fp16 matrix-vector product
    dense16 = endor.decompress(m).view(torch.float16)
    yd = torch.empty(rows, dtype=torch.float16, device="cuda")
    ws1 = torch.empty(max(256, endor.workspace_bytes(rows, cols)), dtype=torch.uint8, device="cuda")
    dbuf = torch.empty((rows, cols), dtype=torch.int16, device="cuda")
    timed("reference_dense_mv", lambda: torch.mv(dense16, x, out=yd), 2 * n + 2 * cols + 2 * rows,
          note="torch.mv on the already decompressed fp16 matrix (the vendor GEMV), for comparison")
    timed("reference_decompress_then_mv",
          lambda: (endor.decompress(m, out=dbuf, workspace=ws1), torch.mv(dbuf.view(torch.float16), x, out=yd)),
          2 * n + n // 8 + 2 * nnz + 2 * n, note="endor_decompress followed by torch.mv: the unfused path")
    X16 = torch.randn((16, cols), device="cuda").to(torch.float16)
    Y16 = torch.empty((16, rows), dtype=torch.float16, device="cuda")
    timed("reference_dense_mm_nb16", lambda: torch.matmul(X16, dense16.t(), out=Y16), 2 * n + 2 * 16 * cols + 2 * 16 * rows,
          note="torch.matmul of 16 right-hand sides with the already decompressed fp16 matrix (the vendor GEMM)")
    return out


def ceilings_leg(torch, nbytes=1 << 30, reps=10):
    """The streaming yardstick: plain kernels from libendor_probe.so, one 16-byte unit per
    thread, timed with HIP events on the launch stream."""
    path = os.path.join(ROOT, "paper_2406_11674_amd", "libendor_probe.so")
    if not os.path.exists(path):
        return None
    P = ctypes.CDLL(path)
    P.endor_probe_stream.restype = ctypes.c_int
    P.endor_probe_stream.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                     ctypes.c_void_p, ctypes.c_void_p]
    src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()
    res = {"bytes_per_launch": nbytes}
    for kind, name, moved in ((0, "write", nbytes), (1, "read", nbytes), (2, "copy", 2 * nbytes),
                              (3, "mix_1.125r_2w", nbytes + nbytes * 9 // 16)):
        def fn():
            rc = P.endor_probe_stream(kind, src.data_ptr(), dst.data_ptr(), nbytes, sink.data_ptr(), stream.cuda_stream)
            assert rc == 0
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = _events(torch)
        a.record(stream)
        for _ in range(reps):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        res[name] = {"ms": round(ms, 4), "GB/s": round(moved / ms / 1e6, 1),
                     "hbm_frac": round(moved / ms / 1e6 / HBM_PEAK_GBS, 4)}
    # the read : write ratio of the other configurations, in 16-byte units read per 256 written
    # (per element: 1/8 byte of bitmap + keep * E bytes of values read, E bytes written)
    if hasattr(P, "endor_probe_mix"):
        P.endor_probe_mix.restype = ctypes.c_int
        P.endor_probe_mix.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                      ctypes.c_void_p, ctypes.c_void_p]
        res["mix_by_ratio"] = {}
        for name, e, keep in (("fp16_keep_0.1", 2, 0.1), ("fp16_keep_0.3", 2, 0.3), ("fp16_keep_0.5", 2, 0.5),
                              ("fp16_keep_0.7", 2, 0.7), ("u8_keep_0.5", 1, 0.5)):
            k = int(round(256 * (0.125 + keep * e) / e))
            def fn():
                rc = P.endor_probe_mix(k, src.data_ptr(), dst.data_ptr(), nbytes, sink.data_ptr(), stream.cuda_stream)
                assert rc == 0
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            a, b = _events(torch)
            a.record(stream)
            for _ in range(reps):
                fn()
            b.record(stream)
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / reps
            moved = nbytes + nbytes * k // 256
            res["mix_by_ratio"][name] = {"reads_per_256_written": k, "ms": round(ms, 4),
                                         "GB/s": round(moved / ms / 1e6, 1),
                                         "hbm_frac": round(moved / ms / 1e6 / HBM_PEAK_GBS, 4)}
    return res


def cpu_baseline(np, host, shapes, seconds):
    """The oracle's Algorithm 2, rows split over the host threads (the analogue of the paper's
    multi-core CPU decompression, Section 5.1), on a bounded sample: whole matrices of the
    workload, largest first, until the budget is spent.  Output buffers are allocated and
    touched before the clock starts."""
    from oracle import endor_oracle as orc
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "1024")))
    order = sorted(range(len(host)), key=lambda i: -host[i].rows * host[i].cols)
    bufs = {}
    for i in order:
        key = (host[i].rows, host[i].cols)
        if key not in bufs:
            bufs[key] = np.zeros(key, np.uint16)
    c0 = host[order[-1]]
    orc.decompress_threaded(c0.rows, c0.cols, c0.bitmap, c0.values, c0.row_offsets, cores,
                            out=bufs[(c0.rows, c0.cols)])       # load the library, start-up costs
    done_bytes, spent, used, passes = 0, 0.0, [], 0
    while spent * cores <= seconds and passes < 20:
        passes += 1
        for i in order:
            c = host[i]
            t = time.perf_counter()
            orc.decompress_threaded(c.rows, c.cols, c.bitmap, c.values, c.row_offsets, cores,
                                    out=bufs[(c.rows, c.cols)])
            spent += time.perf_counter() - t
            done_bytes += 2 * c.rows * c.cols
            used.append(shapes[i][0])
            if spent * cores > seconds:
                break
    return {
        "value": round(done_bytes / spent / 1e9, 3),
        "unit": "GB/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"Algorithm 2 oracle, rows split over {cores} threads, {len(used)} whole matrices of the "
                  f"workload, largest first, cycling ({done_bytes} dense bytes in {spent:.2f} s wall; output "
                  f"buffers touched beforehand)",
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama2_70b_layer", choices=sorted(WORKLOADS))
    ap.add_argument("--keep", type=float, default=0.5)
    ap.add_argument("--row-skew", action="store_true")
    ap.add_argument("--only", action="store_true",
                    help="measure the chosen workload only: no configs / extras / ceilings / CPU baseline")
    ap.add_argument("--no-configs", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="rough CPU-baseline budget (core-seconds)")
    ap.add_argument("--rotate", type=int, default=3,
                    help="number of distinct device copies of the compressed input that the timed steps "
                         "cycle through, so that no step finds its input in a cache left by the one before")
    ap.add_argument("--overlap", action="store_true",
                    help="with --only: also time the pinned host-to-device copy, alone and pipelined with "
                         "decompression on a second stream")
    ap.add_argument("--overlap-blocks", type=int, default=4, help="row blocks per matrix in the pipeline")
    ap.add_argument("--extras", action="store_true", help="with --only: also time the widened entry points")
    ap.add_argument("--ceilings", action="store_true", help="with --only: also run the streaming yardstick kernels")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device-to-device copy of known size (a reference for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no cross-GPU step); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2406_11674_amd as endor
    from paper_2406_11674_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    endor.lib()  # fail loudly if the library is not built
    torch.cuda.set_device(0)
    full = not args.only

    cfg, desc = WORKLOADS[args.workload]
    shapes = synth.CONFIGS[cfg]
    t_gen = time.time()
    host = make_inputs(endor, synth, args.workload, args.keep, args.row_skew)
    t_gen = time.time() - t_gen
    res = Resident(endor, torch, host, args.rotate)

    if args.calibrate_copy:
        # a plain copy of the largest output into a same-sized buffer: reads and
        # writes exactly 2*rows*cols bytes, whatever the counters say about it
        big = max(range(len(res.outs)), key=lambda i: res.outs[i].numel())
        ref = torch.empty_like(res.outs[big])
        ref.copy_(res.outs[big])
        torch.cuda.synchronize()
        print(f"calibration copy: {2 * res.outs[big].numel()} bytes read and written", file=sys.stderr, flush=True)
        del ref

    # ---- whole path: W warm-up steps, then exactly K timed steps
    wall_ms, ev_ms = res.time_steps(args.steps, args.warmup)
    ms_per_step = wall_ms
    dense_gbs = res.dense_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- dominant kernel alone: per-launch duration from HIP events on the launch stream
    expand_ms, per = res.time_expand(max(10, args.steps), args.warmup)
    achieved = res.alg_bytes / (expand_ms * 1e-3) / 1e9

    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{args.workload}.json")
    if os.path.exists(tpath) and args.keep == 0.5 and not args.row_skew:
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")
        traffic_src = ("constant read from profiles/traffic_%s.json (rocprofv3 FETCH_SIZE + WRITE_SIZE runs of "
                       "this command), not measured in this run" % args.workload)

    result = {
        "metric": "decompress throughput, dense GB/s and % of HBM roofline, Llama2-70B layer"
                  if args.workload == "llama2_70b_layer" else f"decompress throughput, dense GB/s, {args.workload}",
        "value": round(dense_gbs, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u16",
        "data": "synthetic",
        "config": {
            "workload": args.workload, "description": desc, "keep": args.keep, "row_skew": args.row_skew,
            "matrices": [[n, r, c] for n, r, c in shapes], "elements": res.elements, "nnz": res.nnz,
            "dense_bytes": res.dense_bytes, "algorithmic_bytes": res.alg_bytes, "input_sets_rotated": res.rotate,
            "launch": "endor_decompress_batch: tile-offset kernel + expand kernel, one pair for the whole batch",
        },
        "path": {
            "ms_per_step_events": round(ev_ms, 4),
            "hbm_frac_whole_path": round(res.alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "hbm_frac_with_offsets": round(achieved / HBM_PEAK_GBS, 4),
            "with_offsets_note": "the table built once or shipped with the blob (endor_decompress_batch_with_offsets): "
                                 "the expand kernel alone",
            "input_generation_s": round(t_gen, 1),
        },
        "roofline": {
            "kernel": "endor_expand_kernel",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "traffic_source": traffic_src,
            "bytes_per_launch": res.alg_bytes,
            "avg_launch_ms": round(expand_ms, 4),
            "median_single_launch_ms": round(per[len(per) // 2], 4),
            "min_single_launch_ms": round(per[0], 4),
        },
    }

    if args.only and args.overlap:
        result["overlap"] = overlap_leg(endor, torch, host, res.outs, args.overlap_blocks)
    if (args.only and args.extras) or (full and not args.no_extras):
        result["extras"] = extras_leg(endor, synth, torch, np, host, shapes, cfg, args.keep)
    if full and not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(np, host, shapes, args.cpu_seconds)
    del res, host
    torch.cuda.empty_cache()

    if full and not args.no_configs:
        csteps, cwarm = min(args.steps, 20), min(args.warmup, 3)
        configs = []
        for wl, keep, skew in (("1024sq", 0.5, False), ("opt66b_attn", 0.5, False), ("opt66b_ffn", 0.5, False),
                               ("down_proj", 0.1, False), ("down_proj", 0.3, False), ("down_proj", 0.5, False),
                               ("down_proj", 0.7, False), ("down_proj", 0.5, True)):
            entry, chost, cres = config_entry(endor, synth, torch, wl, keep, skew, csteps, cwarm, args.rotate)
            if wl == "opt66b_ffn":
                entry["overlap"] = overlap_leg(endor, torch, chost, cres.outs, args.overlap_blocks)
            configs.append(entry)
            del chost, cres
            torch.cuda.empty_cache()
        # the 8-bit transfer (Sections 4.2 and 5.4): 9216x36864 int8 codes through the same pipeline
        w8 = synth.pruned_int8(9216, 36864, 0.5, seed=synth.seed_for(2, 1, 8))
        c8 = endor.compress(w8)
        del w8
        o8 = [torch.empty((c8.rows, c8.cols), dtype=torch.uint8, device="cuda")]
        configs.append({"workload": "opt66b_fc2_int8", "keep": 0.5, "row_skew": False,
                        "overlap": overlap_leg(endor, torch, [c8], o8, args.overlap_blocks)})
        del c8, o8
        torch.cuda.empty_cache()
        result["configs"] = configs
    if (full and not args.no_ceilings) or (args.only and args.ceilings):
        result["ceilings"] = ceilings_leg(torch)

    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
