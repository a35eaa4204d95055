#!/usr/bin/env python3
"""Benchmark of the Endor decompression hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: build the
tile offset table from the bitmaps and expand every matrix of the workload into
its dense fp16 form (endor_decompress_batch), inputs already resident in HBM.

Prints ONE JSON line: dense GB/s produced (whole path), the roofline figures of
the dominant kernel (the expand kernel, timed alone with HIP events on the stream
it runs on) and the CPU oracle timed on the host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
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


def extras_leg(endor, synth, torch, np, host, shapes, cfg, args):
    """Timings of the entry points beyond plain decompression, each with its own
    algorithmic byte count (what the operation must move) against the 8 TB/s HBM peak."""
    big = max(range(len(host)), key=lambda i: host[i].rows * host[i].cols)
    c = host[big]
    rows, cols, n, nnz = c.rows, c.cols, c.rows * c.cols, c.nnz
    m = endor.to_device(c)
    ro = torch.from_numpy(c.row_offsets).cuda()
    stream = torch.cuda.current_stream()
    out = []

    def timed(name, fn, alg_bytes, reps=20, note=""):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        gbs = alg_bytes / ms / 1e6
        out.append({"name": name, "matrix": [shapes[big][0], rows, cols], "ms": round(ms, 4),
                    "algorithmic_bytes": int(alg_bytes), "GB/s": round(gbs, 1),
                    "hbm_frac": round(gbs / HBM_PEAK_GBS, 4), "note": note})

    # 8-bit variant, whole path (same bitmap density, one byte per value)
    w8 = synth.pruned_int8(rows, cols, args.keep, seed=synth.seed_for(cfg, big, 8))
    c8 = endor.compress(w8, want_row_offsets=False)
    m8 = endor.to_device(c8)
    o8 = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
    ws8 = torch.empty(max(256, endor.workspace_bytes(rows, cols)), dtype=torch.uint8, device="cuda")
    timed("decompress_u8", lambda: endor.decompress(m8, out=o8, workspace=ws8), n + n // 8 + c8.nnz,
          note="endor_decompress_u8: offsets + expand, 1 + 1/8 + p bytes per element")
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
    timed("decompress_cols_10pct", lambda: endor.decompress_cols(mw, row, csel, out=ocol),
          cw.rows * cw.cols // 8 + 2 * cw.rows * csel_np.size + 2 * (cw.nnz // 10),
          note="endor_decompress_cols on a sorted random tenth of the columns of %s %dx%d; algorithmic = whole "
               "bitmap + selected values read + output written (the values come 2 bytes at a time out of "
               "32-byte sectors)" % (shapes[wide][0], cw.rows, cw.cols))
    del ocol

    # device-side compressor: dense -> bitmap + values (+ table); two passes over the dense matrix by design
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
          note="endor_compress_device; algorithmic = one read of dense + bitmap + values written "
               "(the implementation reads the dense matrix twice)")
    assert int(nnz_dev.item()) == nnz
    del dense, vals, bm

    # fused consumer
    x = torch.randn(cols, device="cuda").to(torch.float16)
    y = torch.empty(rows, dtype=torch.float32, device="cuda")
    timed("gemv_f16", lambda: endor.gemv_f16(m, ro, x, y=y), n // 8 + 2 * nnz + 8 * (rows + 1) + 2 * cols + 4 * rows,
          note="endor_gemv_f16: bitmap + values + row offsets + x read, y written; a dense fp16 GEMV "
               "would read %d bytes" % (2 * n))
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
    return out


def overlap_leg(endor, torch, host, outs, args):
    """Pinned host -> device copy of the compressed blobs, alone and overlapped with
    decompression (two streams, double-buffered staging).  PCIe-bound by design: these
    figures are reported beside `value`, never as it."""
    pinned = [endor.pin(c) for c in host]
    whole = [endor.HostBlob(c.rows, c.cols, p[0], p[1], c.nnz) for c, p in zip(host, pinned)]
    blocks, block_outs = [], []
    for c, p, o in zip(host, pinned, outs):
        for b in endor.row_blocks(c, p, args.overlap_blocks):
            blocks.append(b)
            block_outs.append(o[b.row_begin:b.row_begin + b.rows])
    s_copy, s_comp = torch.cuda.Stream(), torch.cuda.Stream()
    compressed_bytes = sum(c.bitmap.nbytes + c.values.nbytes for c in host)
    dense_bytes = sum(2 * c.rows * c.cols for c in host)

    def buffers(blobs):
        sb = max(endor.stage_bytes(b.rows, b.cols, b.nnz) for b in blobs)
        wb = max(256, max(endor.workspace_bytes(b.rows, b.cols) for b in blobs))
        return ([torch.empty(sb, dtype=torch.uint8, device="cuda") for _ in range(2)],
                [torch.empty(wb, dtype=torch.uint8, device="cuda") for _ in range(2)])

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / reps * 1e3

    st_w, ws_w = buffers(whole)
    st_b, ws_b = buffers(blocks)
    dev_bm = [torch.empty(c.bitmap.size, dtype=torch.uint8, device="cuda") for c in host]
    dev_v = [torch.empty(c.values.size, dtype=torch.int16, device="cuda") for c in host]

    def copy_only():
        with torch.cuda.stream(s_copy):
            for (pb, pv), db, dv in zip(pinned, dev_bm, dev_v):
                db.copy_(pb, non_blocking=True)
                dv.copy_(pv, non_blocking=True)

    def dense_copy():   # what the uncompressed baseline would move over the same link
        with torch.cuda.stream(s_copy):
            for o, hp in zip(outs, dense_pinned):
                o.copy_(hp, non_blocking=True)

    dense_pinned = [torch.empty((c.rows, c.cols), dtype=torch.int16, pin_memory=True) for c in host]
    mats = [endor.DeviceMatrix(c.rows, c.cols, db, dv, c.nnz) for c, db, dv in zip(host, dev_bm, dev_v)]
    ws = torch.empty(max(256, endor.batch_workspace_bytes(mats)), dtype=torch.uint8, device="cuda")
    copy_only()
    torch.cuda.synchronize()
    ms_copy = timed(copy_only)
    ms_dense_copy = timed(dense_copy)
    ms_dec = timed(lambda: endor.decompress_batch(mats, outs=outs, workspace=ws, stream=s_comp), reps=20)
    ms_pipe_whole = timed(lambda: endor.h2d_decompress_pipeline(whole, outs, st_w, ws_w, s_copy, s_comp))
    ms_pipe_blocks = timed(lambda: endor.h2d_decompress_pipeline(blocks, block_outs, st_b, ws_b, s_copy, s_comp))
    return {
        "compressed_bytes": compressed_bytes, "dense_bytes": dense_bytes,
        "ms_decompress_alone": round(ms_dec, 3),
        "ms_h2d_copy_compressed_alone": round(ms_copy, 3),
        "ms_h2d_copy_dense_alone": round(ms_dense_copy, 3),
        "h2d_GBps": round(compressed_bytes / ms_copy / 1e6, 1),
        "ms_pipeline_whole_matrices": round(ms_pipe_whole, 3),
        "ms_pipeline_row_blocks": round(ms_pipe_blocks, 3),
        "row_blocks_per_matrix": args.overlap_blocks,
        "sum_copy_plus_decompress_ms": round(ms_copy + ms_dec, 3),
        "dense_GBps_pcie_inclusive": round(dense_bytes / ms_pipe_blocks / 1e6, 1),
        "speedup_vs_dense_copy": round(ms_dense_copy / ms_pipe_blocks, 3),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama2_70b_layer", choices=sorted(WORKLOADS))
    ap.add_argument("--keep", type=float, default=0.5)
    ap.add_argument("--row-skew", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="rough CPU-baseline budget (core-seconds)")
    ap.add_argument("--rotate", type=int, default=3,
                    help="number of distinct device copies of the compressed input that the timed steps "
                         "cycle through, so that no step finds its input in a cache left by the one before")
    ap.add_argument("--overlap", action="store_true",
                    help="also time the pinned host-to-device copy, alone and pipelined with decompression "
                         "on a second stream (adds an \"overlap\" object)")
    ap.add_argument("--overlap-blocks", type=int, default=4, help="row blocks per matrix in the pipeline")
    ap.add_argument("--extras", action="store_true",
                    help="also time the widened entry points on the workload's largest matrix: 8-bit "
                         "variant, row subset, device-side compressor, fused y = W x (adds an \"extras\" list)")
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
    dev = torch.device("cuda:0")

    cfg, desc = WORKLOADS[args.workload]
    shapes = synth.CONFIGS[cfg]
    t_gen = time.time()
    host = []
    for i, (name, rows, cols) in enumerate(shapes):
        w = synth.pruned_fp16(rows, cols, args.keep, seed=synth.seed_for(cfg, i), row_skew=args.row_skew)
        host.append(endor.compress(w, want_row_offsets=True))
        del w
    t_gen = time.time() - t_gen

    rotate = max(1, args.rotate)
    mats_sets = [[endor.to_device(c, dev) for c in host] for _ in range(rotate)]
    mats = mats_sets[0]
    outs = [torch.empty((c.rows, c.cols), dtype=torch.int16, device=dev) for c in host]
    ws_bytes = max(256, endor.batch_workspace_bytes(mats))
    workspaces = [torch.empty(ws_bytes, dtype=torch.uint8, device=dev) for _ in range(rotate)]
    stream = torch.cuda.current_stream()
    turn = [0]

    n_total = sum(c.rows * c.cols for c in host)
    nnz_total = sum(c.nnz for c in host)
    dense_bytes = 2 * n_total
    alg_bytes = 2 * n_total + sum((c.rows * c.cols + 7) // 8 for c in host) + 2 * nnz_total

    def step():
        k = turn[0] = (turn[0] + 1) % rotate
        endor.decompress_batch(mats_sets[k], outs=outs, workspace=workspaces[k], stream=stream)

    def expand_only():
        k = turn[0] = (turn[0] + 1) % rotate
        endor.decompress_batch_with_offsets(mats_sets[k], workspaces[k], outs=outs, stream=stream)

    if args.calibrate_copy:
        # a plain copy of the largest output into a same-sized buffer: reads and
        # writes exactly 2*rows*cols bytes, whatever the counters say about it
        big = max(range(len(outs)), key=lambda i: outs[i].numel())
        ref = torch.empty_like(outs[big])
        ref.copy_(outs[big])
        torch.cuda.synchronize()
        print(f"calibration copy: {2 * outs[big].numel()} bytes read and written", file=sys.stderr, flush=True)
        del ref

    # ---- whole path: W warm-up steps, then exactly K timed steps
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ev_ms = ev0.elapsed_time(ev1) / args.steps
    ms_per_step = wall_ms
    dense_gbs = dense_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- dominant kernel alone (every workspace holds its input set's table by now):
    # per-launch duration from HIP events recorded around every launch
    for k in range(rotate):
        endor.build_offsets_batch(mats_sets[k], workspace=workspaces[k], stream=stream)
    for _ in range(max(2, args.warmup)):
        expand_only()
    torch.cuda.synchronize()
    reps = max(10, args.steps)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record(stream)
        expand_only()
        b.record(stream)
    torch.cuda.synchronize()
    per = sorted(a.elapsed_time(b) for a, b in evs)
    # back-to-back launches, one event pair around all of them: the average launch duration
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(reps):
        expand_only()
    b.record(stream)
    torch.cuda.synchronize()
    expand_ms = a.elapsed_time(b) / reps
    achieved = alg_bytes / (expand_ms * 1e-3) / 1e9

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{args.workload}.json")
    if os.path.exists(tpath) and args.keep == 0.5 and not args.row_skew:
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")

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
            "matrices": [[n, r, c] for n, r, c in shapes], "elements": n_total, "nnz": nnz_total,
            "dense_bytes": dense_bytes, "algorithmic_bytes": alg_bytes, "input_sets_rotated": rotate,
            "launch": "endor_decompress_batch: tile-offset kernel + expand kernel, one pair for the whole batch",
        },
        "path": {
            "ms_per_step_events": round(ev_ms, 4),
            "hbm_frac_whole_path": round(alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
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
            "bytes_per_launch": alg_bytes,
            "avg_launch_ms": round(expand_ms, 4),
            "median_single_launch_ms": round(per[len(per) // 2], 4),
            "min_single_launch_ms": round(per[0], 4),
        },
    }

    if args.overlap:
        result["overlap"] = overlap_leg(endor, torch, host, outs, args)
    if args.extras:
        result["extras"] = extras_leg(endor, synth, torch, np, host, shapes, cfg, args)

    if not args.no_cpu_baseline:
        from oracle import endor_oracle as orc
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "1024")))
        # bounded sample: the largest matrices of the workload, whole, until the budget is used
        order = sorted(range(len(host)), key=lambda i: -host[i].rows * host[i].cols)
        done_bytes, spent, used, passes = 0, 0.0, [], 0
        while spent * cores <= args.cpu_seconds and passes < 20:
            passes += 1
            for i in order:
                c = host[i]
                buf = np.empty((c.rows, c.cols), np.uint16)
                t = time.perf_counter()
                orc.decompress_threaded(c.rows, c.cols, c.bitmap, c.values, c.row_offsets, cores, out=buf)
                dt = time.perf_counter() - t
                spent += dt
                done_bytes += 2 * c.rows * c.cols
                used.append(shapes[i][0])
                del buf
                if spent * cores > args.cpu_seconds:
                    break
        result["cpu_baseline"] = {
            "value": round(done_bytes / spent / 1e9, 3),
            "unit": "GB/s",
            "cores": cores,
            "kind": "oracle",
            "sample": f"Algorithm 2 oracle, rows split over {cores} threads, {len(used)} whole matrices of the "
                      f"workload, largest first, cycling ({done_bytes} dense bytes in {spent:.2f} s wall)",
        }

    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
