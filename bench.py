#!/usr/bin/env python3
"""Benchmark of the tiled spGEMM hot path on one MI355X.

One step = one full C = A*A through tsp_spgemm (CSR in, CSR out: conversion to tiles, symbolic
phase, counting pass, MFMA numeric phase, CSR emission, allocation of C) with the inputs already
resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..5] [--no-cpu-baseline]
                  [--no-per-workload]

The headline (value, ms_per_step, roofline, cpu_baseline) is the workload --workload names, by
default the largest of the five benchmark configurations (R-MAT scale 18: 9.49e9 intermediate
products, 2.96e9 entries of C); `per_workload` carries the same figures for all five.

metric: spGEMM GFLOP/s = 2 * intermediate products / second.
roofline: for the kernel that takes the most device time in a step, the bytes the method itself has
to move in one launch (packed fp16 elements, a 32-byte bitmap and a 16-byte record per tile, 8 bytes
per task-list entry, 8 bytes per entry of C: `algorithmic_bytes`) divided by the kernel's average
duration (HIP events on the launch stream, recorded by the library around every kernel), against the
8 TB/s HBM peak.  `layout_bytes_per_launch` is the same count for the arrays this library actually
keeps (operand groups of 16 bytes, row offsets per output tile), for comparison.
phase_hbm: the same for the conversion, the symbolic phase (with the counting pass), the numeric
phase with its CSR emission, and a separately timed tsp_compact_zeros call on the result.
cpu_baseline: the CPU oracle (row-wise Gustavson, fp64) timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16 MFMA, published
CSRC = os.path.join(ROOT, "paper_2009_14600_amd", "csrc")

# HBM bytes per launch measured with rocprofv3 (--pmc FETCH_SIZE, then --pmc WRITE_SIZE, one run each, on
# this bench with --no-per-workload --steps 3), scaled by what the same counters read for a 1 GiB device
# copy: fetched bytes = 2048 * FETCH_SIZE, written bytes = 1024 * WRITE_SIZE.  Every reading carries the
# first 12 hex digits of the SHA-256 of the kernel's source file as it was when the reading was taken; a
# reading whose source has changed since is not reported (traffic: null) instead of going stale silently.
# profiles/hbm_traffic_all_kernels.txt holds the readings and the commands.
#   (workload, kernel): (source file, sha256[:12] at the time, FETCH_SIZE, WRITE_SIZE)
MEASURED_TRAFFIC = {
    (1, "convert"): ("convert.hip", "67ac7a722d7c", 201.6, 782.7),
    (1, "count_masks"): ("symbolic.hip", "65d32d837ef3", 733.6, 128.0),
    (1, "numeric"): ("numeric.hip", "ed6fb3a14cf6", 1264.8, 499.0),
    (1, "row_offsets"): ("symbolic.hip", "65d32d837ef3", 91.1, 262.0),
    (1, "scan_rows"): ("symbolic.hip", "65d32d837ef3", 6.4, 8.3),
    (1, "scan_sym"): ("symbolic.hip", "65d32d837ef3", 7.2, 1.3),
    (1, "sym_count"): ("symbolic.hip", "65d32d837ef3", 190.2, 10.0),
    (1, "sym_emit"): ("symbolic.hip", "65d32d837ef3", 203.6, 478.3),
    (2, "convert"): ("convert.hip", "67ac7a722d7c", 6120.4, 43223.1),
    (2, "numeric"): ("numeric.hip", "ed6fb3a14cf6", 30663.9, 26555.3),
    (2, "scan_rows"): ("symbolic.hip", "65d32d837ef3", 790.2, 2048.5),
    (2, "scan_sym"): ("symbolic.hip", "65d32d837ef3", 256.6, 214.2),
    (2, "sym_count"): ("symbolic.hip", "65d32d837ef3", 6153.1, 1280.0),
    (2, "sym_emit"): ("symbolic.hip", "65d32d837ef3", 11418.3, 24504.0),
    (3, "convert"): ("convert.hip", "67ac7a722d7c", 82440.9, 294561.7),
    (3, "numeric"): ("numeric.hip", "ed6fb3a14cf6", 340006.1, 1194490.5),
    (3, "scan_rows"): ("symbolic.hip", "65d32d837ef3", 994.2, 2592.3),
    (3, "scan_sym"): ("symbolic.hip", "65d32d837ef3", 312.2, 271.0),
    (3, "sym_count"): ("symbolic.hip", "65d32d837ef3", 22562.4, 3241.0),
    (3, "sym_emit"): ("symbolic.hip", "65d32d837ef3", 71423.4, 266006.1),
    (4, "convert"): ("convert.hip", "67ac7a722d7c", 38660.3, 473242.6),
    (4, "count_masks"): ("symbolic.hip", "65d32d837ef3", 119848216.4, 4612574.6),
    (4, "numeric"): ("numeric.hip", "ed6fb3a14cf6", 269244343.1, 33419349.5),
    (4, "row_offsets"): ("symbolic.hip", "65d32d837ef3", 4666779.8, 9241581.6),
    (4, "scan_rows"): ("symbolic.hip", "65d32d837ef3", 790.4, 2049.1),
    (4, "scan_sym"): ("symbolic.hip", "65d32d837ef3", 255.9, 196.9),
    (4, "sym_count"): ("symbolic.hip", "65d32d837ef3", 15365684.4, 508990.6),
    (4, "sym_emit"): ("symbolic.hip", "65d32d837ef3", 50858751.2, 70878252.9),
    (5, "convert"): ("convert.hip", "67ac7a722d7c", 14192.6, 50065.9),
    (5, "numeric"): ("numeric.hip", "ed6fb3a14cf6", 53954.3, 270245.2),
    (5, "scan_rows"): ("symbolic.hip", "65d32d837ef3", 406.2, 1024.5),
    (5, "scan_sym"): ("symbolic.hip", "65d32d837ef3", 153.4, 98.5),
    (5, "sym_count"): ("symbolic.hip", "65d32d837ef3", 4864.1, 1280.0),
    (5, "sym_emit"): ("symbolic.hip", "65d32d837ef3", 8703.7, 16309.8),
}

KERNEL_SOURCE = {"convert": "convert.hip", "sym_count": "symbolic.hip", "scan_sym": "symbolic.hip",
                 "sym_emit": "symbolic.hip", "count_masks": "symbolic.hip", "row_offsets": "symbolic.hip",
                 "scan_rows": "symbolic.hip", "numeric": "numeric.hip"}


def source_digest(name: str) -> str:
    with open(os.path.join(CSRC, name), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:12]


def measured_traffic(workload: int, kernel: str):
    rec = MEASURED_TRAFFIC.get((workload, kernel))
    if rec is None or source_digest(rec[0]) != rec[1]:
        return None
    return int(2048 * rec[2] + 1024 * rec[3])


def popcount32(x):
    x = x.astype(np.uint32)
    x = x - ((x >> 1) & 0x55555555)
    x = (x & 0x33333333) + ((x >> 2) & 0x33333333)
    x = (x + (x >> 4)) & 0x0F0F0F0F
    return ((x * 0x01010101) >> 24).astype(np.int64)


def algorithmic_bytes(kernel, A, st):
    """Bytes the method itself has to move in one launch of `kernel`: every object read or written
    once, in the paper's packed tile format (Section 2.1.2 at a tile edge of 16: 2 bytes per stored
    element, a 32-byte bitmap and a 16-byte record {tile column, occupancy words, element offset} per
    tile), 8 bytes per task-list entry, 16 bytes of coordinates and segment offset per output tile, a
    32-byte bitmap per output tile, 8 bytes per entry of C and 8 per row pointer of C.  Re-reads of
    tiles through the task list are not counted, nor is anything this library's own layout adds."""
    n, nnz = A.rows, A.nnz
    ta, ct, pairs, cnnz = st["a_tiles"], st["c_tiles"], st["pairs"], st["c_nnz"]
    ntr = (n + 15) // 16
    tiles_packed = 2 * nnz + 48 * ta
    table = {
        "convert": 4 * (n + 1) + 6 * nnz + tiles_packed,                   # CSR in, tiles out
        "sym_count": 16 * ta + 16 * ntr,                                   # tile records in, sizes per tile-row out
        "scan_sym": 24 * ntr,
        "sym_emit": 16 * ta + 16 * ntr + 8 * pairs + 16 * ct,              # tile records in, task list out
        "count_masks": 8 * pairs + 16 * ct + 32 * ta + 32 * ct,            # task list and bitmaps in, C bitmaps out
        "row_offsets": 32 * ct + 4 * n,                                    # C bitmaps in, entries per row out
        "scan_rows": 4 * n + 8 * (n + 1),
        "numeric": tiles_packed + 8 * pairs + 16 * ct + 32 * ct + 8 * cnnz + 8 * (n + 1),
        # the task-list kernel when it also runs the counting pass: the task list and the C bitmaps are not read back
        "sym_emit_fused": 16 * ta + 16 * ntr + 8 * pairs + 16 * ct + 32 * ta + 32 * ct + 4 * n,
    }
    return int(table[kernel])


def layout_bytes(kernel, A, st, groups_left, groups_right):
    """The same count for the arrays this library keeps (operand groups of 16 bytes in both forms,
    60 bytes of tile metadata, 64 bytes of row offsets per output tile)."""
    n, nnz = A.rows, A.nnz
    ta, ct, pairs, cnnz = st["a_tiles"], st["c_tiles"], st["pairs"], st["c_nnz"]
    ntr = (n + 15) // 16
    tile_meta = ta * (4 + 32 + 4 + 4 + 8 + 8)
    csr_in = 4 * (n + 1) + 6 * nnz
    table = {
        "convert": csr_in + 8 * ntr + tile_meta + 16 * (groups_left + groups_right),
        "sym_count": 8 * ntr + 8 * ta + 8 * st["candidate_pairs"] + 12 * ntr,
        "sym_emit": 8 * ntr + 8 * ta + 8 * st["candidate_pairs"] + 16 * ntr + 16 * ct + 8 * pairs,
        "count_masks": 8 * ct + 8 * pairs + 32 * ta + 32 * ta + 32 * ct,
        "row_offsets": 4 * ntr + 32 * ct + 64 * ct + 4 * n,
        "numeric": (8 * ct + 8 * pairs + 8 * ct + 32 * ct + 64 * ct + 8 * (n + 1)
                    + 16 * ta + 16 * (groups_left + groups_right) + 8 * cnnz),
        "scan_sym": 24 * ntr, "scan_rows": 16 * n,
    }
    return int(table[kernel])


def hbm(bytes_, us):
    gbs = bytes_ / (us * 1e-6) / 1e9 if us > 0 else 0.0
    return {"algorithmic_bytes": int(bytes_), "us": round(us, 2), "achieved_gbs": round(gbs, 1),
            "frac": round(gbs / HBM_PEAK_GBS, 5)}


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def oracle_leg(A, handle, tsp, sA, budget_products, seconds):
    """The CPU oracle on a leading block of rows holding about `budget_products` products: timed (when
    seconds > 0), and compared with the same rows of the GPU result (Eq. 3's SMAPE between the fp32
    result and the oracle's fp64 sums of the same fp16 inputs, and the largest error over the bound)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import reference
    reference.build_lib()
    threads = min(16, os.cpu_count() or 1)
    rl = np.diff(A.row_ptr).astype(np.int64)
    csum = np.concatenate([[0], np.cumsum(rl[A.col_idx])])
    per_row = csum[A.row_ptr.astype(np.int64)]          # products of rows [0, i)
    rows = int(np.searchsorted(per_row, budget_products, side="right"))
    rows = max(1, min(A.rows, rows))
    sample_products = int(per_row[rows])
    ops = (reference._Operand(A), reference._Operand(A))   # fp16 -> fp64 widening, once, outside the timing
    bounds = np.searchsorted(per_row[:rows + 1], np.linspace(0, sample_products, 8 * threads + 1)).astype(np.int64)
    bounds[0], bounds[-1] = 0, rows
    bounds = np.unique(bounds)

    def run(nthreads):
        if nthreads == 1:
            return [reference.spgemm_rows(A, A, 0, rows, _ops=ops)]
        with ThreadPoolExecutor(max_workers=nthreads) as pool:
            return list(pool.map(lambda i: reference.spgemm_rows(A, A, int(bounds[i]), int(bounds[i + 1]), _ops=ops),
                                 range(bounds.shape[0] - 1)))

    def timed(nthreads):
        t0 = time.perf_counter()
        parts = run(nthreads)
        dt = time.perf_counter() - t0
        reps = int(min(2000, seconds / max(dt, 1e-4)))
        if reps > 1:
            t0 = time.perf_counter()
            for _ in range(reps):
                run(nthreads)
            dt = (time.perf_counter() - t0) / reps
        return parts, dt, max(reps, 1)

    out = {}
    if seconds > 0:
        p1, t1, _ = timed(1)
        parts, tn, reps = timed(threads)
        assert sum(p.products for p in p1) == sample_products
        out["cpu_baseline"] = {
            "value": round(2.0 * sample_products / tn / 1e9, 4), "unit": "GFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"rows [0,{rows}) of {A.rows} of C = A*A ({sample_products} products, "
                      f"{sum(p.nnz for p in parts)} entries of C), mean of {reps} runs",
            "includes": "per block of rows: the sizing pass (structural row lengths) and the value pass "
                        "(dense accumulator, fp64 sums and sums of magnitudes, column sort); excludes the "
                        "one-off widening of the fp16 inputs to fp64 and the generation of the inputs",
            "cpu": cpu_model(), "host_cores_visible": os.cpu_count(),
            "single_thread_value": round(2.0 * sample_products / t1 / 1e9, 4),
            "seconds": round(tn, 3), "single_thread_seconds": round(t1, 3)}
    else:
        parts = run(threads)
    # the same rows of the GPU result
    raw = handle.spgemm_raw(sA, sA)
    C = handle._wrap_output(raw)
    rp = C.row_ptr[:rows + 1].cpu().numpy()
    hi = int(rp[-1])
    col, val = C.col_idx[:hi].cpu().numpy(), C.val[:hi].cpu().numpy().astype(np.float64)
    C.free()
    ref_col = np.concatenate([p.col for p in parts])
    ref_val = np.concatenate([p.val for p in parts])
    ref_mag = np.concatenate([p.mag for p in parts])
    same = ref_col.shape == col.shape and np.array_equal(ref_col, col)
    out["accuracy"] = {"rows": rows, "entries": int(hi), "pattern_equal": bool(same)}
    if same and hi:
        out["accuracy"]["smape_percent"] = round(reference.smape_percent(ref_val, val), 8)
        out["accuracy"]["max_error_over_bound"] = round(float(np.max(np.abs(val - ref_val) / (1e-5 * ref_mag + 1e-7))), 5)
    return out


PAPER_PIPELINE_MAX_PAIRS = 200_000_000     # larger task lists: its sorted candidate arrays take tens of GB and seconds


def paper_pipeline_leg(handle, tsp, torch, dA, own_ms):
    """The same product by the paper's own pipeline (tsp_spgemm_paper: packed bitmap tiles, task list by
    expansion and a library sort, elements placed by bitmap into dense LDS tiles) at tile edges 8, 16 and 32:
    time per call with its host waits, device time per phase, tile and task-list counts at that edge, and
    whether the pattern equals the library's."""
    own = handle.spgemm(dA, dA)
    legs = []
    for T in (8, 16, 32):
        leg = {"tile_edge": T}
        try:
            C = handle.spgemm_paper(dA, dA, T)                 # sizes the workspace
        except tsp.TspError as e:
            leg["status"] = str(e)
            legs.append(leg)
            continue
        leg["pattern_equal_to_library"] = bool(C.nnz == own.nnz and torch.equal(C.row_ptr, own.row_ptr)
                                               and torch.equal(C.col_idx[:C.nnz], own.col_idx[:own.nnz]))
        C.free()
        handle.set_option(tsp.OPT_PHASE_TIMERS, 1)
        reps = 3
        phases = {k: 0.0 for k in tsp.PHASES}
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            C = handle.spgemm_paper(dA, dA, T)
            st = handle.stats()
            for k in phases:
                phases[k] += st["phase_us"][k]
            C.free()
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / reps
        handle.set_option(tsp.OPT_PHASE_TIMERS, 0)
        leg.update({"ms_per_call": round(ms, 4), "times_the_library": round(ms / own_ms, 1),
                    "phase_us": {k: round(v / reps, 1) for k, v in phases.items()},
                    "a_tiles": st["a_tiles"], "candidate_pairs": st["candidate_pairs"], "pairs": st["pairs"],
                    "c_tiles": st["c_tiles"]})
        legs.append(leg)
    own.free()
    return legs


def run_workload(index, steps, warmup, args, tsp, inputs, torch, headline):
    A = inputs.config(index)
    products = int(np.diff(A.row_ptr).astype(np.int64)[A.col_idx].sum())
    flop = 2.0 * products
    dA = tsp.to_device(A)
    sA = dA._struct()
    handle = tsp.Handle(validate=not args.no_validate)
    if args.no_matrix_cores:
        handle.set_option(tsp.OPT_MATRIX_CORES, 0)
    if args.compact_zeros:
        handle.set_option(tsp.OPT_COMPACT_ZEROS, 1)
    if args.numeric_run:
        handle.set_option(tsp.OPT_NUMERIC_RUN, args.numeric_run)
    if args.strip_order:
        handle.set_option(tsp.OPT_STRIP_ORDER, args.strip_order)
    if args.wide_index:
        handle.set_option(tsp.OPT_WIDE_INDEX, 1)

    def step():
        out = handle.spgemm_raw(sA, sA)
        handle._free_csr(out)

    # one untimed call sizes the workspace and tells us how long a step takes
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step()
    torch.cuda.synchronize()
    first = time.perf_counter() - t0
    t0 = time.perf_counter()
    step()
    torch.cuda.synchronize()
    est = max(time.perf_counter() - t0, 1e-5)
    if steps is None:
        steps = int(min(200, max(5, (10.0 if headline else 1.0) / est)))
    if warmup is None:
        warmup = min(5, steps)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / steps
    gflops = flop / (elapsed / steps) / 1e9
    st = handle.stats()

    # per-kernel device time: same steps again with the library's event timers on
    handle.set_option(tsp.OPT_PHASE_TIMERS, 1)
    tsteps = min(steps, 20)
    ksum = {k: 0.0 for k in tsp.KERNELS}
    psum = {k: 0.0 for k in tsp.PHASES}
    total_us = 0.0
    for _ in range(tsteps):
        step()
        s2 = handle.stats()
        for k in ksum:
            ksum[k] += s2["kernel_us"][k]
        for k in psum:
            psum[k] += s2["phase_us"][k]
        total_us += s2["total_us"]
    handle.set_option(tsp.OPT_PHASE_TIMERS, 0)
    kavg = {k: v / tsteps for k, v in ksum.items()}
    pavg = {k: v / tsteps for k, v in psum.items()}

    # the library's own count of the intermediate products (an extra kernel, so outside the timed steps),
    # against the count from the row lengths above; and the paper's selection criteria for this operand
    handle.set_option(tsp.OPT_COUNT_PRODUCTS, 1)
    step()
    torch.cuda.synchronize()
    s3 = handle.stats()
    handle.set_option(tsp.OPT_COUNT_PRODUCTS, 0)
    assert s3["products"] == products, (s3["products"], products)
    regime = {"nnz_A_over_300000": A.nnz > 300000, "mean_row_A": round(s3["a_mean_row"], 2),
              "entries_per_tile_A": round(s3["a_tile_fill"], 2), "in_paper_regime": bool(s3["in_paper_regime"]),
              "well_filled_tiles": bool(s3["well_filled_tiles"])}

    # group counts of the tile storage, for the layout's own byte count
    tiles = handle.convert(dA)
    tv = tiles.view()
    valid = tsp.tile_indices(tv)                           # the tile arrays have unused slots between tile-rows
    groups_left = int(popcount32(tv["left_group_mask"][valid].cpu().numpy().view(np.uint32)).sum())
    groups_right = int(popcount32(tv["right_group_mask"][valid].cpu().numpy().view(np.uint32)).sum())
    tiles.free()

    fused_count = kavg.get("count_masks", 0.0) == 0.0       # the task-list kernel ran the counting pass as well
    dominant = max(kavg, key=kavg.get)
    dom_bytes = algorithmic_bytes(dominant, A, st)
    dom_layout = layout_bytes(dominant, A, st, groups_left, groups_right)
    if dominant == "sym_emit" and fused_count:
        dom_bytes = algorithmic_bytes("sym_emit_fused", A, st)
        dom_layout += sum(layout_bytes(k, A, st, groups_left, groups_right) for k in ("count_masks", "row_offsets"))
    dom_us = kavg[dominant]
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9 if dom_us > 0 else 0.0
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5),
                "traffic": measured_traffic(index, dominant),
                "algorithmic_bytes_per_launch": dom_bytes, "layout_bytes_per_launch": dom_layout,
                "avg_launch_us": round(dom_us, 2)}
    # the numeric kernel is the one dense contraction: issued MFMA work against the matrix-core peak
    num_us = kavg["numeric"]
    mfma_flop = st["pairs"] * 2.0 * 16 ** 3
    mfma = {"kernel": "numeric", "issued_dense_tflops": round(mfma_flop / (num_us * 1e-6) / 1e12, 3) if num_us else 0.0,
            "peak_tflops": MFMA_F16_PEAK_TFLOPS,
            "frac": round(mfma_flop / (num_us * 1e-6) / 1e12 / MFMA_F16_PEAK_TFLOPS, 5) if num_us else 0.0,
            "useful_fraction_of_issued": round(flop / mfma_flop, 4) if mfma_flop else 0.0}
    if A.nnz <= 3 * st["a_tiles"] and not args.no_matrix_cores:
        # (the kernel for tiles with a few entries packs the halves of pairs that meet, four to a step)
        mfma["note"] = ("counted as two of the four slots of a step per pair; on this workload the kernel fills a step "
                        "with the halves of up to four pairs that meet, so the issued work is lower")
    whole_bytes = (4 * (A.rows + 1) + 6 * A.nnz) + 8 * st["c_nnz"] + 8 * (A.rows + 1)
    end_to_end = {"compulsory_bytes": whole_bytes,
                  "hbm_frac": round(whole_bytes / (elapsed / steps) / 1e9 / HBM_PEAK_GBS, 5)}

    # achieved HBM rate per pass (algorithmic bytes over the device time of the pass's kernels)
    sym_kernels = ("sym_count", "scan_sym", "sym_emit", "count_masks", "row_offsets", "scan_rows")
    sym_bytes = sum(algorithmic_bytes(k, A, st) for k in sym_kernels if kavg[k] > 0.0 and not (fused_count and k == "sym_emit"))
    if fused_count:
        sym_bytes += algorithmic_bytes("sym_emit_fused", A, st)
    phase_hbm = {
        "convert": hbm(algorithmic_bytes("convert", A, st), kavg["convert"]),
        "symbolic_and_count": hbm(sym_bytes, sum(kavg[k] for k in sym_kernels)),
        "numeric_and_csr_emission": hbm(algorithmic_bytes("numeric", A, st), kavg["numeric"]),
    }
    if not args.compact_zeros:
        # the compaction of zero-valued entries (Section 4.4) as a call of its own on the result: counts the
        # survivors per row, then copies them into a new matrix
        raw = handle.spgemm_raw(sA, sA)
        cz = handle._lib.tsp_compact_zeros
        import ctypes
        reps = 3
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        us = 0.0
        out_nnz = raw.nnz
        for _ in range(reps + 1):
            out = type(raw)()
            ev0.record()
            rc = cz(handle._h, ctypes.byref(raw), ctypes.byref(out), handle._stream())
            ev1.record()
            torch.cuda.synchronize()
            if rc != 0:
                break
            out_nnz = out.nnz
            handle._free_csr(out)
            us = ev0.elapsed_time(ev1) * 1e3                # the last repetition counts (the first sizes the workspace)
        # counting pass: the values and row_ptr in, survivors per row out; prefix sum; copy pass: columns and values
        # in, the survivors and the new row_ptr out
        moved = (4 * raw.nnz + 8 * (A.rows + 1) + 4 * A.rows) + (4 * A.rows + 8 * (A.rows + 1)) + (8 * raw.nnz + 8 * out_nnz + 8 * (A.rows + 1))
        phase_hbm["compact_zeros"] = dict(hbm(moved, us), entries_removed=int(raw.nnz - out_nnz),
                                          note="separate call on the result, its host wait included")
        handle._free_csr(raw)

    res = {
        "workload": f"configs[{index - 1}]: {inputs.CONFIG_NAMES[index]}",
        "value": round(gflops, 3), "ms_per_step": round(ms_per_step, 5), "steps": steps, "warmup": warmup,
        "config": {"workload": f"configs[{index - 1}]: {inputs.CONFIG_NAMES[index]}",
                   "rows": A.rows, "nnz_A": A.nnz, "products": products, "nnz_C": st["c_nnz"],
                   "a_tiles": st["a_tiles"], "pairs": st["pairs"], "c_tiles": st["c_tiles"],
                   "validate_inputs": not args.no_validate, "matrix_cores": not args.no_matrix_cores,
                   "compact_zeros": args.compact_zeros, "first_call_ms": round(first * 1e3, 3),
                   "selection_criteria": regime},
        "roofline": roofline, "mfma": mfma, "end_to_end": end_to_end, "phase_hbm": phase_hbm,
        "kernel_us": {k: round(v, 2) for k, v in kavg.items()},
        "phase_us": {k: round(v, 2) for k, v in pavg.items()},
        "device_us_per_step_with_timers": round(total_us / tsteps, 2),
    }
    if not args.no_paper_pipeline and st["pairs"] <= PAPER_PIPELINE_MAX_PAIRS:
        res["paper_pipeline"] = paper_pipeline_leg(handle, tsp, torch, dA, ms_per_step)
    if not args.no_cpu_baseline:
        leg = oracle_leg(A, handle, tsp, sA, 4e8 if headline else 2e7, 10.0 if headline else 0.0)
        res["accuracy_vs_oracle_sample"] = leg["accuracy"]
        if headline:
            res["cpu_baseline"] = leg["cpu_baseline"]
    handle.close()
    del dA
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", type=int, default=4, help="headline benchmark configuration 1..5 (see inputs.CONFIG_NAMES)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-workload", action="store_true", help="measure the headline workload only")
    ap.add_argument("--no-paper-pipeline", action="store_true",
                    help="skip the comparison runs of the paper's own pipeline at tile edges 8, 16, 32")
    ap.add_argument("--no-validate", action="store_true", help="switch the input validation kernel off")
    ap.add_argument("--no-matrix-cores", action="store_true",
                    help="block products on the vector ALUs instead of MFMA (the paper's nonTCU comparison)")
    ap.add_argument("--compact-zeros", action="store_true",
                    help="finish every step with the compaction of zero-valued entries (paper Section 4.4)")
    ap.add_argument("--numeric-run", type=int, default=0, help="tiles per wave of the multiplication kernel (0: automatic)")
    ap.add_argument("--wide-index", action="store_true", help="force the kernels that address arrays through 64-bit pointers")
    ap.add_argument("--strip-order", type=int, default=0,
                    help="order of the output tiles in the counting and multiplication kernels (0: automatic, 1: strips, 2: row-major)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); the path has no multi-GPU part",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2009_14600_amd import inputs, tsp
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    tsp.load_library()
    torch.cuda.set_device(0)

    per = []
    if not args.no_per_workload:
        for index in (1, 2, 3, 5, 4):
            if index == args.workload:
                continue
            r = run_workload(index, None, None, args, tsp, inputs, torch, headline=False)
            per.append(r)
            print(f"bench.py: workload {index}: {r['value']} GFLOP/s, {r['ms_per_step']} ms per step", file=sys.stderr, flush=True)
    head = run_workload(args.workload, args.steps, args.warmup, args, tsp, inputs, torch, headline=True)
    per.append(head)
    per.sort(key=lambda r: r["workload"])

    line = {
        "metric": "spGEMM GFLOP/s (2 x intermediate products / s), C = A*A, CSR in -> CSR out",
        "value": head["value"], "unit": "GFLOP/s", "n_gpus": 1, "steps": head["steps"], "warmup": head["warmup"],
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 x f16 -> f32", "data": "synthetic",
        "config": head["config"],
        "roofline": head["roofline"], "mfma": head["mfma"], "end_to_end": head["end_to_end"],
        "phase_hbm": head["phase_hbm"],
        "kernel_us": head["kernel_us"], "phase_us": head["phase_us"],
        "device_us_per_step_with_timers": head["device_us_per_step_with_timers"],
        "accuracy_vs_oracle_sample": head.get("accuracy_vs_oracle_sample"),
        "cpu_baseline": head.get("cpu_baseline"),
        "per_workload": [{k: r[k] for k in ("workload", "value", "ms_per_step", "steps", "roofline", "mfma", "end_to_end",
                                            "phase_hbm", "kernel_us", "accuracy_vs_oracle_sample", "paper_pipeline") if k in r}
                         for r in per],
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
