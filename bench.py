#!/usr/bin/env python3
"""Benchmark of the tiled spGEMM hot path on one MI355X.

One step = one full C = A*A through tsp_spgemm (CSR in, CSR out: conversion to tiles, symbolic
phase, counting pass, MFMA numeric phase, CSR emission, allocation of C) with the inputs already
resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..5] [--no-cpu-baseline]

metric: spGEMM GFLOP/s = 2 * intermediate products / second.
roofline: for the kernel that takes the most device time in a step, algorithmic HBM bytes per
launch divided by its average duration (HIP events on the launch stream, recorded by the
library around every kernel), against the 8 TB/s HBM peak.
cpu_baseline: the CPU oracle (row-wise Gustavson, fp64) timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
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


# HBM bytes per launch measured with rocprofv3 (--pmc FETCH_SIZE, then --pmc WRITE_SIZE, one run each, on
# this bench at --steps 3), scaled by what the same counters read for a 1 GiB device copy: fetched bytes =
# 2048 * FETCH_SIZE, written bytes = 1024 * WRITE_SIZE.  profiles/hbm_traffic_all_kernels.txt holds the
# readings and commands.  Keyed by (workload, kernel); a kernel that has changed since needs a new reading.
MEASURED_TRAFFIC_BYTES = {
    (2, "numeric"): 2048 * 30665.9 + 1024 * 26555.3,
    (2, "sym_emit"): 2048 * 11415.9 + 1024 * 24759.9,      # with the counting pass and the row offsets
    (3, "numeric"): 2048 * 341237.0 + 1024 * 1196171.5,
}


def popcount32(x):
    x = x.astype(np.uint32)
    x = x - ((x >> 1) & 0x55555555)
    x = (x & 0x33333333) + ((x >> 2) & 0x33333333)
    x = (x + (x >> 4)) & 0x0F0F0F0F
    return ((x * 0x01010101) >> 24).astype(np.int64)


def algorithmic_bytes(kernel, A, st, groups_left, groups_right):
    """Bytes the method itself has to move in one launch of `kernel` (every array read or written
    exactly once; re-reads of tiles through the task list are not counted)."""
    n, nnz = A.rows, A.nnz
    ta, ct, pairs, cnnz = st["a_tiles"], st["c_tiles"], st["pairs"], st["c_nnz"]
    ntr = (n + 15) // 16
    tile_meta = ta * (4 + 32 + 4 + 4 + 8 + 8)          # tile_col, row masks, 2 group masks, 2 headers {mask, first group}
    csr_in = 4 * (n + 1) + 6 * nnz
    table = {
        "convert": csr_in + 8 * ntr + tile_meta + 16 * (groups_left + groups_right),
        # symbolic kernels: tile CSR of A, and per candidate the B tile's column and occupancy word
        "sym_count": 8 * ntr + 8 * ta + 8 * st["candidate_pairs"] + 12 * ntr,
        "sym_emit": 8 * ntr + 8 * ta + 8 * st["candidate_pairs"] + 16 * ntr + 16 * ct + 8 * pairs,
        "count_masks": 8 * ct + 8 * pairs + 32 * ta + 32 * ta + 32 * ct,
        "row_offsets": 4 * ntr + 32 * ct + 64 * ct + 4 * n,
        "numeric": (8 * ct + 8 * pairs + 8 * ct + 32 * ct + 64 * ct + 8 * (n + 1)      # task list, C tile info
                    + 16 * ta + 16 * (groups_left + groups_right)                    # tile headers and groups, each once
                    + 8 * cnnz),                                                     # C col_idx + val
        "scan_sym": 24 * ntr, "scan_rows": 16 * n,
    }
    return int(table[kernel])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", type=int, default=2, help="benchmark configuration 1..5 (see inputs.CONFIG_NAMES)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-validate", action="store_true", help="switch the input validation kernel off")
    ap.add_argument("--no-matrix-cores", action="store_true",
                    help="block products on the vector ALUs instead of MFMA (the paper's nonTCU comparison)")
    ap.add_argument("--compact-zeros", action="store_true",
                    help="finish every step with the compaction of zero-valued entries (paper Section 4.4)")
    ap.add_argument("--numeric-run", type=int, default=0, help="tiles per wave of the multiplication kernel (0: automatic)")
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

    A = inputs.config(args.workload)
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
    steps = args.steps if args.steps is not None else int(min(200, max(5, 10.0 / est)))
    warmup = args.warmup if args.warmup is not None else min(5, steps)

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
    ksum = {k: 0.0 for k in tsp.KERNELS}
    psum = {k: 0.0 for k in tsp.PHASES}
    total_us = 0.0
    for _ in range(steps):
        step()
        s2 = handle.stats()
        for k in ksum:
            ksum[k] += s2["kernel_us"][k]
        for k in psum:
            psum[k] += s2["phase_us"][k]
        total_us += s2["total_us"]
    handle.set_option(tsp.OPT_PHASE_TIMERS, 0)
    kavg = {k: v / steps for k, v in ksum.items()}
    pavg = {k: v / steps for k, v in psum.items()}

    # group counts of the tile storage, for the algorithmic byte model
    tiles = handle.convert(dA)
    tv = tiles.view()
    valid = tsp.tile_indices(tv)                           # the tile arrays have unused slots between tile-rows
    groups_left = int(popcount32(tv["left_group_mask"][valid].cpu().numpy().view(np.uint32)).sum())
    groups_right = int(popcount32(tv["right_group_mask"][valid].cpu().numpy().view(np.uint32)).sum())
    tiles.free()

    dominant = max(kavg, key=kavg.get)
    dom_bytes = algorithmic_bytes(dominant, A, st, groups_left, groups_right)
    if dominant == "sym_emit" and kavg.get("count_masks", 0.0) == 0.0:
        # the task-list kernel also ran the counting pass and the row offsets (they report 0 then)
        dom_bytes += sum(algorithmic_bytes(k, A, st, groups_left, groups_right) for k in ("count_masks", "row_offsets"))
    dom_us = kavg[dominant]
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9 if dom_us > 0 else 0.0
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5),
                "traffic": (int(MEASURED_TRAFFIC_BYTES[(args.workload, dominant)])
                            if (args.workload, dominant) in MEASURED_TRAFFIC_BYTES else None),
                "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_us": round(dom_us, 2)}
    # the numeric kernel is the one dense contraction: issued MFMA work against the matrix-core peak
    num_us = kavg["numeric"]
    mfma_flop = st["pairs"] * 2.0 * 16 ** 3
    mfma = {"kernel": "numeric", "issued_dense_tflops": round(mfma_flop / (num_us * 1e-6) / 1e12, 3) if num_us else 0.0,
            "peak_tflops": MFMA_F16_PEAK_TFLOPS,
            "frac": round(mfma_flop / (num_us * 1e-6) / 1e12 / MFMA_F16_PEAK_TFLOPS, 5) if num_us else 0.0,
            "useful_fraction_of_issued": round(flop / mfma_flop, 4) if mfma_flop else 0.0}
    whole_bytes = (4 * (A.rows + 1) + 6 * A.nnz) + 8 * st["c_nnz"] + 8 * (A.rows + 1)
    end_to_end = {"compulsory_bytes": whole_bytes,
                  "hbm_frac": round(whole_bytes / (elapsed / steps) / 1e9 / HBM_PEAK_GBS, 5)}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import reference
        reference.build_lib()
        threads = min(16, os.cpu_count() or 1)
        # bounded sample: leading rows holding about a fixed number of products
        rl = np.diff(A.row_ptr).astype(np.int64)
        csum = np.concatenate([[0], np.cumsum(rl[A.col_idx])])
        per_row = csum[A.row_ptr.astype(np.int64)]          # products of rows [0, i)
        budget = 4e8                      # products: a few seconds of single-thread oracle work per run
        rows = int(np.searchsorted(per_row, budget, side="right"))
        rows = max(1, min(A.rows, rows))
        sample_products = int(per_row[rows])
        sub = inputs.CSRMatrix(rows, A.cols, A.row_ptr[:rows + 1], A.col_idx[:A.row_ptr[rows]],
                               A.val[:A.row_ptr[rows]])
        def timed(nthreads, seconds=10.0):
            """Repeat the sample until about `seconds` of wall time have gone by; mean time of one run."""
            t0 = time.perf_counter()
            r = reference.spgemm(sub, A, threads=nthreads)
            dt = time.perf_counter() - t0
            reps = int(min(2000, seconds / max(dt, 1e-4)))
            if reps > 1:
                t0 = time.perf_counter()
                for _ in range(reps):
                    reference.spgemm(sub, A, threads=nthreads)
                dt = (time.perf_counter() - t0) / reps
            return r, dt, max(reps, 1)

        r1, t1, _ = timed(1)
        _, tn, reps = timed(threads)
        assert r1.products == sample_products
        cpu = {"value": round(2.0 * sample_products / tn / 1e9, 4), "unit": "GFLOP/s", "cores": threads,
               "kind": "oracle",
               "sample": f"rows [0,{rows}) of {A.rows} of C = A*A ({sample_products} products, {r1.nnz} entries of C), "
                         f"mean of {reps} runs",
               "single_thread_value": round(2.0 * sample_products / t1 / 1e9, 4),
               "seconds": round(tn, 3), "single_thread_seconds": round(t1, 3)}

    line = {
        "metric": "spGEMM GFLOP/s (2 x intermediate products / s), C = A*A, CSR in -> CSR out",
        "value": round(gflops, 3), "unit": "GFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 x f16 -> f32", "data": "synthetic",
        "config": {"workload": f"configs[{args.workload - 1}]: {inputs.CONFIG_NAMES[args.workload]}",
                   "rows": A.rows, "nnz_A": A.nnz, "products": products, "nnz_C": st["c_nnz"],
                   "a_tiles": st["a_tiles"], "pairs": st["pairs"], "c_tiles": st["c_tiles"],
                   "validate_inputs": not args.no_validate, "matrix_cores": not args.no_matrix_cores, "compact_zeros": args.compact_zeros, "first_call_ms": round(first * 1e3, 3)},
        "roofline": roofline, "mfma": mfma, "end_to_end": end_to_end,
        "kernel_us": {k: round(v, 2) for k, v in kavg.items()},
        "phase_us": {k: round(v, 2) for k, v in pavg.items()},
        "device_us_per_step_with_timers": round(total_us / steps, 2),
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    handle.close()


if __name__ == "__main__":
    main()
