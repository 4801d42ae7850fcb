#!/usr/bin/env python3
"""Benchmark of the sparse ternary GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--variant tcsc|signed|packed]

One step = one tstgemm() call (the whole hot path: X packing / tile staging, gather-add, K-block carry,
split-K reduction, bias epilogue) on one batch of synthetic input that is already resident in HBM.  The
TCSC build and the GPU re-blocking pass run once per matrix before the timed region ("at load time",
Sec. 3 of the paper) and are reported separately in the config object.  Prints ONE JSON line.

Before the W warm-up calls the same calls run for --preheat seconds (default 0.5): the GPU needs some tenths of a
second of load to reach its clock, whatever --warmup and --steps are.  The timed region is EXACTLY --steps calls
between two synchronisations (`ms_per_step`, `value`); --repeats more regions of the same length give the median
and the minimum beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

# Every effective add consumes one 4-byte operand gathered from the LDS, so the binding resource of the large-M
# kernel is the LDS read port: 256 B/clk per compute unit on gfx950 (ds_read_b64/b128), 256 CUs, 2.4 GHz
# = 157.3 TB/s = 39.32 T operands (= adds) per second.  The plain VALU add rate is not the limit: the datasheet's
# 157.3 TFLOP/s fp32 vector figure is 78.6 T lane-operations/s (FMA counted as 2 flops), twice the LDS rate.
PEAK_LDS_GATHER_TFLOPS = 256 * 256 * 2.4e9 / 4 / 1e12
PEAK_ALU_ADD_TFLOPS = 157.3 / 2
PEAK_HBM_GBS = 8000.0
PEAK_ALU_INSTR_T = 256 * 64 * 2.4e9 / 1e12     # vector lane-instructions per second (an FMA counts once)

# HBM bytes (read + written) of one launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script, each counter scaled by what it reads for a copy kernel of known size in the same run.  A counter run cannot
# be part of a timed run, so these are constants: (bytes, the tracked summary they come from).  Keyed by (workload,
# variant); workloads without a counter run report null.
_T_ALL = "profiles/hbm_traffic_all_configs.md"
_T_OTHER = "profiles/hbm_traffic_other_workloads.md"
MEASURED_TRAFFIC = {
    ("C1", "tcsc"): (1820253, _T_ALL), ("C2", "tcsc"): (46305018, _T_ALL), ("C3a", "tcsc"): (46361795, _T_ALL),
    ("C3b", "tcsc"): (46404792, _T_ALL), ("C4-1", "tcsc"): (46039073, _T_ALL), ("C4-8", "tcsc"): (47360812, _T_ALL),
    ("C5a", "tcsc"): (929168828, _T_ALL), ("C5b", "tcsc"): (922709707, _T_ALL), ("C5c", "tcsc"): (902583812, _T_ALL),
    ("M64-K16384-N4096-d0.5", "tcsc"): (163358221, _T_OTHER),
    ("C4-1", "packed"): (9610285, _T_OTHER), ("C4-8", "packed"): (11881214, _T_OTHER),
}
ORACLE_FLAGS = "gcc -O3 -fstrict-aliasing -DNDEBUG -fopenmp (the paper's flags, Sec. 4, without -march=native)"
INFINITY_CACHE_BYTES = 256 << 20


def cpu_baseline(W, X, b, nnz, variant="tcsc", budget_s=10.0):
    """The oracle as it stands, on the host cores, on the same workload; repeated for about budget_s.  For the TCSC
    path a second, short run on ONE thread (the figure comparable to the paper's single-core numbers)."""
    import oracle
    t = oracle.tcsc_build(W)
    M, K = X.shape
    rows = None
    if M * nnz > 4e10:   # keep the sample to seconds: a slice of rows (the cost per row does not depend on M)
        rows = np.arange(0, M, M // 64, dtype=np.int32)[:64]
    if variant == "signed":
        enc = oracle.signed_build(t)
    elif variant == "packed":
        enc = oracle.pack5(W)
    times = []
    used = os.cpu_count() or 1   # the variant routines do not report their thread count: OpenMP's default, all cores
    t_start = time.perf_counter()
    while len(times) < 3 or (time.perf_counter() - t_start < budget_s and len(times) < 200):
        t0 = time.perf_counter()
        if variant == "signed":
            oracle.tstgemm_signed(X, enc[0], enc[1], b, K)
        elif variant == "packed":
            oracle.tstgemm_packed(X, enc, b, K)
        else:
            _, _, used = oracle.tstgemm(X, t, b) if rows is None else oracle.tstgemm(X, t, b, rows=rows)
        times.append(time.perf_counter() - t0)
    # (after the all-core run: the oracle's thread count, once set, stays set for later calls)
    one = None
    if variant == "tcsc":
        # one thread: as many evenly spaced rows as take about a tenth of a second each time, for about 3 s
        n1 = int(max(1, min(M, 2e8 // max(nnz, 1))))
        rows1 = np.arange(0, M, max(1, M // n1), dtype=np.int32)[:n1]
        t1, t_start = [], time.perf_counter()
        while len(t1) < 3 or (time.perf_counter() - t_start < 3.0 and len(t1) < 50):
            t0 = time.perf_counter()
            _, _, used1 = oracle.tstgemm(X, t, b, rows=rows1, threads=1)
            t1.append(time.perf_counter() - t0)
        one = {"value": len(rows1) * nnz / min(t1) / 1e9, "unit": "Gadds/s", "cores": int(used1),
               "sample": f"{len(rows1)} of {M} rows, evenly spaced, best of {len(t1)}"}
    mean = float(np.mean(times))
    m_used = M if rows is None else len(rows)
    out = {"value": m_used * nnz / mean / 1e9, "unit": "Gadds/s", "cores": int(used), "kind": "oracle",
           "sample": (f"whole workload (all {M} rows)" if rows is None else f"{m_used} of {M} rows, evenly spaced")
                     + f", {len(times)} repetitions, mean; best {m_used * nnz / min(times) / 1e9:.2f} Gadds/s",
           "ms": mean * 1e3, "best": m_used * nnz / min(times) / 1e9, "flags": ORACLE_FLAGS}
    if one is not None:
        out["one_thread"] = one
    return out


def large_cols_per_wave(m_tiles, n_pad, density, cus):
    """Columns of Y per wavefront the large-M path takes for a call in one slab: the library's rule, restated."""
    if n_pad % 128:
        return 4
    gain8 = (3760.0 * density + 520.0) / (3966.0 * density + 316.0)
    slots = 2 * cus
    groups8 = m_tiles * (n_pad // 128)
    rounds8, rounds4 = -(-groups8 // slots), -(-2 * groups8 // slots)
    if groups8 >= slots and 2.0 * rounds8 <= rounds4 * gain8:
        return 8
    if groups8 < slots and 2 * groups8 >= slots and gain8 >= 1.3:
        return 8
    return 4


def measured_peaks(tg, torch, stream, index_bytes):
    """What the machine delivers on the two resources the kernels are priced against, from the library's two probe
    kernels, run right after the timed work (clocks up): conflict-free 16-byte LDS reads at the large-M kernel's
    occupancy, and a plain streaming read of 1 GiB (four times the Infinity Cache: from HBM) and of a buffer of the
    size of the workload's index data read again and again (what repeated calls on one matrix can get from the cache)."""
    def best_ms(launch, reps=5):
        launch()
        torch.cuda.synchronize()
        ms = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            launch()
            e1.record(stream)
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        return min(ms)

    lds_bytes = [0]

    def lds():
        lds_bytes[0] = tg.tstgemm_probe_lds_read(2000, stream)
    ms = best_ms(lds)
    out = {"lds_read_tb_per_s": lds_bytes[0] / (ms * 1e-3) / 1e12,
           "lds_gather_tadds_per_s": lds_bytes[0] / 4 / (ms * 1e-3) / 1e12}
    big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    big.zero_()
    ms = best_ms(lambda: tg.tstgemm_probe_stream_read(big, stream))
    out["hbm_stream_read_gb_per_s"] = (1 << 30) / (ms * 1e-3) / 1e9
    del big
    if index_bytes >= 1 << 20:
        small = torch.empty(int(index_bytes) // 16 * 16, dtype=torch.uint8, device="cuda")
        small.zero_()
        ms = best_ms(lambda: tg.tstgemm_probe_stream_read(small, stream))
        out["cached_stream_read_gb_per_s"] = small.numel() / (ms * 1e-3) / 1e9
        out["cached_stream_read_bytes"] = small.numel()
    # the tile exchange of the tiled kernels by itself: 64 KiB pieces of a 4 MiB buffer (the size of C2's packed X: it
    # stays in the L2s) into the LDS of 2 x 16 wavefronts per compute unit, between the same two barriers
    tiles = torch.empty(4 << 20, dtype=torch.uint8, device="cuda")
    tiles.zero_()
    copied = [0]

    def tile_copy():
        copied[0] = tg.tstgemm_probe_tile_copy(tiles, 200, stream)
    ms = best_ms(tile_copy)
    out["tile_copy_tb_per_s"] = copied[0] / (ms * 1e-3) / 1e12
    del tiles
    out["note"] = ("probe kernels of the library (tstgemm_probe_lds_read: 2 x 16 wavefronts per CU, ds_read_b128 only; "
                   "tstgemm_probe_stream_read: 16-byte loads, grid-stride; tstgemm_probe_tile_copy: 64 KiB pieces of a 4 MiB "
                   "buffer into the LDS, load - barrier - LDS write - barrier, 2 x 16 wavefronts per CU), best of 5, at the "
                   "clock the chip holds under that load; the datasheet peaks assume 2.4 GHz and 8 TB/s")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--variant", default="tcsc", choices=["tcsc", "signed", "packed"],
                    help="tcsc: tstgemm(); signed / packed: the M <= 8 entry points on the paper's inverted-index / "
                         "value-compression encodings (Sec. 3)")
    ap.add_argument("--rotate", type=int, default=0,
                    help="upload this many copies of the matrix and take them in turn, call after call, so that the index "
                         "data of a call is no longer in the 256 MB Infinity Cache when its turn comes again.  0 (default): "
                         "1 copy for M > 8 (not bound by index bytes), for M <= 8 as many copies as hold 3 x 256 MB of index data")
    ap.add_argument("--preheat", type=float, default=0.5,
                    help="seconds of the same calls before the warm-up calls, to bring the GPU to its clock")
    ap.add_argument("--repeats", type=int, default=8,
                    help="further timed regions of --steps calls each (events on the launch stream) for the median and minimum")
    ap.add_argument("--cols-per-wave", type=int, default=0, help="tuning runs: the cols_per_wave option of tstgemm_ex()")
    ap.add_argument("--k-slices", type=int, default=0, help="tuning runs: the k_slices option of tstgemm_ex()")
    ap.add_argument("--list-walk", type=int, default=0, help="tuning runs: the list_walk option of tstgemm_ex() (8 < M <= 64)")
    ap.add_argument("--wide-lists", action="store_true",
                    help="M <= 8: the decode_wide_lists option of tstgemm_ex() (the 32-bit TCSC lists instead of their 16-bit copy)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the measured-peak probes (roofline.peak_measured)")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run a plain 256 MiB copy kernel a few times (for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs: "
                         "what the counters read for it gives their scale)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2510_06957_amd as tg
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    wl = si.workload(args.workload)
    if args.variant != "tcsc" and wl.M > 8:
        print("bench.py: the signed and packed variants are small-M paths (M <= 8)", file=sys.stderr)
        sys.exit(2)
    gemm = {"tcsc": tg.tstgemm, "signed": tg.tstgemm_signed, "packed": tg.tstgemm_packed}[args.variant]
    W, X, b = si.make_workload(wl.name)
    t0 = time.perf_counter()
    t = tg.tcsc_build(W)
    build_ms = (time.perf_counter() - t0) * 1e3
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tg.tcsc_upload(t)
    torch.cuda.synchronize()
    upload_ms = (time.perf_counter() - t0) * 1e3
    nnz = t.nnz
    lay = tg.tcsc_layout(t)
    adds = wl.M * nnz
    # defaults: about 0.5 s of timed work for the headline workload, fewer steps for big ones
    est_ms = max(adds / 20e12 * 1e3, 0.01)
    steps = args.steps if args.steps is not None else int(min(5000, max(20, 500.0 / est_ms)))
    warmup = args.warmup if args.warmup is not None else 10

    decode = wl.M <= 8          # the library's rules for its decode kernel ...
    small = 8 < wl.M <= 64      # ... and its small-tile kernel
    # index data one call reads (what must not be in the Infinity Cache for an HBM figure)
    narrow = (decode and args.variant == "tcsc" and bool(lay.has_lists16) and not args.wide_lists
              and wl.K <= 150 * 1024 // (4 * wl.M) - 1)   # the library's rule for its padded 16-bit lists
    if args.variant == "packed":
        index_bytes = lay.n_chunks5 * lay.n_pad * 16
    elif decode:
        index_bytes = 2 * (lay.nnz16_pos + lay.nnz16_neg) if narrow else 4 * nnz
    elif small:
        index_bytes = 4 * nnz + 8 * (lay.n_cuts + 1) * lay.n_pad
    else:
        index_bytes = 16 * lay.n_kblocks * lay.n_pad
    n_copies = args.rotate
    if n_copies <= 0:
        n_copies = min(64, -(-3 * INFINITY_CACHE_BYTES // max(index_bytes, 1))) if decode else 1

    Xd = torch.from_numpy(X).cuda()
    bd = torch.from_numpy(b).cuda()
    Yd = torch.empty((wl.M, wl.N), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    copies = [t] + [tg.tcsc_upload(tg.tcsc_build(W)) for _ in range(n_copies - 1)]
    turn = [0]

    tuning = {k: v for k, v in (("cols_per_wave", args.cols_per_wave), ("k_slices", args.k_slices),
                                ("wide_lists", args.wide_lists), ("list_walk", args.list_walk)) if v}

    def gemm_next(**options):
        h = copies[turn[0] % len(copies)]
        turn[0] += 1
        gemm(Xd, h, bd, Yd, stream, **tuning, **options)

    if args.traffic_calibration:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")   # 256 MiB read, 256 MiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # clock ramp: the same calls for a fixed time, whatever --warmup says
    preheat_calls = 0
    t_end = time.perf_counter() + max(0.0, args.preheat)
    while time.perf_counter() < t_end:
        for _ in range(32):
            gemm_next()
        preheat_calls += 32
        torch.cuda.synchronize()
    for _ in range(warmup):
        gemm_next()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(steps):
        gemm_next()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps
    call_ms = ev0.elapsed_time(ev1) / steps      # HIP events on the launch stream around all K calls

    # further regions of the same length, back to back, for the spread: time per call of each region from its events
    region_ms = [call_ms]
    for _ in range(max(0, args.repeats)):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            gemm_next()
        e1.record(stream)
        torch.cuda.synchronize()
        region_ms.append(e0.elapsed_time(e1) / steps)

    # one matrix only, call after call: its index data stays in the Infinity Cache (labelled as such)
    warm_ms = None
    if len(copies) > 1:
        for _ in range(warmup):
            gemm(Xd, t, bd, Yd, stream, **tuning)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            gemm(Xd, t, bd, Yd, stream, **tuning)
        e1.record(stream)
        torch.cuda.synchronize()
        warm_ms = e0.elapsed_time(e1) / steps

    # The dominant kernel alone: the library records a pair of HIP events (an option of the call) around its launch, on the
    # launch stream, in every call of a second, equally long run (back to back as before, so the clocks stay up).
    n_k = max(min(steps, 1000), 20)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_k)]
    for a, c in pairs:
        a.record(stream)
        c.record(stream)
    torch.cuda.synchronize()
    for pair in pairs:
        gemm_next(events=pair)
    torch.cuda.synchronize()
    kernel_raw = np.array([a.elapsed_time(c) for a, c in pairs])
    # What an event pair reads with nothing between its two records, on the same busy stream: the cost of the
    # second record itself, which the pair around the kernel contains as well.
    for a, c in pairs:
        gemm_next()
        a.record(stream)
        c.record(stream)
    torch.cuda.synchronize()
    pair_ms = float(np.mean([a.elapsed_time(c) for a, c in pairs]))
    kernel_raw_ms = float(np.mean(kernel_raw))
    kernel_ms = kernel_raw_ms - pair_ms
    kernel_ms_median = float(np.median(kernel_raw)) - pair_ms
    kernel_ms_min = float(np.min(kernel_raw)) - pair_ms
    if decode:
        # The M <= 8 paths are ONE kernel per call: the time per call of the back-to-back timed region is that kernel's
        # time (with the gap between two launches), and it is what agrees with the profiler's average duration; the
        # event pair between two such kernels delays them and then takes off too much.
        kernel_ms, kernel_ms_median, kernel_ms_min = call_ms, float(np.median(region_ms)), float(np.min(region_ms))

    measured = MEASURED_TRAFFIC.get((wl.name, args.variant))
    traffic = measured[0] if measured else None
    if args.variant == "packed":
        # dense decode: every entry of the padded W costs one conversion and M multiply-adds on the vector ALUs
        # (256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-instructions/s); the codes are 1.6 bits per entry
        entries = lay.n_chunks5 * 80 * lay.n_pad
        alg_bytes = index_bytes + 4 * wl.M * wl.K + 4 * wl.M * wl.N + 4 * wl.N
        roof = {"bound": "alu", "achieved": entries * (wl.M + 1) / (kernel_ms * 1e-3) / 1e12, "peak": PEAK_ALU_INSTR_T,
                "unit": "T lane-instructions/s", "traffic": traffic,
                "note": "per entry of W (zeros included): 1 byte-to-float conversion + M fused multiply-adds, the form this "
                        "kernel chose (the conversion is its own overhead, not the method's); "
                        "peak = 256 CUs x 64 lanes x 2.4 GHz (one vector instruction per SIMD and 4 clocks)"}
    elif decode:
        # small-M path streams the index arrays once (TCSC: four arrays; signed: one pointer array less): index-bandwidth
        # bound.  tstgemm() reads the padded 16-bit copy of the lists where the matrix has one and X fits the LDS whole.
        alg_bytes = index_bytes + 8 * (wl.N + 1) + 4 * wl.M * wl.K + 4 * wl.M * wl.N + 4 * wl.N
        roof = {"bound": "hbm", "achieved": alg_bytes / (kernel_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                "unit": "GB/s", "traffic": traffic}
    else:
        # index data the kernel reads (small tile: the TCSC row numbers and the list cuts; else the 64-bit row sets)
        # + X + Y + b
        alg_bytes = index_bytes + 4 * wl.M * wl.K + 4 * wl.M * wl.N + 4 * wl.N
        roof = {"bound": "lds", "achieved": adds / (kernel_ms * 1e-3) / 1e12, "peak": PEAK_LDS_GATHER_TFLOPS,
                "unit": "TFLOP/s", "traffic": traffic,
                "note": "1 flop = 1 fp32 add = one 4-byte LDS gather; peak = LDS read port, 256 B/clk/CU x 256 CUs x "
                        "2.4 GHz; the fp32 add rate of the vector ALUs (alu_add_peak) is twice that",
                "alu_add_peak": PEAK_ALU_ADD_TFLOPS}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["kernel"] = ("k_packed" if args.variant == "packed" else "k_decode (signed lists)" if args.variant == "signed"
                      else "k_decode" if decode else "k_small" if small else "k_large")
    if decode and args.variant == "tcsc":
        roof["kernel"] += " (16-bit lists)" if narrow else " (32-bit lists)"
    roof["kernel_ms"] = kernel_ms
    roof["kernel_ms_median"] = kernel_ms_median
    roof["kernel_ms_min"] = kernel_ms_min
    roof["kernel_ms_event_pair"] = kernel_raw_ms     # as read from the event pair ...
    roof["empty_event_pair_ms"] = pair_ms            # ... minus what an empty pair reads = kernel_ms
    # HBM side of the same launch: measured bytes (counter runs) if there are any, else the algorithmic bytes
    hbm_bytes = traffic if traffic is not None else alg_bytes
    roof["hbm_gb_per_s"] = hbm_bytes / (kernel_ms * 1e-3) / 1e9
    roof["hbm_frac"] = roof["hbm_gb_per_s"] / PEAK_HBM_GBS
    roof["hbm_bytes_are"] = (f"constant from {measured[1]} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script; a counter "
                             "run cannot be part of a timed run, so not re-measured here)" if measured else "algorithmic")
    roof["algorithmic_adds_per_launch"] = adds
    roof["algorithmic_bytes_per_launch"] = alg_bytes
    # the same accounting for the whole call (packing pre-pass + main kernel + split-K reduction)
    roof["call_ms"] = call_ms
    roof["call_ms_median"] = float(np.median(region_ms))
    roof["call_ms_min"] = float(np.min(region_ms))
    roof["call_frac"] = roof["frac"] * kernel_ms / call_ms   # the same work over the time of the whole call
    if not decode:
        roof["alu_frac"] = roof["achieved"] / PEAK_ALU_ADD_TFLOPS
        # What this build can reach at most: without packed fp32 a compute unit issues one vector instruction per
        # clock (64 lanes), which is the same 39.3 T lane-operations/s as the LDS port's gathers, and every 16-byte
        # gather costs four additions and one address instruction.  C5a runs on this bound (0.80 of the LDS roofline),
        # C2 at nine tenths of it (counters: profiles/shader_counters_all_configs.md).
        roof["valu_issue_bound"] = PEAK_LDS_GATHER_TFLOPS * 4.0 / 5.0
        roof["frac_of_valu_issue_bound"] = roof["achieved"] / roof["valu_issue_bound"]
    if not decode and not small:
        # Bytes the main kernel copies from the packed X (in the L2s) into the LDS: every workgroup one K-block of its
        # row tile (64 rows of W x TM rows of X x 4 bytes) per K-block it walks, whatever the density.  The columns
        # per workgroup follow the library's own rule for its launch shape (tstgemm_large.hip, choose_shape), restated
        # here; an override on the command line takes its place.
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        tm = 128 if wl.M <= 128 else 256
        m_tiles = -(-wl.M // tm)
        ncw = args.cols_per_wave or large_cols_per_wave(m_tiles, lay.n_pad, nnz / (wl.K * wl.N), cus)
        if ncw == 8 and lay.n_pad % 128:
            ncw = 4
        tile_bytes = m_tiles * (lay.n_pad // (16 * ncw)) * lay.n_kblocks * 64 * tm * 4
        roof["tile_copy"] = {"columns_per_workgroup": 16 * ncw, "bytes_per_launch": tile_bytes,
                             "tb_per_s": tile_bytes / (kernel_ms * 1e-3) / 1e12,
                             "note": "packed X from the L2s into the LDS, one K-block of a row tile per workgroup and K-block"}
    if warm_ms is not None:
        roof["warm_cache_call_ms"] = warm_ms
        roof["warm_cache_note"] = ("one matrix called again and again: its index data comes from the 256 MB Infinity Cache, "
                                   "not from HBM; every other figure of this line rotates over the copies")
    if not args.no_probes:
        pk = measured_peaks(tg, torch, stream, index_bytes)
        roof["peak_measured"] = pk
        if "tile_copy" in roof:
            # how much of what the copies alone can reach the kernel's copies take: at low density this, not the
            # gathers, is what the main kernel is made of
            roof["tile_copy"]["frac_of_measured_copy_rate"] = roof["tile_copy"]["tb_per_s"] / pk["tile_copy_tb_per_s"]
        if roof["bound"] == "lds":
            roof["frac_of_measured_peak"] = roof["achieved"] / pk["lds_gather_tadds_per_s"]
            roof["call_frac_of_measured_peak"] = roof["frac_of_measured_peak"] * kernel_ms / call_ms
        elif roof["bound"] == "hbm":
            roof["frac_of_measured_peak"] = roof["achieved"] / pk["hbm_stream_read_gb_per_s"]

    out = {
        "metric": "effective Gadds/s (M*nnz(W)), fp32 X, sparse ternary GEMM Y = XW + b",
        "value": adds / (ms_per_step * 1e-3) / 1e9,
        "unit": "Gadds/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": float(np.median(region_ms)), "ms_per_step_min": float(np.min(region_ms)),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: M={wl.M} K={wl.K} N={wl.N} density={wl.density} X,b~{wl.dist} "
                               f"seed={wl.seed}", "nnz": nnz, "variant": args.variant, "matrix_copies_in_rotation": len(copies),
                   "index_bytes_per_call": int(index_bytes), "launch_shape_overrides": tuning or None,
                   "preheat_s": args.preheat, "preheat_calls": preheat_calls, "timed_regions": len(region_ms),
                   "spread": "ms_per_step is the wall clock over the first region of `steps` calls; median / min are over "
                             "the time per call of all regions (events on the launch stream)",
                   "index_type": "int32 TCSC in; on device the TCSC arrays or their padded 16-bit copy (M <= 64), or 64-bit row sets "
                                 "per K-block",
                   "tcsc_build_ms_host": build_ms, "upload_and_reblock_ms": upload_ms},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(W, X, b, nnz, args.variant)
        out["cpu_baseline"]["paper_context"] = ("paper, Apple M1, one core: best scalar kernel 5.98x its BaseTCSC and 50.2 % of a "
                                                "4-fadd/cycle peak (M=64, K=16384, N=4096, 50 %; Sec. 4) -- other hardware, "
                                                "not a target")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
