#!/usr/bin/env python3
"""Benchmark of the sparse-MTTKRP hot path on one MI355X.

One step = mode-n MTTKRP for every mode n of one synthetic tensor (output definition, COO-group,
CSL-group and B-CSF-group kernels per mode), inputs resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--only-headline]

GFLOP/s uses 3*R*nnz floating-point operations per mode (the COO operation count of Section
III-A), R = 32.  The roofline entry is for the B-CSF-group kernel and prices its algorithmic
bytes (its format arrays once + each distinct factor row it gathers once + each output row it
writes once) against the 8 TB/s HBM peak.
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

HBM_PEAK_GBS = 8000.0
# The published fp32 vector peak (157.3 TFLOP/s) counts a packed two-wide FMA on every lane; this build turns packed
# fp32 formation off, so the vector ALUs can retire one FMA per lane and cycle: half of the published figure
# (256 CUs x 4 SIMDs x 16 lanes x 2 flops x 2.4 GHz = 78.6 TFLOP/s).
FP32_VECTOR_PEAK_GFLOPS = 157300.0 / 2
FP64_VECTOR_PEAK_GFLOPS = 78600.0   # published fp64 vector peak: one FMA per lane and cycle
KERNELS = ("define", "coo", "csl", "csf")
OTHER_WORKLOADS = ("cfg3", "cfg4", "cfg2")   # measured after the headline workload, same process
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def measured_traffic(workload: str):
    """HBM-side bytes per B-CSF-kernel launch (mean over the modes) from profiles/traffic.json, which
    `bench.py --ingest-counters` writes from two rocprofv3 --pmc runs of this script (FETCH_SIZE, WRITE_SIZE, each
    scaled by what the same counter reads for a plain copy of known size).  None when the file has no entry."""
    try:
        with open(TRAFFIC_FILE) as f:
            entry = json.load(f)["workloads"].get(workload)
    except (OSError, ValueError, KeyError):
        return None
    return None if entry is None else entry["csf_bytes_per_launch"]


def ingest_counters(fetch_csv: str, write_csv: str, workload: str, commit: str, log) -> int:
    """Reads the counter_collection CSVs of `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of
    `bench.py --workload W --only-headline` and stores, per kernel of the library, the mean KiB per launch and the scaled
    bytes in profiles/traffic.json under workload W (other workloads' entries are kept)."""
    import collections
    import csv

    scale = {"FETCH_SIZE": 2.0, "WRITE_SIZE": 1.0}   # counter reading for a 1 GiB copy: 0.5 GiB read, 1 GiB written
    per_kernel = collections.defaultdict(dict)
    for path, counter in ((fetch_csv, "FETCH_SIZE"), (write_csv, "WRITE_SIZE")):
        acc = collections.defaultdict(list)
        with open(path) as f:
            for r in csv.DictReader(f):
                if r["Counter_Name"] == counter and "hbcsf::" in r["Kernel_Name"]:
                    acc[r["Kernel_Name"].split("(")[0].replace("void ", "")].append(float(r["Counter_Value"]))
        for k, v in acc.items():
            per_kernel[k][counter] = {"kib_per_launch": round(sum(v) / len(v), 1), "launches": len(v)}
    entry = {"commit": commit, "scale": scale, "kernels": per_kernel, "csf_bytes_per_launch": None,
             "command": "rocprofv3 --pmc <FETCH_SIZE | WRITE_SIZE> --output-format csv -d <dir> -o t -- python3 bench.py "
                        f"--workload {workload} --only-headline --no-cpu-baseline --als-iterations 0 --steps 3 --warmup 1"}
    for k, c in per_kernel.items():
        if "csf_group_kernel" in k and "FETCH_SIZE" in c and "WRITE_SIZE" in c:
            entry["csf_kernel"] = k
            entry["csf_bytes_per_launch"] = round(1024 * (scale["FETCH_SIZE"] * c["FETCH_SIZE"]["kib_per_launch"]
                                                          + scale["WRITE_SIZE"] * c["WRITE_SIZE"]["kib_per_launch"]))
    try:
        with open(TRAFFIC_FILE) as f:
            doc = json.load(f)
    except (OSError, ValueError):
        doc = {"what": "HBM-side traffic per kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch as "
                       "reported, mean over all launches of the run), written by `python bench.py --ingest-counters`",
               "workloads": {}}
    doc["workloads"][workload] = entry
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(doc, f, indent=1, sort_keys=True)
        f.write("\n")
    log(f"[bench] {TRAFFIC_FILE}: {workload}: {json.dumps(entry)}")
    return 0


def algorithmic_bytes(st: dict, rank: int, order: int, elem: int = 4) -> dict:
    """Algorithmic HBM bytes of one mode's kernels from the builder's statistics (elem = bytes per factor element)."""
    row = elem * rank
    rows_total = st["rows"]
    out = {}
    for g, name in enumerate(("coo", "csl", "csf")):
        if st["group_nnz"][g] == 0:
            out[name] = 0
            continue
        gathered = sum(st["distinct_rows"][g][l] for l in range(1, order))
        out[name] = st["stream_bytes"][g] + row * gathered + row * st["group_slices"][g]
    # define kernel: the owned-row bitmap once + every row no kernel stores (zero fill)
    out["define"] = 4 * ((rows_total + 31) // 32) + row * (rows_total - st["owned_rows"])
    # the whole mode: format arrays and distinct factor rows per kernel, plus the dense output exactly once (a row
    # that several kernels or pieces add to is still one row) and the owned-row bitmap
    out["total"] = (sum(out[k] - row * st["group_slices"][g] for g, k in enumerate(("coo", "csl", "csf")) if out[k])
                    + 4 * ((rows_total + 31) // 32) + row * rows_total)
    return out


def gather_bytes(st: dict, rank: int, order: int, elem: int = 4) -> int:
    """Bytes through the cache hierarchy when every row gather is counted (not HBM bytes): format arrays +
    one factor row per leaf-level gather and per fiber-segment gather + the output once."""
    row = elem * rank
    coo, csl, csf = st["group_nnz"]
    gathers = (order - 1) * (coo + csl) + csf + sum(st["segments"][: order - 2])
    return sum(st["stream_bytes"]) + row * gathers + row * st["rows"]


def calibrate(torch, log) -> int:
    """Attainable bandwidth of plain streaming kernels, and a known-size copy for counter scaling."""
    n = 1 << 28  # 2^28 floats = 1 GiB
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    res = {}
    for name, fn, nbytes in (("copy_1GiB", lambda: dst.copy_(src), 2 * 4 * n),
                             ("fill_1GiB", lambda: dst.zero_(), 4 * n),
                             ("read_1GiB", lambda: src.sum(), 4 * n)):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 10
        res[name] = {"ms": round(dt * 1e3, 4), "GB/s": round(nbytes / dt / 1e9, 1), "bytes": nbytes}
        log(f"[calibrate] {name}: {res[name]}")
    # Row-gather ceiling: 128-byte rows from tables of growing size, no MTTKRP work.  Uniform row numbers, and
    # bounded-Zipf ones (the index laws of the benchmark tensors: popular rows are re-gathered while still cached).
    import numpy as np

    from paper_1904_03329_amd import binding as B

    n = 1 << 26
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(7)
    cases = [(256, 0.0), (18_000, 0.0), (1_000_000, 0.0), (40_000_000, 0.0),
             (2_000, 1.1), (18_000, 1.1), (50_000, 1.1), (40_000_000, 1.05)]
    for rows, alpha in cases:
        table = torch.zeros((rows, 32), dtype=torch.float32, device="cuda")
        if alpha > 0:
            cdf = np.cumsum(np.arange(1, rows + 1, dtype=np.float64) ** -alpha)
            rank = np.searchsorted(cdf, rng.uniform(0.0, cdf[-1], size=n)).astype(np.int64)
            rank = np.minimum(rank, rows - 1)
            idx = torch.from_numpy(((rank * 2654435761) % rows).astype(np.int32)).cuda()   # popular rows scattered
            del cdf, rank
        else:
            idx = torch.randint(0, rows, (n,), dtype=torch.int64, device="cuda").to(torch.int32)
        stream = torch.cuda.current_stream().cuda_stream
        law = f"zipf{alpha}" if alpha > 0 else "uniform"
        # 8: every lane of a load instruction gathers; 2 / 1 (small tables only): the B-CSF kernel's fiber-row
        # loads, which only the lane groups whose segment ends at that step execute
        for active in ((8, 2, 1) if rows <= 18_000 and alpha == 0 else (8,)):
            got, instr = B.probe_row_gather(idx.data_ptr(), n, table.data_ptr(), rows, sink.data_ptr(), stream, active)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                B.probe_row_gather(idx.data_ptr(), n, table.data_ptr(), rows, sink.data_ptr(), stream, active)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / 5
            key = f"gather_rows_{rows}_{law}" + ("" if active == 8 else f"_active{active}of8")
            res[key] = {"ms": round(dt * 1e3, 4), "Grows/s": round(got / dt / 1e9, 1),
                        "GB/s": round(got * 128 / dt / 1e9, 1), "table_MB": round(rows * 128 / 1e6, 1),
                        "active_lane_groups": active, "G_load_instr/s": round(instr / dt / 1e9, 2),
                        "ns_per_load_instr_per_CU": round(dt * 1e9 * torch.cuda.get_device_properties(0).multi_processor_count / instr, 2)}
            log(f"[calibrate] gather, {law} over {rows} rows, {active} of 8 lane groups per load: {res[key]}")
        del table, idx
    print(json.dumps({"calibrate": res}), flush=True)
    return 0


def trace_cu_spread(torch, np, B, ht, dfacs, outs, order, log):
    """Per-CU busy time (union of its wavefronts' [start, end] intervals) of the CSL and B-CSF kernels."""
    cap = 1 << 20
    buf = torch.zeros(4 + 4 * cap, dtype=torch.int64, device="cuda")
    B.tune(ht.handle, B.TUNE_TRACE_CAPACITY, cap)
    B.tune(ht.handle, B.TUNE_TRACE_BUFFER, buf.data_ptr())
    result = []
    for m in range(order):
        buf[0] = 0
        ht.mttkrp(m, dfacs, outs[m])
        torch.cuda.synchronize()
        n = min(int(buf[0].item()), cap)
        rec = buf[4:4 + 4 * n].cpu().numpy().reshape(n, 4)
        for kind, name in ((1, "csl"), (2, "csf")):
            r = rec[rec[:, 0] == kind]
            if r.shape[0] == 0:
                continue
            hw = r[:, 1] & 0xFFFFFFFF
            xcc = r[:, 1] >> 32
            cu_key = (xcc << 8) | (((hw >> 13) & 7) << 5) | (((hw >> 12) & 1) << 4) | ((hw >> 8) & 15)
            t0 = int(r[:, 2].min())
            span = (int(r[:, 3].max()) - t0) / 100.0  # wall clock ticks are 10 ns -> microseconds
            busy = []
            for key in np.unique(cu_key):
                iv = r[cu_key == key][:, 2:4]
                iv = iv[np.argsort(iv[:, 0])]
                total, cur_s, cur_e = 0, int(iv[0, 0]), int(iv[0, 1])
                for a, b in iv[1:]:
                    if a > cur_e:
                        total += cur_e - cur_s
                        cur_s, cur_e = int(a), int(b)
                    else:
                        cur_e = max(cur_e, int(b))
                busy.append((total + cur_e - cur_s) / 100.0)
            busy = np.asarray(busy)
            entry = {"mode": m, "kernel": name, "wavefronts": int(r.shape[0]), "cus": int(busy.size),
                     "makespan_us": round(span, 1), "busy_us_mean": round(float(busy.mean()), 1),
                     "busy_us_min": round(float(busy.min()), 1), "busy_us_max": round(float(busy.max()), 1),
                     "max_over_mean": round(float(busy.max() / busy.mean()), 4),
                     "cv": round(float(busy.std() / busy.mean()), 4)}
            result.append(entry)
            log(f"[bench] per-CU busy spread: {entry}")
    B.tune(ht.handle, B.TUNE_TRACE_BUFFER, 0)
    return result


def time_device_build(torch, np, B, HbcsfTensor, t, host_tensor, args, log):
    """Pre-processing on the GPU (the cost Section VI-E weighs against the MTTKRP time): the same format built by
    the device-side builder from COO arrays resident in HBM.  Two builds; the first also loads the sort / scan
    code objects.  Returns None when the packed coordinate does not fit 64 bits (host builder only)."""
    t0 = time.perf_counter()
    di = [torch.from_numpy(x.view(np.int32)).cuda() for x in t.inds]
    dv = torch.from_numpy(t.vals).cuda()
    torch.cuda.synchronize()
    upload_s = time.perf_counter() - t0
    times = []
    try:
        for _ in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            dev = HbcsfTensor.from_device_coo(t.dims, di, dv, compact=False, fiber_threshold=args.fiber_threshold,
                                              slice_threshold=args.slice_threshold,
                                              mode_order_policy=args.mode_order_policy, group_mask=args.group_mask,
                                              coo_row_flags=args.coo_row_flags, mid_blocking=args.mid_blocking,
                                              hybrid_granularity=args.hybrid_granularity)
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t0)
            same = B.device_bytes(dev.handle) == B.device_bytes(host_tensor.handle)
            dev.close()
    except B.HbcsfError as e:
        log(f"[bench] device build not available for this tensor: {e}")
        return None
    report = {"seconds": round(min(times), 4), "first_call_seconds": round(times[0], 4),
              "coo_upload_seconds": round(upload_s, 3), "same_bytes_as_host_build": bool(same)}
    log(f"[bench] device-side format build: {report}")
    return report


def time_als(torch, ht, dfacs, rank, iterations, build_s, dev_build, log):
    """CPD-ALS iterations (Algorithm "CPD-ALS") from copies of the benchmark's factor matrices: wall time per
    iteration with the factors' Gram matrices carried over (the steady state of a decomposition), and the
    library's own split into MTTKRP / Gram / host / product time."""
    from paper_1904_03329_amd import CpdAls

    facs = [f.clone() for f in dfacs]
    als = CpdAls(ht, rank)
    fits, wall, phases = [], [], []
    for it in range(iterations + 1):          # the first iteration also computes the initial Gram matrices
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        # as the algorithm's outer loop runs them: the closing normalisation is put off to the end of the loop
        fits.append(als.iteration(facs, keep_grams=it > 0, lazy=True))
        wall.append(1e3 * (time.perf_counter() - t0))
        phases.append(als.phase_ms())
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    als.normalise(facs)
    torch.cuda.synchronize()
    normalise_ms = 1e3 * (time.perf_counter() - t0)
    als.close()
    steady = wall[1:]
    ph = [sum(p[k] for p in phases[1:]) / len(steady) for k in range(4)]
    ms = sum(steady) / len(steady)
    rows = sum(ht.dims)
    dense_bytes = 2.0 * rows * rank * 4       # per iteration: the product kernel reads M and writes the factor
    report = {
        "iterations": iterations,
        "ms_per_iteration": round(ms, 3),
        "first_iteration_ms": round(wall[0], 3),
        "closing_normalisation_ms": round(normalise_ms, 3),
        "phase_ms": {"mttkrp": round(ph[0], 3), "gram": round(ph[1], 3), "host": round(ph[2], 3),
                     "product": round(ph[3], 3)},
        "mttkrp_share": round(ph[0] / max(sum(ph), 1e-9), 3),
        "dense_pass_gbs": round(dense_bytes / max((ph[1] + ph[3]) * 1e-3, 1e-12) / 1e9, 1),
        "fit": [round(f, 6) for f in fits],
        "iterations_to_equal_host_build_time": round(build_s * 1e3 / ms, 1),
        "iterations_to_equal_device_build_time": round(dev_build["seconds"] * 1e3 / ms, 1) if dev_build else None,
    }
    log(f"[bench] als: {json.dumps(report)}")
    return report


def cpu_baseline_of(np, t, facs, rank, order, log):
    """The oracle as it stands, timed on the host: single thread (the parity reference) on a bounded sample, then
    the same loop on every host core with atomic adds (oracle/mttkrp_oracle_omp.c).  A reported baseline only."""
    import oracle  # test infrastructure: used here for the reported CPU baseline only

    sample = min(t.nnz, 30_000_000)
    si = [x[:sample] for x in t.inds]
    sv = t.vals[:sample]
    t0 = time.perf_counter()
    for m in range(order):
        oracle.mttkrp(t.dims, si, sv, facs, m)
    cpu_s = time.perf_counter() - t0
    base = {
        "value": round(3.0 * rank * sample * order / cpu_s / 1e9, 3),
        "unit": "GFLOP/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"first {sample} of {t.nnz} nonzeros (generator order), all {order} modes, {cpu_s:.1f}s",
    }
    t0 = time.perf_counter()
    threads = 1
    for m in range(order):
        _, threads = oracle.mttkrp_all_cores(t.dims, si, sv, facs, m)
    omp_s = time.perf_counter() - t0
    base["all_cores"] = {
        "value": round(3.0 * rank * sample * order / omp_s / 1e9, 3),
        "unit": "GFLOP/s",
        "cores": threads,
        "kind": "oracle loop split over the host cores with atomic fp64 adds",
        "sample": f"the same {sample} nonzeros, all {order} modes, {omp_s:.1f}s",
    }
    log(f"[bench] cpu baseline: {base}")
    return base


def measure_single_representation(torch, np, B, HbcsfTensor, t, facs, rank, full_bytes, steps, log) -> dict:
    """The single-representation variant (one stored tree instead of one per mode) on the same tensor: device bytes
    and milliseconds per mode, timed with events on the launch stream (torch's current stream)."""
    t0 = time.time()
    ht = HbcsfTensor(t.dims, t.inds, t.vals, single_representation=1).to_device()
    build_s = time.time() - t0
    dfacs = [torch.from_numpy(f).cuda() for f in facs]
    outs = [torch.empty((t.dims[m], rank), dtype=torch.float32, device="cuda") for m in range(t.order)]
    ms = []
    for m in range(t.order):
        ht.mttkrp(m, dfacs, outs[m])
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            ht.mttkrp(m, dfacs, outs[m])
        b.record()
        torch.cuda.synchronize()
        ms.append(a.elapsed_time(b) / steps)
    res = {"device_bytes": B.device_bytes(ht.handle), "device_bytes_one_per_mode": full_bytes,
           "build_seconds": round(build_s, 2), "mode_ms": [round(x, 4) for x in ms],
           "ms_per_step": round(sum(ms), 4),
           "value": round(3.0 * rank * t.nnz * t.order / (sum(ms) * 1e-3) / 1e9, 1)}
    ht.close()
    log(f"[bench] single representation: {json.dumps(res)}")
    return res


def measure(name: str, args, headline: bool, log) -> dict:
    """Generates one workload, builds and uploads its format and times `args.steps` steps (one step = MTTKRP on
    every mode).  The headline workload also gets the device-side build, the CPD-ALS iterations, the per-CU
    trace (on request) and the CPU baseline; the others are timed only."""
    import numpy as np
    import torch

    import synthgen
    from paper_1904_03329_amd import HbcsfTensor, binding as B

    w = synthgen.WORKLOADS[name]
    t0 = time.time()
    t, facs, rank = synthgen.workload(name)
    if args.rank and args.rank != rank:   # the workload's tensor with factor matrices of another rank
        rank = args.rank
        facs = synthgen.factors(t.dims, rank, w.seed)
    gen_s = time.time() - t0
    log(f"[bench] {name}: dims={t.dims} nnz={t.nnz} draws={t.draws} R={rank} generated in {gen_s:.1f}s")
    t0 = time.time()
    ht = HbcsfTensor(t.dims, t.inds, t.vals, fiber_threshold=args.fiber_threshold,
                     slice_threshold=args.slice_threshold, mode_order_policy=args.mode_order_policy,
                     group_mask=args.group_mask, hybrid_granularity=args.hybrid_granularity,
                     coo_row_flags=args.coo_row_flags, mid_blocking=args.mid_blocking)
    build_s = time.time() - t0
    t0 = time.time()
    ht.to_device()
    upload_s = time.time() - t0
    order = t.order
    stats = []
    for m in range(order):
        st = ht.stats(m)
        st["rows"] = t.dims[m]
        stats.append(st)
    log(f"[bench] format built in {build_s:.1f}s, uploaded {B.device_bytes(ht.handle) / 1e9:.2f} GB in {upload_s:.1f}s")
    dev_build = time_device_build(torch, np, B, HbcsfTensor, t, ht, args, log) if headline else None
    f64 = args.dtype == "f64"
    elem = 8 if f64 else 4
    dfacs = [torch.from_numpy(f).cuda().double() if f64 else torch.from_numpy(f).cuda() for f in facs]
    outs = [torch.empty((t.dims[m], rank), dtype=torch.float64 if f64 else torch.float32, device="cuda")
            for m in range(order)]

    def step():
        for m in range(order):
            ht.mttkrp(m, dfacs, outs[m])

    if args.waves_per_cu:
        B.tune(ht.handle, B.TUNE_WAVES_PER_CU, args.waves_per_cu)
    if args.kernel_steps:
        B.tune(ht.handle, B.TUNE_STEPS, args.kernel_steps)
    if args.fiber_row_gather:
        B.tune(ht.handle, B.TUNE_DENSE_MID, args.fiber_row_gather)
    if args.fuse_coo >= 0:
        B.tune(ht.handle, B.TUNE_FUSE_COO, args.fuse_coo)
    B.tune(ht.handle, B.TUNE_PROFILE, order * args.steps)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.tune(ht.handle, B.TUNE_PROFILE, order * args.steps)  # restart the ring: timed calls only
    t_begin = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_begin
    ms_per_step = 1e3 * elapsed / args.steps

    # per-kernel durations of every timed call, from the HIP events the library recorded on the
    # launch stream inside the timed region
    kms = np.zeros((args.steps, order, 4))
    for s in range(args.steps):
        for m in range(order):
            back = (args.steps - 1 - s) * order + (order - 1 - m)
            kms[s, m] = B.kernel_ms(ht.handle, back)
    kmean = kms.mean(axis=0)  # [mode][kernel]

    flops_mode = 3.0 * rank * t.nnz
    value = flops_mode * order / (ms_per_step * 1e-3) / 1e9
    per_mode = []
    csf_bytes, csf_ms, csf_launches = 0.0, 0.0, 0
    for m in range(order):
        ab = algorithmic_bytes(stats[m], rank, order, elem)
        tot_ms = float(kmean[m].sum())
        entry = {
            "mode": m,
            "level_modes": stats[m]["level_mode"][:order],
            "ms": round(tot_ms, 4),
            "gflops_3Rnnz": round(flops_mode / (tot_ms * 1e-3) / 1e9, 1),
            "model_bytes": ab["total"],
            "hbm_gbs_model": round(ab["total"] / (tot_ms * 1e-3) / 1e9, 1),
            "hbm_frac": round(ab["total"] / (tot_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "kernel_ms": {k: round(float(kmean[m][i]), 4) for i, k in enumerate(KERNELS)},
            "kernel_model_bytes": {k: ab[k] for k in KERNELS},
            "group_nnz": stats[m]["group_nnz"],
            "slices": stats[m]["slices"],
            "segments": stats[m]["segments"][: order - 2],
            "shared_slices": stats[m]["shared_slices"],
            "real_gflops": round(stats[m]["flops_real"] * rank / (tot_ms * 1e-3) / 1e9, 1),
        }
        # the two roofs side by side: time the algorithmic bytes need at the HBM peak, time the multiply-adds really
        # done need at the vector fp32 peak without packed FMA, and the larger of the two over the measured time
        t_hbm = ab["total"] / (HBM_PEAK_GBS * 1e9) * 1e3
        t_alu = stats[m]["flops_real"] * rank / ((FP64_VECTOR_PEAK_GFLOPS if f64 else FP32_VECTOR_PEAK_GFLOPS) * 1e9) * 1e3
        gb = gather_bytes(stats[m], rank, order, elem)
        entry.update({"t_hbm_ms": round(t_hbm, 4), "t_alu_ms": round(t_alu, 4),
                      "roof_frac": round(max(t_hbm, t_alu) / tot_ms, 4),
                      "gather_model_bytes": gb, "gather_gbs": round(gb / (tot_ms * 1e-3) / 1e9, 1)})
        if order == 4:
            entry["gflops_4Rnnz"] = round(4.0 * rank * t.nnz / (tot_ms * 1e-3) / 1e9, 1)
        per_mode.append(entry)
        if stats[m]["group_nnz"][2] > 0:
            csf_bytes += ab["csf"]
            csf_ms += float(kmean[m][3])
            csf_launches += 1
        log(f"[bench] {name} mode {m}: {json.dumps(entry)}")

    achieved = csf_bytes / (csf_ms * 1e-3) / 1e9 if csf_ms > 0 else 0.0
    roofline = {
        "kernel": f"{'f64::' if f64 else ''}csf_group_kernel<{rank * elem // 16},{order}>",
        "bound": "hbm",
        "achieved": round(achieved, 1),
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": None if f64 else measured_traffic(name),
        "bytes_per_launch": round(csf_bytes / max(csf_launches, 1)),
        "ms_per_launch": round(csf_ms / max(csf_launches, 1), 4),
        "launches_per_step": csf_launches,
    }
    res = {
        "workload": f"{name}: order {order}, dims {'x'.join(str(d) for d in t.dims)}, nnz {t.nnz}, "
                    f"Zipf alphas {list(w.alpha)}, R={rank}",
        "value": round(value, 1),
        "ms_per_step": round(ms_per_step, 4),
        "hbm_gbs_model_all_modes": round(sum(p["model_bytes"] for p in per_mode) / (ms_per_step * 1e-3) / 1e9, 1),
        "roof_frac_all_modes": round(sum(max(p["t_hbm_ms"], p["t_alu_ms"]) for p in per_mode) / ms_per_step, 4),
        "fiber_threshold": stats[0]["fiber_threshold"],
        "order": order,
        "build_seconds": round(build_s, 2),
        "upload_seconds": round(upload_s, 2),
        "generate_seconds": round(gen_s, 2),
        "device_build": dev_build,
        "per_mode": per_mode,
        "roofline": roofline,
    }
    if order == 4:
        res["value_4Rnnz"] = round(value * 4.0 / 3.0, 1)
    if headline and args.single_representation:
        res["single_representation"] = measure_single_representation(torch, np, B, HbcsfTensor, t, facs, rank,
                                                                     B.device_bytes(ht.handle), 5, log)
    if headline:
        if args.cu_spread:
            res["cu_busy_spread"] = trace_cu_spread(torch, np, B, ht, dfacs, outs, order, log)
        res["als"] = (time_als(torch, ht, dfacs, rank, args.als_iterations, build_s, dev_build, log)
                      if args.als_iterations > 0 and not f64 else None)
    del outs, dfacs
    ht.close()
    torch.cuda.empty_cache()
    if headline:
        res["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline_of(np, t, facs, rank, order, log)
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5", help="cfg1..cfg5: the headline workload (default: the largest, cfg5)")
    ap.add_argument("--only-headline", action="store_true",
                    help="do not measure the other workloads (cfg3, cfg4, cfg2) after the headline one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fiber-threshold", type=int, default=0)
    ap.add_argument("--slice-threshold", type=int, default=0)
    ap.add_argument("--mode-order-policy", type=int, default=0)
    ap.add_argument("--group-mask", type=int, default=0)
    ap.add_argument("--single-representation", action="store_true",
                    help="also time the single-representation variant (only mode 0's tree stored) on the headline "
                         "workload and report its device bytes and per-mode times under \"single_representation\"")
    ap.add_argument("--mid-blocking", type=int, default=0,
                    help="blocking of the first fiber level: 0 off, 2..13 bits (2^bits blocks) in every mode")
    ap.add_argument("--coo-row-flags", type=int, default=0,
                    help="1: the COO group stores row flags instead of a root index per nonzero")
    ap.add_argument("--hybrid-granularity", type=int, default=0,
                    help="1: COO / CSL / CSF chosen per fiber inside heavy slices (host builder only)")
    ap.add_argument("--waves-per-cu", type=int, default=0)
    ap.add_argument("--kernel-steps", type=int, default=0)
    ap.add_argument("--fuse-coo", type=int, default=-1,
                    help="HBCSF_TUNE_FUSE_COO: 0 separate COO kernel, 1 COO rows in the output-definition pass, 2 that "
                         "for small outputs (library default)")
    ap.add_argument("--rank", type=int, default=0,
                    help="factor-matrix rank other than the workload's 32 (8, 16, 64, 128; fp64: 16, 64); the ALS "
                         "timing then uses the plain vector-ALU dense kernels")
    ap.add_argument("--dtype", choices=("f32", "f64"), default="f32",
                    help="element type of the factor matrices, partial sums and output (f64: hbcsf_mttkrp_f64; the "
                         "ALS timing and the single-representation comparison are fp32 only)")
    ap.add_argument("--fiber-row-gather", type=int, default=0,
                    help="B-CSF kernel variant: 1 = fiber-level rows gathered through an LDS row cache")
    ap.add_argument("--als-iterations", type=int, default=3,
                    help="after the timed MTTKRP steps, time this many CPD-ALS iterations built on the same "
                         "library (reported under \"als\", not part of `value`); 0 skips them")
    ap.add_argument("--cu-spread", action="store_true",
                    help="after the timed steps, trace every wavefront of one more pass and report the "
                         "per-CU busy-time spread of the CSL and B-CSF kernels (profiling only)")
    ap.add_argument("--calibrate", action="store_true",
                    help="time a plain 1 GiB device copy, fill and read instead of the benchmark "
                         "(also the known-size kernel that scales the rocprofv3 byte counters)")
    ap.add_argument("--ingest-counters", nargs=3, metavar=("FETCH_CSV", "WRITE_CSV", "COMMIT"),
                    help="no GPU work: read the counter_collection CSVs of two rocprofv3 --pmc runs of this script "
                         "(FETCH_SIZE, WRITE_SIZE) for --workload and record them in profiles/traffic.json")
    args = ap.parse_args()
    log = lambda *a: print(*a, file=sys.stderr, flush=True)
    if args.ingest_counters:
        return ingest_counters(args.ingest_counters[0], args.ingest_counters[1], args.workload,
                               args.ingest_counters[2], log)
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.calibrate:
        return calibrate(torch, log)

    head = measure(args.workload, args, True, log)
    others = {}
    if not args.only_headline:
        for name in OTHER_WORKLOADS:
            if name == args.workload:
                continue
            r = measure(name, args, False, log)
            # the compact form: per-mode detail stays in the log
            others[name] = {k: r[k] for k in ("workload", "value", "ms_per_step", "hbm_gbs_model_all_modes",
                                              "roof_frac_all_modes", "fiber_threshold", "roofline")}
            if "value_4Rnnz" in r:
                others[name]["value_4Rnnz"] = r["value_4Rnnz"]
            others[name]["mode_ms"] = [p["ms"] for p in r["per_mode"]]
            others[name]["mode_hbm_frac"] = [p["hbm_frac"] for p in r["per_mode"]]
            others[name]["mode_gather_gbs"] = [p["gather_gbs"] for p in r["per_mode"]]

    order = head["order"]
    line = {
        "metric": f"sparse MTTKRP GFLOP/s (3*R*nnz per mode, all modes) at rank R={args.rank or 32}",
        "value": head["value"],
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.dtype,
        "data": "synthetic",
        "config": {
            "workload": head["workload"],
            "fiber_threshold": head["fiber_threshold"],
            "step": f"MTTKRP on all {order} modes",
            "hbm_gbs_model_all_modes": head["hbm_gbs_model_all_modes"],
            "roof_frac_all_modes": head["roof_frac_all_modes"],
            "build_seconds": head["build_seconds"],
            "device_build": head["device_build"],
            "upload_seconds": head["upload_seconds"],
            "generate_seconds": head["generate_seconds"],
        },
        "per_mode": head["per_mode"],
        "roofline": head["roofline"],
        "cpu_baseline": head["cpu_baseline"],
        "als": head["als"],
        "other_workloads": others,
    }
    if "cu_busy_spread" in head:
        line["cu_busy_spread"] = head["cu_busy_spread"]
    if "single_representation" in head:
        line["single_representation"] = head["single_representation"]
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
