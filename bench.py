#!/usr/bin/env python3
"""Benchmark of the balanced sparse kernels on one MI355X.

`python bench.py --gpus 1 --steps K --warmup W` prints ONE JSON line.  A step is
one whole call of the hot path (partition search + partitioned execution +
carry fix-up) on the headline workload: configuration 2 of the baseline workload list, the
power-law CSR SpMV (2M x 2M, ~50M nnz, fp64), inputs resident in HBM.

Extra objects on the line:
  roofline      dominant kernel's algorithmic bytes / its measured duration vs
                the 8 TB/s HBM peak (durations from HIP events recorded by the
                library around each kernel on the launch stream), and vs the
                streaming-read ceiling measured in the same run
  ceilings      this GPU's own streaming read, copy and independent-gather rates,
                measured in the same run with the library's probe kernels
  cpu_baseline  the serial CPU oracle timed on this machine's host cores
  balance       max/mean work per wavefront: from the partition table, and
                measured (items, items + rows, cycles per wavefront) with the
                instrumented build of the library
  workloads     the other configurations (one call each, same protocol), each
                with its own roofline object
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0


def _traffic_entry(kernel: str, workload: str):
    """HBM/fabric bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), recorded in
    profiles/traffic.json with the commit they were measured on; None when nothing is committed."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        t = json.load(f)
    return t.get(f"{kernel}@{workload}")


def _time_steps(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return e0.elapsed_time(e1) / steps, wall


def _kernel_ms(fn, reps):
    """Average duration of every kernel of one call (library-recorded HIP events)."""
    from paper_2604_17198_amd import binding as nb
    nb.profile_enable(True)
    acc = {}
    for _ in range(reps):
        fn()
        for name, ms in nb.profile_read():
            acc.setdefault(name, []).append(ms)
    nb.profile_enable(False)
    return {k: float(np.mean(v)) for k, v in acc.items()}


def _paper_protocol(fn):
    """Warm-up, 14 runs, drop the 2 fastest and 2 slowest, mean (paper, Section 5)."""
    import torch
    fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(14):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    ts = sorted(ts)[2:-2]
    return float(np.mean(ts))


def _measured_balance(fn, n_waves):
    """One call through the instrumented build of the library: what every wavefront of the
    executing kernel really worked on (its item and row counters) and how long it took."""
    import torch
    from paper_2604_17198_amd import binding as nb
    rb = np.dtype(nb.WAVE_RECORD).itemsize
    nb.select_library(True)
    try:
        fn()                                    # (first use of the instrumented code object)
        torch.cuda.synchronize()
        rec = torch.zeros(n_waves * rb, dtype=torch.uint8, device="cuda")
        nb.instrument(rec)
        fn()
        torch.cuda.synchronize()
        nb.instrument(None)
        r = rec.cpu().numpy().view(np.dtype(nb.WAVE_RECORD))
    finally:
        nb.select_library(False)
    r = r[r["t_begin"] > 0]
    items = r["items"].astype(np.float64)
    both = items + r["rows"].astype(np.float64)
    cyc = r["cycles"].astype(np.float64)
    busy = items > 0
    span_us = float((r["t_end"].max() - r["t_begin"].min()) / 100.0)
    return {"wavefronts": int(r.shape[0]), "items_total": int(items.sum()),
            "items_max_over_mean": float(items.max() / items.mean()),
            "items_plus_rows_max_over_mean": float(both.max() / both.mean()),
            "cycles_max_over_mean": float(cyc[busy].max() / cyc[busy].mean()),
            "cycles_mean": float(cyc[busy].mean()), "kernel_span_us": span_us}


def measure_ceilings():
    """Streaming read, copy and gather rates of this GPU (the library's probe kernels, HIP events)."""
    import torch
    from paper_2604_17198_amd import binding as nb
    n = 512 * 1024 * 1024                                   # bytes
    src = torch.ones(n // 8, dtype=torch.float64, device="cuda")
    dst = torch.empty_like(src)
    sink = torch.zeros(2, dtype=torch.int64, device="cuda")
    out = {}

    def timed(fn, reps=10):
        fn()
        ms, _ = _time_steps(fn, reps, 2)
        return ms

    ms = timed(lambda: nb.probe(nb.PROBE_READ, sink, src, n))
    out["stream_read_GBps"] = n / ms / 1e6
    ms = timed(lambda: nb.probe(nb.PROBE_COPY, dst, src, n))
    out["copy_GBps_read_plus_write"] = 2 * n / ms / 1e6
    g = 1 << 26
    for label, window in (("gather_1MiB_window_Gper_s", 1 << 20), ("gather_16MiB_window_Gper_s", 1 << 24),
                          ("gather_512MiB_window_Gper_s", n)):
        ms = timed(lambda: nb.probe(nb.PROBE_GATHER, sink, src, window, g), 5)
        out[label] = g / ms / 1e6
    out["bytes"] = n
    out["gathers"] = g
    return out


def _cpu_info():
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return model, os.cpu_count()


def bench_spmv(args, ceilings):
    import torch
    from paper_2604_17198_amd import binding as nb
    from paper_2604_17198_amd import workloads

    cfg = workloads.config(2)
    A = cfg["A"]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda")
    op = nb.csr(dev(A["pos"]), dev(A["crd"]), A["n_rows"], A["n_cols"], dev(A["val"]))
    x = dev(cfg["x"])
    y = torch.empty(A["n_rows"], dtype=torch.float64, device="cuda")
    ws = torch.empty(nb.workspace_bytes(nb.OP_SPMV, [op], nb.F64), dtype=torch.uint8, device="cuda")
    nnz = int(A["pos"][-1])
    n_rows, n_cols = A["n_rows"], A["n_cols"]

    step = lambda: nb.nacho_spmv(op, x, y, ws=ws)
    ms, wall_ms = _time_steps(step, args.steps, args.warmup)
    kms = _kernel_ms(step, 10)
    proto_ms = _paper_protocol(step)

    # algorithmic bytes: every input array once, the output once, the partition table
    P = nb.num_partitions(nb.OP_SPMV, [op], nb.F64)
    exec_bytes = nnz * 12 + (n_rows + 1) * 4 + n_cols * 8 + n_rows * 8 + (P + 1) * 16 + P * 12
    call_bytes = exec_bytes
    exec_ms = kms["spmv_exec"]
    achieved = exec_bytes / exec_ms / 1e6

    # balance from the partition table the fused call stored in its workspace
    torch.cuda.synchronize()
    parts = nb.workspace_parts(nb.OP_SPMV, [op], nb.F64, ws)
    work = np.diff(parts["cost"].cpu().numpy())
    rows_touched = np.diff(parts["coord"].cpu().numpy()[:, 0].astype(np.int64)) + 1
    both = work + rows_touched
    balance = {"partitions": int(P), "max_over_mean_nnz": float(work.max() / work.mean()),
               "max": int(work.max()), "mean": float(work.mean()),
               "table_nnz_plus_rows_max_over_mean": float(both.max() / both.mean()),
               "measured": _measured_balance(step, int(P))}

    # the row-aware cost variant on the same matrix (every row costs one unit on top of its non-zeros):
    # what balancing non-zeros + rows buys (or costs) against the paper's non-zero count
    P_rc = nb.rowcost_partitions(op, nb.F64, 1)
    ws_rc = torch.empty(nb.workspace_bytes(nb.OP_SPMV, [op], nb.F64, 0, P_rc), dtype=torch.uint8, device="cuda")
    step_rc = lambda: nb.nacho_spmv_rowcost(op, x, y, 1, ws=ws_rc)
    ms_rc, _ = _time_steps(step_rc, max(5, args.steps // 2), 2)
    rowcost = {"row_cost": 1, "partitions": int(P_rc), "ms_per_step": ms_rc, "kernel_ms": _kernel_ms(step_rc, 5),
               "measured": _measured_balance(step_rc, int(P_rc))}
    del ws_rc
    # the same call without a partition pass: every executing wavefront searches its own boundaries
    step_fu = lambda: nb.nacho_spmv_fused(op, x, y, ws=ws)
    ms_fu, _ = _time_steps(step_fu, max(5, args.steps // 2), 2)
    fused = {"ms_per_step": ms_fu, "kernel_ms": _kernel_ms(step_fu, 5)}

    # parity check of the timed configuration (full vector) and the oracle's own time
    import oracle
    best, ref, sabs = oracle.time_spmv_native(A["pos"], A["crd"], A["val"], cfg["x"], reps=3)
    step()
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    ok = bool(np.all(np.abs(got - ref) <= 1e-12 * np.maximum(np.abs(ref), sabs)))
    cpu_model, nproc = _cpu_info()

    tr = _traffic_entry("spmv_exec", "C2")
    return {
        "metric": "nnz/s (balanced CSR SpMV, partitioning included)",
        "value": nnz / (ms * 1e-3),
        "unit": "nnz/s",
        "ms_per_step": ms,
        "dtype": "f64",
        "config": {"workload": "C2: CSR SpMV y=Ax, fp64, 2,000,000 x 2,000,000, Zipf(1.3) rows, "
                               f"{nnz} nnz, 30% empty rows, seed 2", "nnz": nnz,
                   "partitions": int(P)},
        "call_GBps_algorithmic": call_bytes / ms / 1e6,
        "call_frac_of_peak": call_bytes / ms / 1e6 / PEAK_HBM_GBS,
        "host_wall_ms_per_step": wall_ms,
        "paper_protocol_ms": proto_ms,
        "kernel_ms": kms,
        "parity_ok": ok,
        "roofline": {"bound": "hbm", "kernel": "spmv_exec", "achieved": achieved, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                     "algorithmic_bytes_per_launch": exec_bytes,
                     "traffic": None if tr is None else tr.get("bytes_per_launch"),
                     "traffic_measured_on_commit": None if tr is None else tr.get("commit"),
                     "ceiling_GBps": ceilings["stream_read_GBps"],
                     "frac_of_ceiling": achieved / ceilings["stream_read_GBps"],
                     "gathers_per_launch": nnz,
                     "gather_rate_Gper_s": nnz / exec_ms / 1e6,
                     "gather_ceiling_16MiB_Gper_s": ceilings["gather_16MiB_window_Gper_s"]},
        "balance": balance,
        "row_aware_cost_variant": rowcost,
        "fused_search_variant": fused,
        "cpu_baseline": {"value": nnz / best, "unit": "nnz/s", "cores": 1, "kind": "oracle",
                         "seconds": best, "nproc": nproc, "cpu_model": cpu_model,
                         "build": "gcc -O3 -march=native (this host), timed in C with CLOCK_MONOTONIC",
                         "sample": "the whole C2 matrix, best of 3 runs of the serial long-double oracle"},
    }


def bench_others(steps, warmup, only=None, ceilings=None):
    """Configurations 3, 4 and 5 of the baseline workload list, one fused call per step, same timing
    protocol; algorithmic bytes = every input array once + every output array once."""
    import torch
    from paper_2604_17198_amd import binding as nb
    from paper_2604_17198_amd import workloads

    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda")
    res = {}

    def record(tag, what, fn, nnz, nbytes, table=None, main_kernel=None, waves=0, note=None):
        ms, _ = _time_steps(fn, steps, warmup)
        kms = _kernel_ms(fn, 5)
        res[tag] = {"workload": what, "ms_per_step": ms, "nnz_per_s": nnz / (ms * 1e-3),
                    "GBps_algorithmic": nbytes / ms / 1e6,
                    "frac_of_hbm_peak": nbytes / ms / 1e6 / PEAK_HBM_GBS,
                    "kernel_ms": kms}
        if main_kernel is not None:
            # the workload's own roofline object: its dominant kernel against the HBM peak and this GPU's ceiling
            k_ms = kms[main_kernel]
            tr = _traffic_entry(main_kernel, tag)
            ach = nbytes / k_ms / 1e6
            roof = {"bound": "hbm", "kernel": main_kernel, "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": ach / PEAK_HBM_GBS, "algorithmic_bytes_per_launch": int(nbytes),
                    "duration_ms": k_ms, "traffic": None if tr is None else tr.get("bytes_per_launch"),
                    "traffic_measured_on_commit": None if tr is None else tr.get("commit")}
            if ceilings is not None:
                roof["ceiling_GBps"] = ceilings["copy_GBps_read_plus_write"]
                roof["frac_of_ceiling"] = ach / ceilings["copy_GBps_read_plus_write"]
            if note:
                roof["note"] = note
            res[tag]["roofline"] = roof
        if table is not None:
            # work per partition from the table the fused call stored in its workspace
            torch.cuda.synchronize()
            work = np.diff(table()["cost"].cpu().numpy())
            res[tag]["balance"] = {"partitions": int(work.shape[0]), "max": int(work.max()),
                                   "mean": float(work.mean()), "max_over_mean": float(work.max() / work.mean())}
            if waves:
                res[tag]["balance"]["measured"] = _measured_balance(fn, waves)

    want = lambda tag: only is None or tag in only
    for c, fmt in ((3, "vector"), (4, "dcsr")):
        if not want(f"C{c}"):
            continue
        cfg = workloads.config(c)
        if fmt == "vector":
            ops = [nb.vector(dev(v["i"]), v["extent"], dev(v["v"])) for v in cfg["ops"]]
            rows = 0
        else:
            ops = [nb.dcsr(dev(m["pos0"]), dev(m["crd0"]), dev(m["pos1"]), dev(m["crd1"]),
                           m["n_rows"], m["n_cols"], dev(m["val"])) for m in cfg["ops"]]
            rows = sum(int(m["crd0"].shape[0]) for m in cfg["ops"])
        tot = sum(o.nnz for o in ops)
        out = nb.SparseOut(fmt, rows, tot, torch.float32, "cuda")
        ws = torch.empty(nb.workspace_bytes(nb.OP_SPADD, ops, nb.F32), dtype=torch.uint8, device="cuda")
        fn = lambda: nb.nacho_spadd_k(ops, out, ws=ws)
        fn()
        torch.cuda.synchronize()
        n_rows_out, n_out = (int(v) for v in out.counts.cpu().numpy()[:2])
        nbytes = tot * 8 + n_out * 8 + (rows * 8 + n_rows_out * 8 if fmt == "dcsr" else 0)
        what = ("C3: 3 sparse vectors (10M + 1M + 100k nnz, index space 2^30), fp32 union add" if c == 3 else
                "C4: DCSR + DCSR, 1,000,000 x 1,000,000, ~20M nnz each, fp32 union add")
        P_add = nb.num_partitions(nb.OP_SPADD, ops, nb.F32)
        record(f"C{c}", what + f", {tot} input nnz, {n_out} output nnz", fn, tot, nbytes,
               table=lambda: nb.workspace_parts(nb.OP_SPADD, ops, nb.F32, ws), main_kernel="spadd_merge",
               waves=P_add * nb.merge_wavefronts())
        if c == 3:
            # the same sum with the boundary search fused into the merge kernel (no partition kernel)
            ff = lambda: nb.nacho_spadd_fused(ops, out, ws=ws)
            ff()
            torch.cuda.synchronize()
            ms_f, _ = _time_steps(ff, steps, warmup)
            res["C3"]["fused_search_variant"] = {
                "what": "nacho_spadd_fused: every workgroup of the merge kernel searches its own two boundaries",
                "ms_per_step": ms_f, "kernel_ms": _kernel_ms(ff, 5),
                "same_output_count": int(out.counts.cpu().numpy()[1]) == n_out}
            fm = lambda: nb.nacho_spmul_k(ops, out, ws=ws)
            fm()
            torch.cuda.synchronize()
            n_mul = int(out.counts.cpu().numpy()[1])
            record("F2_vec3", f"3-way sparse-vector multiply (intersection) on the C3 vectors, {tot} input nnz, "
                   f"{n_mul} output nnz", fm, tot, tot * 8 + n_mul * 8)
        if c == 4:
            # F3: the same two matrices multiplied: an OUTER intersection, recursive partitioning
            outm = nb.SparseOut("dcsr", min(int(m["crd0"].shape[0]) for m in cfg["ops"]), min(o.nnz for o in ops),
                                torch.float32, "cuda")
            wsm = torch.empty(nb.workspace_bytes(nb.OP_SPMUL, ops, nb.F32), dtype=torch.uint8, device="cuda")
            fm = lambda: nb.nacho_spmul_k(ops, outm, ws=wsm)
            fm()
            torch.cuda.synchronize()
            r_mul, n_mul = (int(v) for v in outm.counts.cpu().numpy()[:2])
            tab = nb.workspace_parts(nb.OP_SPMUL, ops, nb.F32, wsm)
            work = int(tab["cost"][-1])                 # entries in the rows both operands store
            m_rows = int(tab["coord"][-1, 0])
            nbytes_m = work * 8 + rows * 4 + m_rows * 2 * 4 * len(ops) + n_mul * 8 + r_mul * 8
            # what the remapped cost function buys (the paper's comparison of recursive and plain hierarchical
            # partitioning, Section 5): the same number of partitions by the plain non-zero count, and
            # the entries each of them would really coiterate (those in rows both operands store)
            plain = nb.nacho_partition(ops, int(tab["P"]))
            torch.cuda.synchronize()
            pos_plain = plain["posn"].cpu().numpy()[:, :, 1]
            both = np.intersect1d(cfg["ops"][0]["crd0"], cfg["ops"][1]["crd0"])
            work_plain = np.zeros(int(tab["P"]), dtype=np.int64)
            for t, m in enumerate(cfg["ops"]):
                in_both = np.isin(m["crd0"], both)
                cum = np.concatenate([[0], np.cumsum(np.repeat(in_both, np.diff(m["pos1"])), dtype=np.int64)])
                work_plain += np.diff(cum[pos_plain[:, t]])
            plain_balance = {"max": int(work_plain.max()), "mean": float(work_plain.mean()),
                             "max_over_mean": float(work_plain.max() / max(work_plain.mean(), 1e-9))}
            record("F3_dcsr2", f"DCSR Hadamard product of the C4 matrices (recursive partitioning): {rows} stored "
                   f"rows, {m_rows} in both, {work} of {tot} input nnz coiterated, {n_mul} output nnz", fm, work,
                   nbytes_m, table=lambda: nb.workspace_parts(nb.OP_SPMUL, ops, nb.F32, wsm))
            res["F3_dcsr2"]["balance_with_plain_nonzero_cost"] = plain_balance
            del outm, wsm
            # F4: the same two matrices as coordinate lists (COO + COO, COO Hadamard)
            cops = []
            for m in cfg["ops"]:
                rws = np.repeat(m["crd0"], np.diff(m["pos1"])).astype(np.int32)
                cops.append(nb.coo(dev(rws), dev(m["crd1"]), m["n_rows"], m["n_cols"], dev(m["val"])))
            outc = nb.SparseOut("coo", 0, tot, torch.float32, "cuda")
            wsc = torch.empty(nb.workspace_bytes(nb.OP_SPADD, cops, nb.F32), dtype=torch.uint8, device="cuda")
            fa = lambda: nb.nacho_spadd_k(cops, outc, ws=wsc)
            fa()
            torch.cuda.synchronize()
            n_add = int(outc.counts.cpu().numpy()[1])
            record("F4_coo2_add", f"COO + COO on the C4 matrices, {tot} input nnz, {n_add} output nnz", fa, tot,
                   tot * 12 + n_add * 12, table=lambda: nb.workspace_parts(nb.OP_SPADD, cops, nb.F32, wsc))
            fh = lambda: nb.nacho_spmul_k(cops, outc, ws=wsc)
            fh()
            torch.cuda.synchronize()
            n_had = int(outc.counts.cpu().numpy()[1])
            record("F4_coo2_mul", f"COO Hadamard product of the C4 matrices, {tot} input nnz, {n_had} output nnz", fh,
                   tot, tot * 12 + n_had * 12)
            del cops, outc, wsc
        del ops, out, ws, cfg
    for kk in (2, 3, 8):
        if not want(f"F1_k{kk}"):
            continue
        cfg = workloads.csr_add_config(kk) if kk < 8 else workloads.csr_add_config(kk, nnz_each=2_000_000)
        ops = [nb.csr(dev(m["pos"]), dev(m["crd"]), m["n_rows"], m["n_cols"], dev(m["val"])) for m in cfg["ops"]]
        tot = sum(o.nnz for o in ops)
        out = nb.SparseOut("csr", 0, tot, torch.float32, "cuda", n_rows=cfg["n_rows"])
        ws = torch.empty(nb.workspace_bytes(nb.OP_SPADD, ops, nb.F32), dtype=torch.uint8, device="cuda")
        fn = lambda: nb.nacho_spadd_k(ops, out, ws=ws)
        fn()
        torch.cuda.synchronize()
        n_out = int(out.counts.cpu().numpy()[1])
        nbytes = tot * 8 + n_out * 8 + (kk + 1) * (cfg["n_rows"] + 1) * 4
        record(f"F1_k{kk}", f"fused {kk}-way CSR add, power-law 100,000 x 100,000 (shape of the paper's "
               f"skew experiment), fp32, {tot} input nnz, {n_out} output nnz", fn, tot, nbytes,
               main_kernel="spadd_merge")
        if kk == 2:
            fm = lambda: nb.nacho_spmul_k(ops, out, ws=ws)
            fm()
            torch.cuda.synchronize()
            n_mul = int(out.counts.cpu().numpy()[1])
            record("F2_csr2", f"CSR Hadamard product of the same two matrices, {tot} input nnz, {n_mul} output nnz",
                   fm, tot, tot * 8 + n_mul * 8 + 3 * (cfg["n_rows"] + 1) * 4)
        del ops, out, ws, cfg
    if want("F4_csf3"):
        cfg = workloads.csf3_add_config()
        names = ("pos0", "crd0", "pos1", "crd1", "pos2", "crd2")
        ops = [nb.csf3(*[dev(t[n]) for n in names], cfg["shape"], dev(t["val"])) for t in cfg["ops"]]
        tot = sum(int(t["crd2"].shape[0]) for t in cfg["ops"])
        fib = sum(int(t["crd1"].shape[0]) for t in cfg["ops"])
        sl = sum(int(t["crd0"].shape[0]) for t in cfg["ops"])
        out = nb.SparseOut("csf3", sl, tot, torch.float32, "cuda", cap_fibres=fib)
        ws = torch.empty(nb.workspace_bytes(nb.OP_SPADD, ops, nb.F32), dtype=torch.uint8, device="cuda")
        fn = lambda: nb.nacho_spadd_k(ops, out, ws=ws)
        fn()
        torch.cuda.synchronize()
        s_out, f_out, n_out = (int(v) for v in out.counts.cpu().numpy())
        nbytes = (tot + n_out) * 8 + (fib + f_out) * 8 + (sl + s_out) * 8
        record("F4_csf3", f"CSF + CSF, third-order tensors {cfg['shape']}, fp32 union add, {tot} input nnz in {fib} "
               f"fibres, {n_out} output nnz in {f_out} fibres and {s_out} slices", fn, tot, nbytes,
               table=lambda: nb.workspace_parts(nb.OP_SPADD, ops, nb.F32, ws), main_kernel="spadd_merge")
        del ops, out, ws, cfg
    if not want("C5"):
        return res
    cfg = workloads.config(5)
    A = cfg["A"]
    op = nb.csr(dev(A["pos"]), dev(A["crd"]), A["n_rows"], A["n_cols"], dev(A["val"]))
    B = dev(cfg["B"])
    C = torch.empty((A["n_rows"], 64), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.workspace_bytes(nb.OP_SPMM, [op], nb.F32, 64), dtype=torch.uint8, device="cuda")
    nnz = int(A["pos"][-1])
    nbytes = nnz * 8 + (A["n_rows"] + 1) * 4 + A["n_cols"] * 64 * 4 + A["n_rows"] * 64 * 4
    P5 = nb.num_partitions(nb.OP_SPMM, [op], nb.F32, 64)
    record("C5", f"C5: CSR (1,000,000 x 1,000,000, {nnz} nnz) x dense 1,000,000 x 64, fp32 SpMM",
           lambda: nb.nacho_spmm(op, B, C, ws=ws), nnz, nbytes,
           table=lambda: nb.workspace_parts(nb.OP_SPMM, [op], nb.F32, ws, 64), main_kernel="spmm_exec", waves=P5,
           note="compulsory bytes (B and C once); the i -> j -> k order re-reads a 256-byte row of B per stored "
                f"non-zero: {nnz * 256 / 1e9:.2f} GB through the fabric, which is what bounds this kernel")
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--headline-only", action="store_true",
                    help="time configuration 2 only (skip the other configurations)")
    ap.add_argument("--only", default=None,
                    help="comma-separated workload tags (C3, C4, C5, F1_k2, F1_k3, F4_csf3, F1_k8): time only these, "
                         "print their records and skip the headline (for profiler runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run two device-to-device copies of 256 MiB (a kernel of known "
                         "traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path is not sharded in this run); "
                 "use --gpus 1")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.only:
        print(json.dumps({"workloads": bench_others(args.steps, args.warmup, set(args.only.split(",")))}))
        return
    ceilings = measure_ceilings()
    out = bench_spmv(args, ceilings)
    out["ceilings"] = ceilings
    if not args.headline_only:
        out["workloads"] = bench_others(max(5, args.steps // 5), 2, ceilings=ceilings)
    if args.calibrate_copy:
        a = torch.zeros(32 * 1024 * 1024, dtype=torch.float64, device="cuda")
        b = torch.empty_like(a)
        for _ in range(2):
            b.copy_(a)
        torch.cuda.synchronize()
    line = {
        "metric": out.pop("metric"), "value": out.pop("value"), "unit": out.pop("unit"),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": out.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": out.pop("dtype"), "data": "synthetic", "config": out.pop("config"),
    }
    line.update(out)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
