#!/usr/bin/env python3
"""Benchmark of the TRIM filter-then-refine scan on one MI355X.

A step = one pass of the whole hot path over the full query batch of the workload:
coarse-probe selection, query ordering, distance tables (built inside the scan kernel), lower-
bound scan with pruning, exact refinement of survivors and top-k selection (range workloads:
radius filter and CSR output).  Inputs (index, queries) are resident in HBM before the timed
region; results stay on the device.

Every number in the printed line is produced in this run: kernel times by HIP events on the
launch stream, what the kernel touched by its own work counters (one untimed launch), the two
machine ceilings it is priced against (streaming read, table lookups out of LDS) by the
library's measurement aids, recall / average precision against ground truth from the CPU oracle,
and the oracle's own speed on the host cores.  Prints ONE JSON line.
"""
import argparse
import ctypes
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# LDS peak derived from the chip's unit counts: 256 CUs x 128 bytes per clock x 2.4 GHz; a table
# lookup moves 4 bytes.
LDS_PEAK_GLOOKUPS = 256 * 128 * 2.4 / 4


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C2", help="C1..C5, T384, W768 (default C2, the headline config)")
    ap.add_argument("--gamma", type=float, default=None,
                    help="relaxation to time (default: largest swept gamma with recall@k >= 0.95)")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--truth-queries", type=int, default=0,
                    help="queries behind recall / average precision (0: sized so that the oracle's "
                         "exact search over all n takes about ten seconds)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0,
                    help="CPU time budget for timing the oracle on all threads (0 = skip); the "
                         "single-thread figure gets half of it on top")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-order", action="store_true", help="do not sort queries by first probed list")
    ap.add_argument("--no-list-bounds", action="store_true",
                    help="time the search without the per-list summaries only (no list-level pruning)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the machine-ceiling measurements")
    ap.add_argument("--calibrate", action="store_true",
                    help="run only a plain elementwise pass that reads 1 GiB and writes 1 GiB, three "
                         "times (the known-size kernel that rocprofv3's FETCH_SIZE / WRITE_SIZE are "
                         "scaled by), and exit")
    ap.add_argument("--no-traffic", action="store_true",
                    help="do not measure HBM traffic (four short child runs of this script under "
                         "rocprofv3 --pmc before the GPU is touched here)")
    ap.add_argument("--traffic-child", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--no-compare", action="store_true",
                    help="skip the second timed leg (the same steps without list-level pruning)")
    ap.add_argument("--ceilings-only", action="store_true",
                    help="measure the two machine ceilings (streaming read, LDS table lookups) and exit")
    ap.add_argument("--tables-only", action="store_true",
                    help="time trim_build_lut on the workload's queries (vector-ALU form and matrix-core "
                         "form, 20 launches each) and exit")
    ap.add_argument("--code-bits", type=int, default=8, choices=(8, 4),
                    help="4: index the workload with the 4-bit codes of the FastScan variant "
                         "(d/2 subspaces of 16 centroids) instead of its M subspaces of 256")
    return ap.parse_args()


def _event_ms(fn, reps):
    import torch
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def machine_ceilings(trim):
    """Streaming-read rate of HBM and table-lookup rate of LDS, by the library's aids, now."""
    import torch
    size = 2 << 30
    buf = torch.empty(size // 4, dtype=torch.int32, device="cuda").random_()
    sink = torch.empty(8192, dtype=torch.int32, device="cuda")
    read = max(size / (_event_ms(lambda: trim.trim_ceiling_stream_read(buf, blocks, sink), 5) * 1e-3) / 1e9
               for blocks in (1024, 2048, 4096))
    del buf
    iters = 1024
    fsink = torch.empty(1024 * 512, dtype=torch.float32, device="cuda")
    look = max(blocks * 512 * iters * 32 / (_event_ms(
        lambda: trim.trim_ceiling_lds_gather(blocks, iters, 12345, fsink), 5) * 1e-3) / 1e9
        for blocks in (768, 1024))
    look16 = max(blocks * 512 * iters * 64 / (_event_ms(
        lambda: trim.trim_ceiling_lds_gather(blocks, iters, 12345, fsink, entry_floats=16), 5) * 1e-3) / 1e9
        for blocks in (768, 1024))
    return dict(stream_read_GBps=round(read, 1), lds_random_lookup_Glookups=round(look, 1),
                lds_rows_of_16_lookup_Glookups=round(look16, 1))


def _counter_rows(csv_path, needle):
    """(dispatch id, value) of every dispatch of a kernel whose name contains `needle`, in order."""
    import csv
    rows = {}
    with open(csv_path, newline="") as f:
        for r in csv.DictReader(f):
            if needle in r["Kernel_Name"]:
                rows[int(r["Dispatch_Id"])] = rows.get(int(r["Dispatch_Id"]), 0.0) + float(r["Counter_Value"])
    return [rows[k] for k in sorted(rows)]


def _counter_table(csv_path, needle):
    """{counter: [value per dispatch, in dispatch order]} for the kernels whose name contains `needle`."""
    import csv
    tab = {}
    with open(csv_path, newline="") as f:
        for r in csv.DictReader(f):
            if needle in r["Kernel_Name"]:
                d = tab.setdefault(r["Counter_Name"], {})
                d[int(r["Dispatch_Id"])] = d.get(int(r["Dispatch_Id"]), 0.0) + float(r["Counter_Value"])
    return {c: [d[k] for k in sorted(d)] for c, d in tab.items()}


UNIT_COUNTERS = ("SQ_INSTS_VALU", "SQ_INSTS_LDS", "SQ_ACTIVE_INST_VALU", "SQ_LDS_IDX_ACTIVE", "GRBM_GUI_ACTIVE")


def units_busy(table):
    """How busy the vector ALUs and the LDS were during the search kernel's last three launches,
    from one rocprofv3 --pmc run (UNIT_COUNTERS): a wave instruction occupies its SIMD's vector
    ALU for 4 clocks (64 lanes on 16); SQ_LDS_IDX_ACTIVE counts a CU's LDS-busy clocks;
    GRBM_GUI_ACTIVE is summed over the 8 XCDs.  256 CUs, 1024 SIMDs."""
    try:
        m = {c: sum(table[c][-3:]) / 3 for c in UNIT_COUNTERS}
    except (KeyError, IndexError):
        return None
    cycles = m["GRBM_GUI_ACTIVE"] / 8.0
    if cycles <= 0:
        return None
    return dict(valu=round(m["SQ_ACTIVE_INST_VALU"] * 4.0 / (1024.0 * cycles), 4),
                lds=round(m["SQ_LDS_IDX_ACTIVE"] / (256.0 * cycles), 4),
                valu_wave_instructions=int(m["SQ_INSTS_VALU"]), lds_wave_instructions=int(m["SQ_INSTS_LDS"]),
                gpu_cycles=int(cycles),
                method="rocprofv3 --pmc " + " ".join(UNIT_COUNTERS) + ", one more child run of this script (last 3 "
                       "launches of the search kernel): valu = SQ_ACTIVE_INST_VALU x 4 / (1024 SIMDs x cycles), "
                       "lds = SQ_LDS_IDX_ACTIVE / (256 CUs x cycles), cycles = GRBM_GUI_ACTIVE / 8 XCDs")


def measure_traffic(args):
    """HBM traffic of the dominant kernel in the timed configuration: FETCH_SIZE and WRITE_SIZE (KiB
    per dispatch) of its last three launches in a child run of this script under rocprofv3 --pmc,
    one counter per run, each scaled by what the same counter reads for a plain elementwise pass
    that reads 1 GiB and writes 1 GiB (two more child runs).  Must be called before this process
    touches the GPU.  Returns None if rocprofv3 is not there or a run fails."""
    import glob
    import shutil
    import subprocess
    import tempfile
    prof = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(prof) or any(k.startswith("ROCPROF") for k in os.environ):
        return None
    me = os.path.abspath(__file__)
    child = ["--workload", args.workload, "--code-bits", str(args.code_bits), "--truth-queries",
             str(args.truth_queries), "--traffic-child"]
    for flag, on in (("--no-order", args.no_order), ("--no-list-bounds", args.no_list_bounds),
                     ("--no-sweep", args.no_sweep)):
        if on:
            child.append(flag)
    if args.gamma is not None:
        child += ["--gamma", str(args.gamma)]
    if args.batch:
        child += ["--batch", str(args.batch)]
    env = dict(os.environ, TMPDIR="/tmp")
    got = {}
    try:
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            for what, argv, needle in (("kernel", child, "search_kernel"), ("copy", ["--calibrate"], "elementwise")):
                out = tempfile.mkdtemp(prefix="trim_pmc_", dir="/tmp")
                cmd = ["timeout", "-s", "KILL", "600", prof, "--pmc", counter, "-d", out, "-o", "p",
                       "--output-format", "csv", "--", "python3", me] + argv
                r = subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
                files = glob.glob(os.path.join(out, "**", "p_counter_collection.csv"), recursive=True)
                if r.returncode != 0 or not files:
                    shutil.rmtree(out, ignore_errors=True)
                    return None
                vals = _counter_rows(files[0], needle)
                shutil.rmtree(out, ignore_errors=True)
                if len(vals) < 3:
                    return None
                # the kernel: its last three launches are the timed configuration; the copy: its
                # three largest dispatches are the three passes (the fill before them reads nothing)
                got[(counter, what)] = (sum(vals[-3:]) / 3 if what == "kernel" else sum(sorted(vals)[-3:]) / 3)
    except (OSError, KeyError, ValueError):
        return None
    units = None
    try:        # how busy the units were: a run of its own, and no reason to lose the traffic if it fails
        out = tempfile.mkdtemp(prefix="trim_pmc_", dir="/tmp")
        cmd = ["timeout", "-s", "KILL", "600", prof, "--pmc", *UNIT_COUNTERS, "-d", out, "-o", "p",
               "--output-format", "csv", "--", "python3", me] + child
        r = subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
        files = glob.glob(os.path.join(out, "**", "p_counter_collection.csv"), recursive=True)
        if r.returncode == 0 and files:
            units = units_busy(_counter_table(files[0], "search_kernel"))
        shutil.rmtree(out, ignore_errors=True)
    except (OSError, KeyError, ValueError):
        units = None
    gib_kib = float(1 << 20)
    sf = gib_kib / got[("FETCH_SIZE", "copy")] if got[("FETCH_SIZE", "copy")] > 0 else 0.0
    sw = gib_kib / got[("WRITE_SIZE", "copy")] if got[("WRITE_SIZE", "copy")] > 0 else 0.0
    fetch_b = got[("FETCH_SIZE", "kernel")] * 1024 * sf
    write_b = got[("WRITE_SIZE", "kernel")] * 1024 * sw
    return dict(bytes_per_launch=int(fetch_b + write_b), fetch_bytes=int(fetch_b), write_bytes=int(write_b),
                FETCH_SIZE_KiB=round(got[("FETCH_SIZE", "kernel")], 1), WRITE_SIZE_KiB=round(got[("WRITE_SIZE", "kernel")], 1),
                scale_fetch=round(sf, 4), scale_write=round(sw, 4), units_busy=units,
                method="rocprofv3 --pmc, one counter per child run of this script (last 3 launches of the "
                       "search kernel), scaled by the same counter on a 1 GiB read + 1 GiB write pass")


def host_index(orc, ix, centroids):
    """The device index as the oracle's plain arrays (orc: trim_oracle, or trim_oracle_fs for 4-bit codes)."""
    h = lambda t: None if t is None else t.cpu().numpy()
    return orc.Index(h(ix.base), h(ix.codes), h(ix.dlx), h(ix.codebooks), ids=h(ix.ids),
                     list_offsets=h(ix.list_offsets), centroids=h(centroids))


def set_threads(n):
    """Threads of the oracle's OpenMP loops (the runtime's own call; the oracle is not touched)."""
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def time_oracle(fn_chunk, nq, budget_s, chunk):
    """Run fn_chunk(lo, hi) -> bool (same as the GPU's?) over the query set in order, wrapping
    around, until the time budget is used.  Returns (queries done, seconds, all equal)."""
    done, used, same = 0, 0.0, True
    while used < budget_s:
        lo = done % nq
        hi = min(nq, lo + chunk)
        t1 = time.perf_counter()
        ok = fn_chunk(lo, hi)
        used += time.perf_counter() - t1
        same = same and ok
        done += hi - lo
    return done, used, same


def truth_count(args, w):
    if args.truth_queries > 0:
        return min(args.truth_queries, w.nq)
    # the oracle's exact search costs about n*d multiply-adds per query in float64
    return int(max(50, min(1000, w.nq, 1.0e11 / (w.n * w.d))))


def work_totals(trim, work):
    tot = work.to(dtype=__import__("torch").int64).sum(0).tolist()
    return {name: int(tot[i]) for i, name in enumerate(trim.WORK_NAMES)}


def touched_bytes(w, nq, k_or_results, wt, use_lut, ncent=256):
    """Bytes the launch requested from memory, by the kernel's own counters: codes / scan heads /
    landmark distances / list summaries, raw rows (+ id) of every exact distance, the query, the
    PQ centroids (or the prebuilt table) behind each query's distance table, the results."""
    table_src = nq * (w.M * 1024 if use_lut else w.d * ncent * 4)
    return dict(codes=wt["code_bytes"], rows=wt["rows"] * (4 * w.d + 4), queries=nq * 4 * w.d,
                table_source=table_src, results=k_or_results * 8,
                total=wt["code_bytes"] + wt["rows"] * (4 * w.d + 4) + nq * 4 * w.d + table_src + k_or_results * 8)


def roofline_object(w, nq, scan_ms, alg_bytes, wt, touched, ceil, kernel, fs=False, traffic=None):
    """The dominant kernel against the resource that binds it.  Long codes streamed once per
    query are bound by HBM; short codes shared by many queries through the caches are bound by
    the rate of table lookups out of LDS."""
    sec = scan_ms * 1e-3
    alg = alg_bytes / sec / 1e9
    tch = touched["total"] / sec / 1e9
    looks = wt["lookups"] / sec / 1e9
    hbm = dict(algorithmic_bytes=alg_bytes, algorithmic_GBps=round(alg, 1),
               algorithmic_frac_of_peak=round(alg / HBM_PEAK_GBS, 4),
               touched_bytes=touched, touched_GBps=round(tch, 1),
               touched_frac_of_peak=round(tch / HBM_PEAK_GBS, 4), peak_GBps=HBM_PEAK_GBS,
               stream_read_ceiling_GBps=ceil.get("stream_read_GBps"),
               note="algorithmic = (M+4) B per scanned candidate + (4d+4) B per exact distance + query "
                    "and results, no reuse assumed; touched = what the kernel requested (its work "
                    "counters), part of it served by the caches; bytes beyond L2 are in profiles/")
    lds = dict(lookups=wt["lookups"], Glookups_per_s=round(looks, 1), peak_Glookups=LDS_PEAK_GLOOKUPS,
               frac_of_peak=round(looks / LDS_PEAK_GLOOKUPS, 4),
               lookup_ceiling_Glookups=ceil.get("lds_rows_of_16_lookup_Glookups" if fs else
                                                "lds_random_lookup_Glookups"),
               frac_of_lookup_ceiling=None,
               note="peak = 256 CUs x 128 B/clk x 2.4 GHz / 4 B; the ceiling is the scan's own lookup-and-"
                    "add sequence on random codes with nothing else going on (8-bit codes: 256-entry "
                    "rows, bank conflicts; 4-bit codes: rows of 16, no conflicts), measured in this run")
    if lds["lookup_ceiling_Glookups"]:
        lds["frac_of_lookup_ceiling"] = round(looks / lds["lookup_ceiling_Glookups"], 4)
    # The task's accounting is algorithmic bytes against the HBM peak.  Where that rate exceeds
    # the peak, the bytes cannot have come from HBM (queries share the codes through the caches,
    # lists are passed over): HBM bounds nothing there, and the kernel is priced against the
    # table-lookup rate of LDS instead, with the byte rates listed beside it.
    lookup_ceiling = ceil.get("lds_rows_of_16_lookup_Glookups" if fs else "lds_random_lookup_Glookups")
    f_lds = looks / (lookup_ceiling or LDS_PEAK_GLOOKUPS)
    trf = traffic["bytes_per_launch"] / sec / 1e9 if traffic else None
    hbm["measured_traffic_GBps"] = round(trf, 1) if trf else None
    hbm["measured_traffic_frac_of_peak"] = round(trf / HBM_PEAK_GBS, 4) if trf else None
    if alg <= HBM_PEAK_GBS:
        head = dict(bound="hbm", achieved=round(alg, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(alg / HBM_PEAK_GBS, 4), achieved_is="algorithmic bytes / kernel time")
    elif trf and trf / HBM_PEAK_GBS >= f_lds:
        # the model's bytes exceed the peak (the first pass reads 12 bytes instead of M + 4, lists
        # are passed over, queries share codes), yet what does reach HBM is the larger share
        head = dict(bound="hbm", achieved=round(trf, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(trf / HBM_PEAK_GBS, 4),
                    achieved_is="HBM traffic measured in this run (rocprofv3 counters) / kernel time; the "
                                "algorithmic bytes would exceed the peak")
    else:
        head = dict(bound="lds", achieved=round(looks, 1), peak=LDS_PEAK_GLOOKUPS, unit="Glookup/s",
                    frac=round(looks / LDS_PEAK_GLOOKUPS, 4))
    head.update(traffic=traffic["bytes_per_launch"] if traffic else None, traffic_detail=traffic,
                units_busy=traffic.get("units_busy") if traffic else None,
                kernel=kernel, kernel_ms=round(scan_ms, 4), hbm=hbm, lds=lds, work=wt,
                candidates_per_s=dict(
                    counted=round((wt["first_pass"] + wt["skipped"]) / sec, 1),
                    read=round(wt["first_pass"] / sec, 1),
                    note="counted = every candidate of Section 4.2's scan; read = those whose code was "
                         "looked at (the rest were passed over with their whole list)"))
    return head


def timed_steps(args, step_fn):
    """W warm-up steps, then K timed steps bracketed by synchronisation; per-step events at the
    step's start, before the search launch and at its end."""
    import torch
    for _ in range(args.warmup):
        step_fn(None)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        step_fn(ev[s])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    steps = [e[0].elapsed_time(e[2]) for e in ev]
    scans = [e[1].elapsed_time(e[2]) for e in ev]
    return dict(ms_per_step=max(wall_ms, sum(steps) / len(steps)), step_median=statistics.median(steps),
                scan_mean=sum(scans) / len(scans), scan_median=statistics.median(scans))


def bench_range(args, w, bw, probes_for, setup_s, ceil, traffic=None):
    """Range-search workloads (Section 2.1, range search): a step = probe selection + tables +
    the fused scan / refine / radius filter + offsets + the CSR fill, for the whole query set."""
    import numpy as np
    import torch
    from oracle import trim_oracle
    from paper_2508_17828_amd import synth, trim
    ix, queries, nq = bw.index, bw.queries, w.nq
    oix = host_index(trim_oracle, ix, bw.centroids)
    qh = queries.cpu().numpy()
    # one global radius: the stated percentile of seeded (query, base) pair distances
    qi, bi = synth.pair_sample(w, 256, 10_000)
    qs = qh[qi].astype(np.float64)
    xs = oix.base[np.sort(bi)].astype(np.float64)
    d2 = (qs * qs).sum(1)[:, None] - 2 * qs @ xs.T + (xs * xs).sum(1)[None, :]
    radius = float(np.sqrt(max(np.percentile(d2, w.range_percentile), 0.0)))
    # ground truth on a query subset: Section 2.1's definition over ALL n by the oracle's exact distance
    nt = truth_count(args, w)
    r2 = np.float32(radius) * np.float32(radius)
    pos_all = np.arange(w.n, dtype=np.int64)
    id_of = oix.ids if oix.ids is not None else np.arange(w.n, dtype=np.int32)
    truth = [id_of[trim_oracle.exact_pairs(oix.base, qh, np.full(w.n, q, np.int64), pos_all) <= r2]
             for q in range(nt)]
    rows = []
    gammas = [args.gamma] if args.gamma is not None else sorted(set(w.gammas))
    def order_for(pr):
        return trim.trim_query_order(pr, w.nlist) if pr is not None and not args.no_order else None

    for g in gammas:
        pr = probes_for(queries)
        r = trim.trim_search_range(ix, queries, radius, g, probes=pr, query_order=order_for(pr))
        go, gi = r["offsets"].cpu().numpy(), r["ids"].cpu().numpy()
        # average precision of Section 2.1: |R'| / |R| over the queries with R nonempty (R' is a subset of R)
        vals = [len(np.intersect1d(truth[q], gi[go[q]:go[q + 1]])) / len(truth[q])
                for q in range(nt) if len(truth[q])]
        scanned, exact = int(r["n_scanned"].sum().item()), int(r["n_exact"].sum().item())
        rows.append(dict(gamma=g, average_precision=round(float(np.mean(vals)), 4) if vals else None,
                         results=r["required"], pruning_ratio=round(1 - exact / max(1, scanned), 5),
                         n_scanned=scanned, n_exact=exact))
    ok = [x for x in rows if x["average_precision"] is not None and x["average_precision"] >= 0.95]
    chosen = max(ok, key=lambda x: x["gamma"]) if ok else rows[0]
    gamma = chosen["gamma"]
    cap = max(1, chosen["results"])
    _, mc = ix._cand(probes_for(queries))
    ws = torch.empty((trim.trim_range_workspace_bytes(nq, mc),), dtype=torch.uint8, device="cuda")
    # A table that does not fit the LDS in one piece (M > 128) is refilled for every span of
    # candidates: then the tables are built once per step by trim_build_lut and copied from there.
    use_lut = w.M * 1024 > 128 * 1024
    lut_buf = torch.empty((nq, w.M, 256), dtype=torch.float32, device="cuda") if use_lut else None
    last = {}

    def step(ev):
        if ev: ev[0].record()
        pr = probes_for(queries)
        order = order_for(pr)
        lut = trim.trim_build_lut(queries, ix.codebooks, out=lut_buf) if use_lut else None
        if ev: ev[1].record()
        last["r"] = trim.trim_search_range(ix, queries, radius, gamma, probes=pr, capacity=cap,
                                           want_stats=False, workspace=ws, lut=lut, query_order=order)
        if ev: ev[2].record()

    if args.traffic_child:      # (run under rocprofv3 by measure_traffic: the timed launch, a few times)
        for _ in range(4):
            step(None)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_child": True, "gamma": gamma}))
        return None
    t = timed_steps(args, step)
    got = last["r"]
    # what the launch touched (one untimed launch with the work counters)
    lut = trim.trim_build_lut(queries, ix.codebooks, out=lut_buf) if use_lut else None
    pr = probes_for(queries)
    acc = trim.trim_search_range(ix, queries, radius, gamma, probes=pr, capacity=cap, workspace=ws, lut=lut,
                                 want_work=True, query_order=order_for(pr))
    wt = work_totals(trim, acc["work"])
    touched = touched_bytes(w, nq, chosen["results"], wt, use_lut)
    alg_bytes = (chosen["n_scanned"] * (w.M + 4) + chosen["n_exact"] * (4 * w.d + 4) + nq * 4 * w.d +
                 chosen["results"] * 8 + (nq + 1) * 8)
    roof = roofline_object(w, nq, t["scan_mean"], alg_bytes, wt, touched, ceil,
                           "search_kernel<range> + range_offsets_kernel + range_fill_kernel", traffic=traffic)

    # ---- CPU baseline: the oracle on a bounded sample, results compared with the GPU's ----
    cpu = None
    if args.cpu_seconds > 0:
        go, gi = got["offsets"].cpu().numpy(), got["ids"].cpu().numpy()
        ch = oix.centroids

        def chunk(lo, hi):
            qs_ = np.ascontiguousarray(qh[lo:hi])
            ph = trim_oracle.ivf_probe(qs_, ch, w.nprobe) if w.nlist else None
            ro = trim_oracle.search_range(oix, qs_, radius, gamma, ph)
            return bool(np.array_equal(ro["ids"], gi[go[lo]:go[hi]]) and
                        np.array_equal(ro["offsets"], go[lo:hi + 1] - go[lo]))

        nthr = trim_oracle.num_threads()
        done, used, same = time_oracle(chunk, nq, args.cpu_seconds, min(nq, 4 * nthr))
        set_threads(1)
        done1, used1, same1 = time_oracle(chunk, nq, args.cpu_seconds / 2, 2)
        set_threads(nthr)
        cpu = dict(value=round(done / used, 2), unit="queries/s", cores=nthr, kind="oracle",
                   sample=f"{done} queries (the query set in order) in {used:.1f} s: probe selection + range "
                          f"scan, same index, radius and gamma; result ids equal to the GPU's: {same}",
                   single_thread=dict(value=round(done1 / used1, 2), unit="queries/s", cores=1,
                                      sample=f"{done1} queries in {used1:.1f} s; ids equal: {same1}"))
    return {
        "metric": "queries/sec at average precision>=0.95 (1 MI355X); pruning ratio; scan HBM GB/s",
        "value": round(nq / (t["ms_per_step"] * 1e-3), 1), "unit": "queries/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(t["ms_per_step"], 4),
        "ms_per_step_median": round(t["step_median"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n} base x {nq} queries, d={w.d}, PQ M={w.M}x256, "
                               f"IVF nlist={w.nlist} nprobe={w.nprobe}, range search, radius at the "
                               f"{w.range_percentile} th percentile of sampled pair distances",
                   "gamma": gamma, "radius": round(radius, 6), "average_precision": chosen["average_precision"],
                   "truth": f"all vectors within the radius by the CPU oracle's exact distance over all n, "
                            f"first {nt} queries",
                   "pruning_ratio": chosen["pruning_ratio"], "results": chosen["results"],
                   "timed": "probe selection + query ordering + tables + fused scan/refine/filter + offsets + CSR fill "
                            "(one host read of the result count per step), inputs in HBM",
                   "setup_s": round(setup_s, 1)},
        "roofline": roof, "cpu_baseline": cpu, "ceilings": ceil, "sweep": rows,
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
              "(the path has no collective: queries would simply be dealt out to the GPUs)", file=sys.stderr)
        sys.exit(2)
    # HBM traffic first: its child processes must run before this one touches the GPU
    traffic = None
    if not (args.no_traffic or args.traffic_child or args.calibrate or args.ceilings_only or args.tables_only):
        traffic = measure_traffic(args)
    import numpy as np
    import torch
    from paper_2508_17828_amd import index_setup, synth, trim

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    trim.lib()
    torch.cuda.set_device(0)
    if args.calibrate:
        x = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        y = torch.empty_like(x)
        for _ in range(3):
            torch.add(x, 1.0, out=y)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate": "3 elementwise passes, each reading 1 GiB and writing 1 GiB"}))
        return
    if args.ceilings_only:
        print(json.dumps(machine_ceilings(trim)))
        return
    w = synth.WORKLOADS[args.workload]
    if args.tables_only:
        # random codebooks of the workload's shape do: the table kernels' work does not depend on values
        q = torch.from_numpy(synth.query_vectors(w)).cuda()
        cb = torch.randn((w.M, 256, w.d // w.M), dtype=torch.float32, device="cuda")
        out = torch.empty((w.nq, w.M, 256), dtype=torch.float32, device="cuda")
        res = {"workload": w.name, "table_bytes": out.numel() * 4}
        for name, mfma in (("vector_alu_ms", False), ("matrix_cores_ms", True)):
            res[name] = round(_event_ms(lambda: trim.trim_build_lut(q, cb, mfma=mfma, out=out), 20), 4)
        print(json.dumps(res))
        return
    batch = args.batch or w.batch
    t0 = time.time()
    bw = index_setup.build_workload(w, code_bits=args.code_bits)
    ix, queries = bw.index, bw.queries
    fs = args.code_bits == 4
    code_bytes = ix.codes.shape[1]
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    nq, k = w.nq, w.k
    ceil = {} if args.no_ceilings or args.traffic_child else machine_ceilings(trim)

    def probes_for(q):
        return trim.trim_ivf_probe(q, bw.centroids, w.nprobe) if w.nlist else None

    if w.mode == "range":
        if fs:
            print("bench.py: --code-bits 4 is timed on the kNN workloads", file=sys.stderr)
            sys.exit(2)
        line = bench_range(args, w, bw, probes_for, setup_s, ceil, traffic)
        if line is not None:
            print(json.dumps(line))
        return

    from oracle import trim_oracle, trim_oracle_fs
    orc = trim_oracle_fs if fs else trim_oracle      # the scan's oracle for this code width
    oix = host_index(orc, ix, bw.centroids)
    qh = queries.cpu().numpy()

    # ---- ground truth on a query subset: exact kNN over ALL n in float64 by the CPU oracle ----
    nt = truth_count(args, w)
    t1 = time.time()
    truth_ids, _ = trim_oracle.brute_knn_f64(oix.base, np.ascontiguousarray(qh[:nt]), k, ids=oix.ids)
    truth = torch.from_numpy(truth_ids).cuda()
    truth_s = time.time() - t1

    import dataclasses
    ix_plain = dataclasses.replace(ix, list_bounds=None)     # the same index without list summaries

    def order_for(pr):
        return trim.trim_query_order(pr, w.nlist) if pr is not None and not args.no_order else None

    def run_once(index, gamma, **kw):
        pr = probes_for(queries)
        return trim.trim_search_knn(index, queries, k, gamma, batch, probes=pr, query_order=order_for(pr), **kw)

    # ---- sweep of the relaxation parameter (quality numbers; short timing) ----
    sweep = []
    gammas = sorted(set(list(w.gammas) + ([] if args.no_sweep else [0.2, 0.3, 0.4, 0.45, 0.6, 0.7])))
    if args.gamma is not None:
        gammas = [args.gamma]
    main_ix = ix_plain if args.no_list_bounds else ix
    for g in gammas:
        r = run_once(main_ix, g)
        ms = (_event_ms(lambda: run_once(main_ix, g, want_stats=False), 3)
              if args.gamma is None and not args.traffic_child else None)
        scanned, exact = int(r["n_scanned"].sum().item()), int(r["n_exact"].sum().item())
        sweep.append(dict(gamma=g, recall=round(index_setup.recall_at_k(r["ids"][:nt], truth), 4),
                          pruning_ratio=round(1.0 - exact / max(1, scanned), 5),
                          qps=round(nq / (ms * 1e-3), 1) if ms else None, n_scanned=scanned, n_exact=exact))
    ok = [s for s in sweep if s["recall"] >= 0.95]
    chosen = max(ok, key=lambda s: s["gamma"]) if ok else min(sweep, key=lambda s: s["gamma"])
    gamma = chosen["gamma"]

    # ---- timed region: K steps, events around each step and around the scan kernel ----
    out = (torch.empty((nq, k), dtype=torch.int32, device="cuda"),
           torch.empty((nq, k), dtype=torch.float32, device="cuda"))

    def make_step(index):
        def step(ev):
            if ev: ev[0].record()
            pr = probes_for(queries)
            order = order_for(pr)
            if ev: ev[1].record()
            trim.trim_search_knn(index, queries, k, gamma, batch, probes=pr, want_stats=False, out=out,
                                 query_order=order)
            if ev: ev[2].record()
        return step

    if args.traffic_child:      # (run under rocprofv3 by measure_traffic: the timed launch, a few times)
        step = make_step(main_ix)
        for _ in range(4):
            step(None)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_child": True, "gamma": gamma}))
        return
    t = timed_steps(args, make_step(main_ix))
    got = out[0].cpu().numpy()
    other = None
    if ix.list_bounds is not None and not args.no_list_bounds and not args.no_compare:
        # the same steps without the per-list summaries (no list-level pruning)
        t2 = timed_steps(args, make_step(ix_plain))
        other = dict(value=round(nq / (t2["ms_per_step"] * 1e-3), 1), ms_per_step=round(t2["ms_per_step"], 4),
                     kernel_ms=round(t2["scan_mean"], 4),
                     ids_equal=bool(np.array_equal(out[0].cpu().numpy(), got)))
    qps = nq / (t["ms_per_step"] * 1e-3)

    # ---- what the launch touched: one untimed launch with the kernel's work counters ----
    acc = run_once(main_ix, gamma, want_work=True)
    wt = work_totals(trim, acc["work"])
    assert np.array_equal(acc["ids"].cpu().numpy(), got)
    touched = touched_bytes(w, nq, nq * k, wt, False, 16 if fs else 256)
    # the task's byte model: codes + landmark distance per scanned candidate, raw row + id per
    # exact distance, the query itself and the k results; the table never leaves LDS
    alg_bytes = (chosen["n_scanned"] * (code_bytes + 4) + chosen["n_exact"] * (4 * w.d + 4) +
                 nq * (4 * w.d + 8 * k))
    roof = roofline_object(w, nq, t["scan_mean"], alg_bytes, wt, touched, ceil,
                           "search_kernel<knn, 4-bit codes>" if fs else "search_kernel<knn>", fs, traffic)

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload ----
    cpu = None
    if args.cpu_seconds > 0:
        ch = oix.centroids

        def chunk(lo, hi):
            qs = np.ascontiguousarray(qh[lo:hi])
            ph = trim_oracle.ivf_probe(qs, ch, w.nprobe) if w.nlist else None
            ro = orc.search_knn(oix, qs, k, gamma, batch, ph)
            return bool(np.array_equal(ro["ids"], got[lo:hi]))

        nthr = trim_oracle.num_threads()
        per_q = max(1, int(chosen["n_scanned"] / nq))
        big = max(nthr, min(nq, 1000, int(4e7 / per_q)))
        done, used, same = time_oracle(chunk, nq, args.cpu_seconds, big)
        set_threads(1)
        done1, used1, same1 = time_oracle(chunk, nq, args.cpu_seconds / 2, max(1, big // 32))
        set_threads(nthr)
        cpu = dict(value=round(done / used, 1), unit="queries/s", cores=nthr, kind="oracle",
                   sample=f"{done} queries (the query set in order, wrapping around) in {used:.1f} s: probe "
                          f"selection + scan, same index, gamma and batch; ids equal to the GPU's: {same}",
                   single_thread=dict(value=round(done1 / used1, 1), unit="queries/s", cores=1,
                                      sample=f"{done1} queries in {used1:.1f} s (one thread, the paper's "
                                             f"query protocol); ids equal: {same1}"))

    line = {
        "metric": "queries/sec at recall@10>=0.95 (1 MI355X); pruning ratio; scan HBM GB/s",
        "value": round(qps, 1), "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(t["ms_per_step"], 4),
        "ms_per_step_median": round(t["step_median"], 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n} base x {nq} queries, d={w.d}, "
                               + (f"PQ M={w.d // 2}x16 (4-bit codes), " if fs else f"PQ M={w.M}x256, ") +
                               f"IVF nlist={w.nlist} nprobe={w.nprobe}, kNN k={k}",
                   "gamma": gamma, "batch": batch, "recall_at_k": chosen["recall"],
                   "recall_truth": f"exact kNN over all n in float64 by the CPU oracle, first {nt} queries "
                                   f"({truth_s:.1f} s)",
                   "pruning_ratio": chosen["pruning_ratio"],
                   "list_level_pruning": main_ix.list_bounds is not None,
                   "without_list_level_pruning": other,
                   "timed": "probe selection + query ordering + fused table/scan/refine/select, inputs in HBM",
                   "setup_s": round(setup_s, 1)},
        "roofline": roof, "cpu_baseline": cpu, "ceilings": ceil, "sweep": sweep,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
