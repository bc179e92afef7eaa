#!/usr/bin/env python3
"""Benchmark of the ADC-scan hot path on one MI355X.

A step is one pass of the whole path -- distance tables, distance quantizer, scan
and top-R -- over one batch of queries against the resident code array.  The
headline workload is the PQ 16x4, R=100 exhaustive scan over N = 10,000,000
codes (d = 96), one query per step.  Inputs are seeded synthetic data resident in
HBM before the timed region.  Prints ONE JSON line.

Steps are issued round-robin on four HIP streams (independent requests in
flight), each with private buffers, so that the quantizer kernel of one step can
run beside the scan of another.  The roofline figure is for the scan
kernel alone: it is launched back to back through pq_adc_rescan_candidates between
two HIP events on its stream, and the elapsed time is divided by the launches.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
LLC_BYTES = 256 << 20   # last-level (Infinity) cache



def measured_traffic_bytes(workload, batch):
    """HBM bytes per scan-kernel launch from hardware counters, or None when this workload has
    not been profiled.  Read from the line `traffic_bytes_per_launch: <bytes>` of the summary
    profiles/k_scan_<workload>_batch<batch>.md, which `bench.py --summarize-pmc` writes from two
    rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE), each scaled by the same counter over the
    library's copy kernel of known size."""
    import re
    path = os.path.join(ROOT, "profiles", f"k_scan_{workload}_batch{batch}.md")
    try:
        with open(path) as f:
            m = re.search(r"^\s*traffic_bytes_per_launch:\s*([0-9.eE+]+)", f.read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def summarize_pmc(fetch_dir, write_dir):
    """Print the traffic summary of two rocprofv3 --pmc runs of this script (one with FETCH_SIZE,
    one with WRITE_SIZE, both with --copy-calibration): mean counter value per dispatch of the
    scan kernel's timing pass and of the copy kernel, the scale factors, and the line
    `traffic_bytes_per_launch:` that measured_traffic_bytes() reads."""
    import csv
    import glob

    def rows(d):
        out = []
        for fn in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            with open(fn, newline="") as f:
                out += list(csv.DictReader(f))
        return out

    def per_kernel(d, counter):
        by = {}
        for r in rows(d):
            if r.get("Counter_Name") != counter:
                continue
            name = r["Kernel_Name"]
            key = "k_copy" if "k_copy" in name else ("k_scan" if "k_scan" in name else None)
            if key:
                by.setdefault(key, []).append((int(r["Dispatch_Id"]), float(r["Counter_Value"])))
        return {k: [v for _, v in sorted(vs)] for k, vs in by.items()}

    lines, scaled = [], {}
    for counter, d in (("FETCH_SIZE", fetch_dir), ("WRITE_SIZE", write_dir)):
        by = per_kernel(d, counter)
        copy, scan = by.get("k_copy", []), by.get("k_scan", [])
        if not copy or not scan:
            raise SystemExit(f"{d}: no {counter} rows for k_copy / k_scan")
        tail = scan[-min(len(scan), 1600):]          # the timing pass comes last
        factor = 1048576.0 / (sum(copy) / len(copy))  # the copy moves 2^30 B = 1,048,576 KiB each way
        mean = sum(tail) / len(tail)
        scaled[counter] = mean * factor * 1024.0
        lines.append(f"{counter}: k_copy {sum(copy) / len(copy):.1f} KiB/dispatch over {len(copy)} (factor "
                     f"{factor:.4f}); k_scan timing pass {mean:.1f} KiB/dispatch over {len(tail)} "
                     f"-> {scaled[counter] / 1e6:.3f} MB")
    print("\n".join(lines))
    print(f"traffic_bytes_per_launch: {scaled['FETCH_SIZE'] + scaled['WRITE_SIZE']:.0f}")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--batch", type=int, default=1, help="queries per step")
    ap.add_argument("--streams", type=int, default=4, help="HIP streams the steps rotate over")
    ap.add_argument("--hw-queues", type=int, default=16,
                    help="hardware queues the HIP runtime may use for this process "
                         "(GPU_MAX_HW_QUEUES); streams beyond it share queues")
    ap.add_argument("--unfused", action="store_true",
                    help="issue pq_compute_tables, pq_quantize_tables and pq_adc_scan_topk as three "
                         "calls instead of the fused pq_search_topk (same arithmetic)")
    ap.add_argument("--workload", default="C1", choices=["C0", "C1", "C2", "C3", "C4", "C4coarse", "C1encode", "L8x8", "L664", "L655", "L16x8", "L664x2"],
                    help="C4 is the inverted-list search (ivf_adc_scan_topk); a step is one batch of "
                         "--batch queries (default there: 1000)")
    ap.add_argument("--kmeans-iters", type=int, default=3,
                    help="C4 only: Lloyd iterations for the synthetic coarse quantizer")
    ap.add_argument("--n", type=int, default=0, help="override the number of codes")
    ap.add_argument("--R", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the batch-32/256 legs")
    ap.add_argument("--cpu-queries", type=int, default=24)
    ap.add_argument("--reps", type=int, default=25,
                    help="repetitions of the timed train of --steps steps; the headline is the median")
    ap.add_argument("--summarize-pmc", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no benchmark: print the HBM-traffic summary of two rocprofv3 --pmc runs of "
                         "this script (FETCH_SIZE, WRITE_SIZE; both with --copy-calibration)")
    ap.add_argument("--copy-calibration", type=int, default=0,
                    help="also run this many plain 1 GiB device copies (library kernel k_copy, "
                         "known traffic) so that hardware counters collected around this run "
                         "can be scaled")
    return ap.parse_args()


class Runner:
    """Pre-resolved pointers so that a step is one (or three) C calls and nothing else.
    Step i runs on stream i % streams with that stream's private buffers."""

    def __init__(self, qb, idx, queries, codes, batch, R, t=400, streams=1, fused=True):
        import torch
        self.torch = torch
        self.lib = qb.load()
        self.qb, self.idx, self.batch, self.R, self.t = qb, idx, batch, R, t
        self.queries, self.codes = queries, codes
        self.nq_total = queries.shape[0] // batch * batch
        dev = codes.device
        self.n = codes.shape[0]
        self.fused = fused
        self.ws_bytes = (qb.pq_search_workspace_bytes if fused else qb.pq_workspace_bytes)(
            idx, batch, self.n, R)
        self.sets = []
        for _ in range(max(1, streams)):
            st = torch.cuda.current_stream() if streams <= 1 else torch.cuda.Stream(device=dev)
            bufs = dict(
                tables=torch.empty((batch, idx.table_len), dtype=torch.float32, device=dev),
                qt=torch.empty((batch, idx.table_len), dtype=idx.qdtype, device=dev),
                qp=torch.empty((batch, qb.QPARAMS_BYTES), dtype=torch.uint8, device=dev),
                ids=torch.empty((batch, R), dtype=torch.int32, device=dev),
                keys=torch.empty((batch, R), dtype=torch.uint16, device=dev),
                dist=torch.empty((batch, R), dtype=torch.float32, device=dev),
                ws=torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev))
            ptr = {k: v.data_ptr() for k, v in bufs.items()}
            self.sets.append((st, st.cuda_stream or None, bufs, ptr))
        self.h = idx.handle
        self.qbase = queries.data_ptr()
        self.qrow = queries.shape[1] * 4
        self.cptr = codes.data_ptr()

    def step(self, i, off=None):
        lib = self.lib
        _, stream, _, p = self.sets[i % len(self.sets)]
        if off is None:
            off = (i * self.batch) % self.nq_total
        if self.fused:
            rc = lib.pq_search_topk(self.h, self.qbase + off * self.qrow, self.batch, self.cptr,
                                    self.n, self.t, self.R, p["ids"], p["keys"], p["dist"], p["ws"],
                                    self.ws_bytes, stream)
        else:
            rc = lib.pq_compute_tables(self.h, self.qbase + off * self.qrow, self.batch,
                                       p["tables"], stream)
            rc |= lib.pq_quantize_tables(self.h, p["tables"], self.batch, self.cptr, self.n, self.t,
                                         self.R, p["qt"], p["qp"], stream)
            rc |= lib.pq_adc_scan_topk(self.h, p["qt"], p["qp"], self.batch, self.cptr, self.n,
                                       self.R, p["ids"], p["keys"], p["dist"], p["ws"],
                                       self.ws_bytes, stream)
        if rc != 0:
            raise RuntimeError("libqadc: " + lib.pq_last_error().decode())

    def prime(self, rounds=3):
        """Use every stream set (and so every hardware queue) a few times: the first launches
        on a stream create its queue and load code objects, which is not steady state."""
        for _ in range(rounds):
            for i in range(len(self.sets)):
                self.step(i)
        self.torch.cuda.synchronize()

    def run(self, steps, warmup, reps=1):
        """`warmup` untimed steps, then `reps` trains of exactly `steps` steps, each bracketed
        by a device synchronisation on both sides.  Returns the list of train times (s)."""
        torch = self.torch
        self.prime()
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        times, issue = [], []
        k = warmup
        for _ in range(max(1, reps)):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                self.step(k + i)
            t1 = time.perf_counter()
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t0)
            issue.append(t1 - t0)             # host time to enqueue the steps
            k += steps
        self.issue_s = sorted(issue)[len(issue) // 2]
        return times

    def result_of(self, q0):
        """Run the path for queries [q0, q0+batch) on stream set 0 and return numpy outputs."""
        torch = self.torch
        torch.cuda.synchronize()
        self.step(0, off=q0)  # stream set 0, queries starting at q0
        torch.cuda.synchronize()
        b = self.sets[0][2]
        return b["ids"].cpu().numpy(), b["keys"].cpu().numpy(), b["dist"].cpu().numpy()


def scan_kernel_time(qb, idx, queries, codes, batch, R, nsamples=8, reps=200, t=400):
    """Average duration of one scan-kernel launch: `reps` back-to-back launches between two
    HIP events on the launching stream, for `nsamples` different query batches."""
    import torch
    n = codes.shape[0]
    ws = torch.empty(qb.pq_workspace_bytes(idx, batch, n, R), dtype=torch.uint8, device=codes.device)
    stream = torch.cuda.current_stream()
    total_ms, launches = 0.0, 0
    for s in range(nsamples):
        q = queries[s * batch:(s + 1) * batch].contiguous()
        tables = qb.pq_compute_tables(idx, q)
        qt, qp = qb.pq_quantize_tables(idx, tables, codes, t, R)
        qb.pq_adc_scan_candidates(idx, qt, qp, codes, R, ws)   # prepares the tables in ws
        for _ in range(2):
            qb.pq_adc_rescan_candidates(idx, qt, qp, codes, R, ws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            qb.pq_adc_rescan_candidates(idx, qt, qp, codes, R, ws)
        e1.record(stream)
        e1.synchronize()
        total_ms += e0.elapsed_time(e1)
        launches += reps
    return total_ms / launches, launches


def isolated_latency(run, nsteps=200):
    """One query at a time on one stream with a device synchronisation after each: the wall
    time a lone request sees.  Returns (median_ms, min_ms)."""
    torch = run.torch
    times = []
    for i in range(nsteps + 20):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run.step(0, off=(i * run.batch) % run.nq_total)
        torch.cuda.synchronize()
        if i >= 20:
            times.append((time.perf_counter() - t0) * 1e3)
    times.sort()
    return times[len(times) // 2], times[0]


def graph_replay_latency(run, ngraphs=16, nsteps=200):
    """The same lone request as isolated_latency with the call recorded once into a HIP graph
    per query (a call with a workspace only enqueues kernels) and replayed: what a serving loop
    that pre-records its steps sees.  Returns (median_ms, min_ms, replays checked)."""
    torch = run.torch
    side = torch.cuda.Stream()
    _, _, bufs, _ = run.sets[0]
    keep = run.sets[0]
    run.sets[0] = (side, side.cuda_stream, bufs, keep[3])
    graphs = []
    try:
        with torch.cuda.stream(side):
            run.step(0, off=0)
        torch.cuda.synchronize()
        for g in range(ngraphs):
            cg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(cg, stream=side):
                run.step(0, off=(g * run.batch) % run.nq_total)
            graphs.append(cg)
    finally:
        run.sets[0] = keep
    torch.cuda.synchronize()
    # every replay must give what the eager call gives
    checked = 0
    for g in (0, ngraphs - 1, 1, 0):
        want = run.result_of((g * run.batch) % run.nq_total)
        for b in ("ids", "keys", "dist"):
            bufs[b].zero_()
        graphs[g].replay()
        torch.cuda.synchronize()
        got = bufs["ids"].cpu().numpy(), bufs["keys"].cpu().numpy(), bufs["dist"].cpu().numpy()
        if not all((x == y).all() for x, y in zip(want, got)):
            raise RuntimeError("graph replay differs from the eager call")
        checked += 1
    times = []
    for i in range(nsteps + 20):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        graphs[i % ngraphs].replay()
        torch.cuda.synchronize()
        if i >= 20:
            times.append((time.perf_counter() - t0) * 1e3)
    times.sort()
    return times[len(times) // 2], times[0], checked


def cold_scan_kernel_time(qb, idx, queries, codes, R, copies=5, reps=40, t=400):
    """The scan kernel over `copies` separate copies of the code array in turn (together larger
    than the 256 MB last-level cache), so that every launch streams its codes from HBM."""
    import torch
    n = codes.shape[0]
    bufs = [codes] + [codes.clone() for _ in range(copies - 1)]
    q = queries[:1].contiguous()
    tables = qb.pq_compute_tables(idx, q)
    qt, qp = qb.pq_quantize_tables(idx, tables, codes, t, R)
    wss = []
    for b in bufs:
        ws = torch.empty(qb.pq_workspace_bytes(idx, 1, n, R), dtype=torch.uint8, device=codes.device)
        qb.pq_adc_scan_candidates(idx, qt, qp, b, R, ws)
        wss.append(ws)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for r in range(reps):
        for b, ws in zip(bufs, wss):
            qb.pq_adc_rescan_candidates(idx, qt, qp, b, R, ws)
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) / (reps * copies)


def cpu_baseline(pr, R, nq, t=400):
    """The oracle, as it stands, on a bounded sample: nq whole-list queries, one per thread."""
    import oracle
    lay = pr.layout
    codes = pr.codes.cpu().numpy()
    cb = pr.codebooks.cpu().numpy()
    qs = pr.queries[:nq].cpu().numpy()
    oracle.search(lay.d, lay.nbits, lay.dsub, lay.acc_bits, cb, qs[0], codes[:1000], t, R)  # load
    threads = min(nq, os.cpu_count() or 1, 16)

    def one(q):
        return oracle.search(lay.d, lay.nbits, lay.dsub, lay.acc_bits, cb, qs[q], codes, t, R)

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = list(ex.map(one, range(nq)))
    return res, time.perf_counter() - t0, threads


def main():
    a = parse()
    if a.summarize_pmc:
        return summarize_pmc(*a.summarize_pmc)
    if a.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (multi-GPU sharding is a "
              "design note only, no collective code exists)", file=sys.stderr)
        sys.exit(2)
    # must be in the environment before the HIP runtime starts: independent requests only
    # overlap on the GPU when their streams sit on different hardware queues
    os.environ["GPU_MAX_HW_QUEUES"] = str(max(1, min(a.hw_queues, 32)))
    if a.workload == "C4":
        return main_ivf(a)
    if a.workload == "C4coarse":
        return main_coarse(a)
    if a.workload == "C1encode":
        return main_encode(a)
    import numpy as np
    import torch
    from paper_1812_09162_amd import binding as qb
    from harness import synth

    assert torch.cuda.is_available(), "bench.py needs the GPU; there is no CPU fallback"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = dict(synth.CONFIGS[a.workload])
    if a.n:
        cfg["n"] = a.n
    cfg["nq"] = min(cfg["nq"], 10_000)
    t_build = time.perf_counter()
    pr = synth.build(cfg, device=dev)
    torch.cuda.synchronize()
    t_build = time.perf_counter() - t_build
    lay = pr.layout
    n, cs = pr.codes.shape
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, pr.codebooks, lay.acc_bits)

    if a.copy_calibration:
        # kernel k_copy on 1 GiB (larger than the 256 MB Infinity Cache): 2^30 bytes read from
        # HBM and 2^30 written, i.e. 1048576 KiB each in FETCH_SIZE / WRITE_SIZE units
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(a.copy_calibration):
            qb.pq_copy_bytes(dst, src)
        torch.cuda.synchronize()
        del src, dst


    # headline: whole path, `batch` queries per step; `reps` trains of exactly `steps` steps
    run = Runner(qb, idx, pr.queries, pr.codes, a.batch, a.R, streams=a.streams, fused=not a.unfused)
    trains = sorted(run.run(a.steps, a.warmup, a.reps))
    dt = trains[len(trains) // 2]                      # median train
    ms_per_step = dt / a.steps * 1e3
    codes_per_s = a.batch * n * a.steps / dt
    # a short train does not reach the steady state (streams that start together stay in step for
    # their first queries): the long-train figure is reported beside `value`, never in its place
    steady = None
    if a.steps < 1000 and a.batch == 1:
        long_trains = sorted(run.run(1000, 0, 9))
        steady = {"steps": 1000, "reps": 9, "ms_per_step": long_trains[4] / 1000 * 1e3,
                  "gcodes_per_s": n * 1000 / long_trains[4] / 1e9}

    # dominant kernel: the scan, timed alone with HIP events on its stream
    k_avg_ms, k_cnt = scan_kernel_time(qb, idx, pr.queries, pr.codes, a.batch, a.R)
    alg_bytes = float(n) * cs  # every code byte is read once per launch, whatever the batch
    achieved = alg_bytes / (k_avg_ms * 1e-3) / 1e9
    resident = n * cs <= LLC_BYTES
    roofline = {"bound": "hbm", "kernel": "k_scan", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": measured_traffic_bytes(a.workload, a.batch),
                "kernel_avg_ms": k_avg_ms, "launches": k_cnt,
                "algorithmic_bytes_per_launch": alg_bytes,
                "residency": (f"the {n * cs / 1e6:.0f} MB code array is rescanned back to back and stays in the "
                              f"256 MB last-level cache: `frac` is a cache-resident figure, `frac_cold` the one "
                              f"streamed from HBM" if resident else
                              f"the {n * cs / 1e6:.0f} MB code array exceeds the 256 MB last-level cache")}
    if n * cs <= (1 << 30) and not a.no_extras:
        cold_ms = cold_scan_kernel_time(qb, idx, pr.queries, pr.codes, a.R)
        roofline["achieved_cold"] = alg_bytes / cold_ms / 1e6
        roofline["frac_cold"] = alg_bytes / cold_ms / 1e6 / HBM_PEAK_GBS
        roofline["kernel_avg_ms_cold"] = cold_ms
        roofline["cold_note"] = "5 separate copies of the code array scanned in turn (more than the last-level cache)"

    extras = {}
    if not a.no_extras:
        # a second denominator next to the published peak: what a plain copy kernel of this
        # library moves on this GPU (1 GiB read + 1 GiB written, more than the last-level cache)
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        best = None
        for _ in range(4):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            qb.pq_copy_bytes(dst, src)
            e1.record()
            e1.synchronize()
            gbs = 2.0 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
            best = gbs if best is None or gbs > best else best
        del src, dst
        roofline["measured_copy_gbs"] = best
        roofline["frac_of_measured_copy"] = achieved / best
        if "achieved_cold" in roofline:
            roofline["frac_cold_of_measured_copy"] = roofline["achieved_cold"] / best
        lat = Runner(qb, idx, pr.queries, pr.codes, a.batch, a.R, streams=1, fused=not a.unfused)
        med, mn = isolated_latency(lat)
        extras["isolated_latency_ms"] = {"median": med, "min": mn,
                                         "note": "one step at a time, host-synchronised"}
        gmed, gmn, gchk = graph_replay_latency(lat)
        extras["isolated_latency_ms"]["graph_replay"] = {
            "median": gmed, "min": gmn, "replays_equal_to_eager": gchk,
            "note": "the same step recorded once per query into a HIP graph and replayed"}
        # query-batched passes: bound by LDS reads, not HBM.  Ceiling: one 8-byte table entry per
        # lane, 16 lanes per CU and clock without bank conflicts (128 B/clk) = 256 CUs x 16 x 2.4 GHz
        lds_ceiling = 256 * 16 * 2.4e9
        # the same read measured on this GPU for the kernel's own address pattern (every lane an
        # independent entry of a 2 KB table: bank conflicts included) and for a conflict-free one
        lds_measured = {}
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        for name, pat in (("conflict_free", qb.PQ_LDS_LINEAR), ("random_2kb_table", qb.PQ_LDS_RANDOM_2K)):
            best = None
            for _ in range(4):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                nreads = qb.pq_lds_read_probe(pat, 2048, sink)
                e1.record()
                e1.synchronize()
                rate = nreads / (e0.elapsed_time(e1) * 1e-3)
                best = rate if best is None or rate > best else best
            lds_measured[name] = best
        for bs, st in ((32, 60), (256, 12)):
            r2 = Runner(qb, idx, pr.queries, pr.codes, bs, a.R, streams=min(a.streams, 2),
                        fused=not a.unfused)
            d2 = sorted(r2.run(st, 2, 5))[2]
            kms, _ = scan_kernel_time(qb, idx, pr.queries, pr.codes, bs, a.R, nsamples=2, reps=5)
            # one LDS read of an 8-byte entry serves four queries' lookups of one group
            # (m x 4 layouts: a group is a code byte; irregular layouts: ng groups per code)
            groups = lay.m // 2 if set(lay.nbits) == {4} else None
            reads = ((bs + 3) // 4) * groups * float(n) if groups else None
            extras[f"batch{bs}"] = {
                "ms_per_step": d2 / st * 1e3,
                "gcodes_per_s": bs * n * st / d2 / 1e9,
                "glookups_per_s": bs * n * lay.m * st / d2 / 1e9,
                "scan_kernel_ms": kms,
                "scan_kernel_glookups_per_s": bs * n * lay.m / (kms * 1e-3) / 1e9,
            }
            if reads:
                extras[f"batch{bs}"]["roofline"] = {
                    "bound": "lds", "kernel": "k_scan_mq", "unit": "G 8-byte LDS reads/s",
                    "achieved": reads / (kms * 1e-3) / 1e9, "peak": lds_ceiling / 1e9,
                    "frac": reads / (kms * 1e-3) / lds_ceiling, "lds_reads_per_launch": reads,
                    "peak_measured_conflict_free": lds_measured["conflict_free"] / 1e9,
                    "peak_measured_random_2kb_table": lds_measured["random_2kb_table"] / 1e9,
                    "frac_of_measured_random": reads / (kms * 1e-3) / lds_measured["random_2kb_table"]}
        if a.workload == "C1" and a.batch == 1:
            extras["C2_streaming"] = streaming_leg(qb, synth, dev, "C2", 100)

    entry = ("pq_compute_tables+pq_quantize_tables+pq_adc_scan_topk" if a.unfused
             else "pq_search_topk")
    out = {
        "metric": ("billion codes scanned/sec per GPU (PQ 16x4, R=100), whole path per query"
                   if a.workload == "C1" and a.R == 100 else
                   f"billion codes scanned/sec per GPU ({a.workload}, R={a.R}), whole path per query"),
        "value": codes_per_s / 1e9,
        "unit": "Gcodes/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8" if lay.acc_bits == 8 else "u16",
        "data": "synthetic",
        "config": {"workload": f"{a.workload}: exhaustive ADC, N={n}, d={lay.d}, m={lay.m}, "
                               f"bits={sorted(set(lay.nbits))}, code_bytes={cs}, R={a.R}, t=400, "
                               f"batch={a.batch}, streams={a.streams}, hw_queues={a.hw_queues}, entry={entry}",
                   "seed": cfg["seed"], "dataset_build_s": round(t_build, 2)},
        # `value` and `ms_per_step` are the median of `reps` trains of exactly `steps` steps, each
        # train bracketed by a device synchronisation on both sides
        "timing": {"reps": len(trains), "ms_per_step_median": ms_per_step,
                   "ms_per_step_min": trains[0] / a.steps * 1e3,
                   "ms_per_step_max": trains[-1] / a.steps * 1e3,
                   "ms_per_step_mean": sum(trains) / len(trains) / a.steps * 1e3,
                   "steady_state_long_train": steady},
        "whole_path_hbm_gbs": codes_per_s * cs / 1e9,
        "whole_path_frac_of_hbm_peak": codes_per_s * cs / 1e9 / HBM_PEAK_GBS,
        "host_issue_ms_per_step": run.issue_s / a.steps * 1e3,
        "roofline": roofline,
        "batched": extras,
        # the paper's own figure for this layout, another machine and size: context, not a baseline
        "paper_context": {"value": 1.89, "unit": "Gcodes/s",
                          "what": "Table 3, m x {4,4} 64-bit codes, uint8, AVX-512BW shuffles: 0.53 ms per "
                                  "query over 1,000,000 codes, one core of a Xeon Platinum 8175 (Section 4.1)"},
    }

    if not a.no_cpu_baseline:
        res, cdt, threads = cpu_baseline(pr, a.R, a.cpu_queries)
        try:
            usable = len(os.sched_getaffinity(0))
        except AttributeError:
            usable = os.cpu_count()
        out["cpu_baseline"] = {"value": a.cpu_queries * n / cdt / 1e9, "unit": "Gcodes/s",
                               "cores": threads, "kind": "oracle",
                               "gcodes_per_s_per_core": a.cpu_queries * n / cdt / 1e9 / threads,
                               "nproc": os.cpu_count(), "usable_cpus": usable,
                               "sample": f"{a.cpu_queries} queries x {n} codes (the full list), "
                                         f"one query per thread on {threads} threads, {cdt:.1f} s wall"}
        # parity of the timed configuration against the same oracle results
        ok = True
        for q0 in range(0, min(a.cpu_queries, run.nq_total), max(1, a.batch)):
            ids, keys, dist = run.result_of(q0)
            for j in range(min(a.batch, a.cpu_queries - q0)):
                oi, okk, od = res[q0 + j]
                ok = ok and np.array_equal(ids[j], oi) and np.array_equal(
                    keys[j].astype(np.uint16), okk) and np.array_equal(dist[j], od)
        out["parity_sample"] = {"queries": a.cpu_queries, "bit_exact": bool(ok)}
    print(json.dumps(out))


def streaming_leg(qb, synth, dev, name, R):
    """The scan kernel alone on another exhaustive configuration (C2: 320 MB of codes, more than
    the last-level cache, so every launch streams from HBM), one query per launch."""
    import torch
    cfg = dict(synth.CONFIGS[name])
    cfg["nq"] = 16
    pr = synth.build(cfg, device=dev)
    lay = pr.layout
    n, cs = pr.codes.shape
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, pr.codebooks, lay.acc_bits)
    ms, cnt = scan_kernel_time(qb, idx, pr.queries, pr.codes, 1, R, nsamples=4, reps=50)
    cold = cold_scan_kernel_time(qb, idx, pr.queries, pr.codes, R, copies=4, reps=10)
    run = Runner(qb, idx, pr.queries, pr.codes, 1, R, streams=8)
    trains = sorted(run.run(100, 16, 9))
    torch.cuda.synchronize()
    idx.close()
    nb = float(n) * cs
    return {"workload": f"{name}: N={n}, code_bytes={cs}, R={R}, batch=1",
            "scan_kernel_ms": ms, "launches": cnt, "gb_per_s": nb / ms / 1e6,
            "frac_of_hbm_peak": nb / ms / 1e6 / HBM_PEAK_GBS,
            "scan_kernel_ms_cold": cold, "frac_of_hbm_peak_cold": nb / cold / 1e6 / HBM_PEAK_GBS,
            "whole_path_ms_per_query": trains[len(trains) // 2] / 100 * 1e3,
            "whole_path_frac_of_hbm_peak": nb / (trains[len(trains) // 2] / 100) / 1e9 / HBM_PEAK_GBS}


def main_ivf(a):
    """Workload C4: residual PQ 16x4 behind a coarse quantizer, nprobe lists per query."""
    import numpy as np
    import torch
    from paper_1812_09162_amd import binding as qb
    from harness import synth
    assert torch.cuda.is_available(), "bench.py needs the GPU; there is no CPU fallback"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = dict(synth.CONFIGS["C4"])
    cfg["kmeans_iters"] = a.kmeans_iters
    if a.n:
        cfg["n"] = a.n
        cfg["K"] = max(64, int(cfg["K"] * a.n / synth.CONFIGS["C4"]["n"]))
    t_build = time.perf_counter()
    ip = synth.build(cfg, device=dev)
    torch.cuda.synchronize()
    t_build = time.perf_counter() - t_build
    lay = ip.layout
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, ip.codebooks, lay.acc_bits)
    nq_all, nprobe = ip.probe_ids.shape
    bs = a.batch if a.batch > 1 else 1000
    bs = min(bs, nq_all)
    sizes = ip.list_offsets[1:] - ip.list_offsets[:-1]
    probed = sizes[ip.probe_ids.long()].sum(dim=1)  # codes scanned per query
    ws = torch.empty(qb.ivf_sorted_workspace_bytes(idx, bs, nprobe, a.R, ip.coarse.shape[0]), dtype=torch.uint8,
                     device=dev)
    out = (torch.empty((bs, a.R), dtype=torch.int32, device=dev),
           torch.empty((bs, a.R), dtype=torch.float32, device=dev))

    def go(i):
        lo = (i * bs) % (nq_all - bs + 1)
        qb.ivf_adc_scan_topk(idx, ip.coarse, ip.list_offsets, ip.list_codes, ip.list_ids,
                             ip.queries[lo:lo + bs], ip.probe_ids[lo:lo + bs], 400, a.R,
                             workspace=ws, out=out)
        return lo

    steps = min(a.steps, 200)
    for i in range(min(a.warmup, 5)):
        go(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        go(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = float(probed.float().mean().item()) * bs
    cs = ip.list_codes.shape[1]
    # the optional mode whose quantization bound tightens list by list (one block per query)
    tsteps = max(1, min(steps, 20))
    for i in range(2):
        qb.ivf_adc_scan_topk_tightening(idx, ip.coarse, ip.list_offsets, ip.list_codes, ip.list_ids,
                                        ip.queries[:bs], ip.probe_ids[:bs], 400, a.R, workspace=ws, out=out)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(tsteps):
        lo = (i * bs) % (nq_all - bs + 1)
        qb.ivf_adc_scan_topk_tightening(idx, ip.coarse, ip.list_offsets, ip.list_codes, ip.list_ids,
                                        ip.queries[lo:lo + bs], ip.probe_ids[lo:lo + bs], 400, a.R,
                                        workspace=ws, out=out)
    torch.cuda.synchronize()
    dt_t = time.perf_counter() - t1
    out_d = {
        "metric": "billion codes scanned/sec per GPU (IVF, residual PQ 16x4, R=100), whole path",
        "value": per_step * steps / dt / 1e9, "unit": "Gcodes/s", "n_gpus": 1, "steps": steps,
        "warmup": min(a.warmup, 5), "ms_per_step": dt / steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"C4: IVF ADC, N={ip.list_codes.shape[0]}, K={ip.coarse.shape[0]}, "
                               f"nprobe={nprobe}, d={lay.d}, m={lay.m}, code_bytes={cs}, R={a.R}, t=400, "
                               f"batch={bs}, coarse k-means iterations={a.kmeans_iters}, "
                               f"entry=ivf_adc_scan_topk",
                   "seed": cfg["seed"], "dataset_build_s": round(t_build, 1),
                   "codes_scanned_per_query": float(probed.float().mean().item())},
        "us_per_query": dt / steps / bs * 1e6,
        "list_bytes_per_s_gb": per_step * steps / dt * (cs + 0) / 1e9,
        # bytes of list codes a step reads (every probed list once per query that probes it) and
        # what it would read if each distinct probed list were read once per step
        "list_bytes_per_step": {
            "as_read": per_step * cs,
            "distinct_lists_once": float(sizes[torch.unique(ip.probe_ids[:bs].long())].sum().item()) * cs,
        },
        "tightening_mode": {"entry": "ivf_adc_scan_topk_tightening", "steps": tsteps,
                            "ms_per_step": dt_t / tsteps * 1e3,
                            "gcodes_per_s": per_step * tsteps / dt_t / 1e9},
    }
    print(json.dumps(out_d))


def main_coarse(a):
    """The step before workload C4: nearest 64 of 65,536 cells for 10,000 queries, d = 96
    (ivf_coarse_search).  A step is one call over all queries.  Roofline: fp32 matrix cores."""
    import torch
    from paper_1812_09162_amd import binding as qb
    assert torch.cuda.is_available(), "bench.py needs the GPU; there is no CPU fallback"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, d, nq, nprobe = 65_536, 96, 10_000, 64
    g = torch.Generator(device=dev).manual_seed(18120921)
    cen = torch.randn((K, d), generator=g, device=dev, dtype=torch.float32)
    cen = cen / cen.norm(dim=1, keepdim=True)
    qs = torch.randn((nq, d), generator=g, device=dev, dtype=torch.float32)
    qs = qs / qs.norm(dim=1, keepdim=True)
    ws = torch.empty(qb.ivf_coarse_workspace_bytes(nq, K), dtype=torch.uint8, device=dev)
    out = (torch.empty((nq, nprobe), dtype=torch.int32, device=dev),
           torch.empty((nq, nprobe), dtype=torch.float32, device=dev))
    steps = min(a.steps, 20)
    for _ in range(2):
        qb.ivf_coarse_search(qs, cen, nprobe, workspace=ws, out=out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        qb.ivf_coarse_search(qs, cen, nprobe, workspace=ws, out=out)
    e1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    flops = 2.0 * nq * K * d
    ms = e0.elapsed_time(e1) / steps
    print(json.dumps({
        "metric": "queries routed/sec per GPU (nearest 64 of 65,536 cells, d=96)",
        "value": nq * steps / dt, "unit": "queries/s", "n_gpus": 1, "steps": steps, "warmup": 2,
        "ms_per_step": dt / steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"C4coarse: K={K}, d={d}, nq={nq}, nprobe={nprobe}, entry=ivf_coarse_search",
                   "seed": 18120921},
        "roofline": {"bound": "mfma", "kernel": "k_scores + k_select (whole call)",
                     "achieved": flops / (ms * 1e-3) / 1e12, "peak": 157.3, "unit": "TFLOP/s",
                     "frac": flops / (ms * 1e-3) / 1e12 / 157.3, "traffic": None,
                     "call_ms_by_events": ms, "flops_per_call": flops},
    }))


def main_encode(a):
    """Index build side of workload C1: 10,000,000 vectors of d = 96 encoded to 16x4 codes
    (pq_encode).  A step is one call over all vectors.  Roofline: vector ALU.  eq. (1) read
    literally is a subtract, a multiply and an add per (centroid, dimension), none fused or
    packed, so the ceiling is one such operation per lane and cycle: 256 CUs x 4 SIMDs x 16
    lanes x 2.4 GHz = 39.3 T operations/s."""
    import torch
    from paper_1812_09162_amd import binding as qb
    from harness import synth
    assert torch.cuda.is_available(), "bench.py needs the GPU; there is no CPU fallback"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = synth.scaled("C1", n=100_000, nq=1)
    pr = synth.build(cfg, device=dev)
    lay = pr.layout
    n = a.n or 10_000_000
    g = torch.Generator(device=dev).manual_seed(18120922)
    x = torch.randn((n, lay.d), generator=g, device=dev, dtype=torch.float32)
    idx = qb.PqIndex(lay.d, lay.nbits, lay.dsub, pr.codebooks, lay.acc_bits)
    codes = torch.empty((n, idx.code_size), dtype=torch.uint8, device=dev)
    steps = min(a.steps, 20)
    for _ in range(2):
        qb.pq_encode(idx, x, codes=codes)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        qb.pq_encode(idx, x, codes=codes)
    e1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = e0.elapsed_time(e1) / steps
    nbytes = float(n) * (lay.d * 4 + idx.code_size)
    ops = float(n) * 3.0 * sum((1 << b) * s for b, s in zip(lay.nbits, lay.dsub))
    print(json.dumps({
        "metric": "vectors encoded/sec per GPU (PQ 16x4, d=96)",
        "value": n * steps / dt, "unit": "vectors/s", "n_gpus": 1, "steps": steps, "warmup": 2,
        "ms_per_step": dt / steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"C1encode: n={n}, d={lay.d}, m={lay.m}, bits=4, entry=pq_encode", "seed": 18120922},
        "roofline": {"bound": "alu", "kernel": "k_encode", "achieved": ops / (ms * 1e-3) / 1e12,
                     "peak": 39.3, "unit": "TFLOP/s", "frac": ops / (ms * 1e-3) / 1e12 / 39.3,
                     "traffic": None, "kernel_avg_ms": ms, "flops_per_launch": ops,
                     "hbm_gb_per_s": nbytes / (ms * 1e-3) / 1e9},
    }))


if __name__ == "__main__":
    main()
