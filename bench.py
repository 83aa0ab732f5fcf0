#!/usr/bin/env python3
"""Benchmark of the bucketed approximate top-k hot path on one MI355X.

One step = one pass of the whole hot path over the headline workload (arxiv 2412.04358,
Figure 1 left, restated synthetically): m=128 rows of n=65536 float32 N(0,1), k=64,
k_b=1, b swept over {64, 128, 256, 512, 1024} (b*k_b/k = 1..16; Stage 2 runs for b > 64).
That is five approx_topk calls per step.  Every call reads a different, already resident
input buffer from a ring larger than the 256 MB Infinity Cache, so each launch streams its
rows from HBM ("cold"); the same-buffer ("warm") figure is reported beside it.

Metric: total bandwidth = minimum bytes (m*n*4 read + m*k*8 written) / runtime
(Figure 1 caption), in GB/s and as a fraction of the 8 TB/s HBM peak.
Prints one JSON line.
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

HBM_PEAK_GBPS = 8000.0
M, N, K = 128, 65536, 64
SWEEP_B = [64, 128, 256, 512, 1024]
RING = 12  # 12 x 33.5 MB = 403 MB > 256 MB Infinity Cache


def min_bytes(m, n, k, es=4):
    return m * n * es + m * k * (es + 4)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--detail", action="store_true", help="also time every configuration of the paper's sweeps")
    ap.add_argument("--probe-long", action="store_true",
                    help="profiler run on the 128 x 2^20 rows (cfg4, k=64, k_b=1): 5 plain copies, 5 read-only kernels, "
                         "20 approx_topk calls each at b=64 and b=1024; no timing")
    ap.add_argument("--probe-exact", action="store_true",
                    help="profiler run of exact_topk: 10 calls each on 128 x 65536 f32 (k=64, k=16384) and on "
                         "128 x 2^20 f32 (k=64, k=2^18); no timing")
    ap.add_argument("--timeline", action="store_true",
                    help="phase timeline of the fused kernel on the headline workload: per b, 30 launches of the "
                         "measurement build (atk_trace_approx) on HBM-cold inputs, each right behind an ordinary launch; "
                         "prints when the first, the median and the last wavefront passed every phase boundary")
    ap.add_argument("--probe-floors", action="store_true",
                    help="cfg4 with eight-slot queues (k=64, b=8 and b=128), 10 calls each without and with pooled floors (for rocprofv3)")
    ap.add_argument("--probe-small", action="store_true",
                    help="small batches of long rows (k=64, k_b=1; 1 x 2^20, 8 x 2^20, 32 x 2^17 at b=64 and b=256; 64 x 2^18 at "
                         "b=512): 10 calls each with row splits through scratch (plan override MH=0), then with the library's "
                         "own plan - helpers and a finisher (for rocprofv3)")
    ap.add_argument("--probe-queues", action="store_true",
                    help="profiler run of the kernels with register queues: 5 plain copies, then 20 approx_topk calls each on "
                         "cfg3 (128 x 65536 f32, k=16384) at k_b = 1, 4, 8, 16 and on cfg5 (2048 x 8192 bf16, k=b=512); no timing")
    ap.add_argument("--probe", action="store_true",
                    help="short run for hardware-counter passes: 20 copy launches, 20 read-only launches and 20 "
                         "approx_topk launches per b, nothing else")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (rows shard with no exchange); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2412_04358_amd as atk
    from paper_2412_04358_amd import workloads

    if not os.path.exists(atk.lib_path()):
        import __graft_entry__

        __graft_entry__.build()
    lib = atk.load_library()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.probe_exact:
        st = torch.cuda.current_stream().cuda_stream
        cases = [(1 << 16, 64), (1 << 16, 16384), (1 << 20, 64), (1 << 20, 1 << 18)]
        for n_row, k in cases:
            xe = workloads.normal_rows(M, n_row, seed=0).to(dev)
            ov = torch.empty((M, k), dtype=torch.float32, device=dev)
            oi = torch.empty((M, k), dtype=torch.int32, device=dev)
            for i in range(10):
                rc = atk.exact_topk_raw(xe.data_ptr(), M, n_row, k, atk.ATK_F32, ov.data_ptr(), oi.data_ptr(), st)
                if rc != 0:
                    raise RuntimeError("exact_topk failed: %s" % atk.strerror(rc))
            torch.cuda.synchronize()
            del xe, ov, oi
        print(json.dumps({"probe": "done", "calls_each": 10, "cases": [[M, n_row, k] for n_row, k in cases]}))
        return

    if args.probe_queues:
        st = torch.cuda.current_stream().cuda_stream
        ring = [workloads.normal_rows(M, N, seed=s).to(dev) for s in range(RING)]
        dst = torch.empty_like(ring[0])
        for i in range(5):
            lib.atk_copy(dst.data_ptr(), ring[i % RING].data_ptr(), M * N * 4, st)
        ov = torch.empty((M, 16384), dtype=torch.float32, device=dev)
        oi = torch.empty((M, 16384), dtype=torch.int32, device=dev)
        for k_b in (1, 4, 8, 16):
            for i in range(20):
                rc = lib.approx_topk(ring[i % RING].data_ptr(), M, N, 16384, 16384 // k_b, k_b, atk.ATK_F32, ov.data_ptr(),
                                     oi.data_ptr(), st)
                if rc != 0:
                    raise RuntimeError("approx_topk failed: %s" % atk.strerror(rc))
        torch.cuda.synchronize()
        del ring, dst
        ring5 = [workloads.attention_scores(seed=s).to(dev) for s in range(RING)]
        ov5 = torch.empty((2048, 512), dtype=torch.bfloat16, device=dev)
        oi5 = torch.empty((2048, 512), dtype=torch.int32, device=dev)
        for i in range(20):
            rc = lib.approx_topk(ring5[i % RING].data_ptr(), 2048, 8192, 512, 512, 1, atk.ATK_BF16, ov5.data_ptr(),
                                 oi5.data_ptr(), st)
            if rc != 0:
                raise RuntimeError("approx_topk failed: %s" % atk.strerror(rc))
        torch.cuda.synchronize()
        print(json.dumps({"probe": "done", "copy_bytes": M * N * 4, "launches_each": 20, "cfg3_k_b": [1, 4, 8, 16], "cfg5": True}))
        return

    if args.probe_floors:
        n_long = 1 << 20
        xl = workloads.normal_rows(M, n_long, seed=0).to(dev)
        ov = torch.empty((M, K), dtype=torch.float32, device=dev)
        oi = torch.empty((M, K), dtype=torch.int32, device=dev)
        st = torch.cuda.current_stream().cuda_stream
        plans = {}
        for spec in ("RF=0", ""):  # the override only decides whether the lanes pool their floors
            atk.set_plan_override(spec)
            for b in (8, 128):
                plans["b=%d %s" % (b, spec or "default")] = atk.plan_describe(M, n_long, K, b, 8)
                for i in range(10):
                    rc = lib.approx_topk(xl.data_ptr(), M, n_long, K, b, 8, atk.ATK_F32, ov.data_ptr(), oi.data_ptr(), st)
                    if rc != 0:
                        raise RuntimeError("approx_topk failed: %s" % atk.strerror(rc))
                torch.cuda.synchronize()
        atk.set_plan_override("")
        print(json.dumps({"probe": "done", "launches_each": 10, "plans": plans}))
        return

    if args.probe_small:
        st = torch.cuda.current_stream().cuda_stream
        cases = [(1, 1 << 20, 64), (1, 1 << 20, 256), (8, 1 << 20, 64), (8, 1 << 20, 256), (32, 1 << 17, 64), (32, 1 << 17, 256),
                 (64, 1 << 18, 512)]
        plans = {}
        for spec in ("MH=0", ""):  # the override only decides how the splits of a row meet
            atk.set_plan_override(spec)
            for (m_s, n_s, b) in cases:
                ring = [workloads.normal_rows(m_s, n_s, seed=s).to(dev) for s in range(4)]
                ov = torch.empty((m_s, K), dtype=torch.float32, device=dev)
                oi = torch.empty((m_s, K), dtype=torch.int32, device=dev)
                plans["%d x %d b=%d %s" % (m_s, n_s, b, spec or "default")] = atk.plan_describe(m_s, n_s, K, b, 1)
                for i in range(10):
                    rc = lib.approx_topk(ring[i % 4].data_ptr(), m_s, n_s, K, b, 1, atk.ATK_F32, ov.data_ptr(), oi.data_ptr(), st)
                    if rc != 0:
                        raise RuntimeError("approx_topk failed: %s" % atk.strerror(rc))
                torch.cuda.synchronize()
        atk.set_plan_override("")
        print(json.dumps({"probe": "done", "launches_each": 10, "plans": plans}))
        return

    if args.probe_long:
        n_long = 1 << 20
        xl = workloads.normal_rows(M, n_long, seed=0).to(dev)
        dst = torch.empty_like(xl)
        sink = torch.zeros(65536 // 8, dtype=torch.int64, device=dev)
        ov = torch.empty((M, K), dtype=torch.float32, device=dev)
        oi = torch.empty((M, K), dtype=torch.int32, device=dev)
        st = torch.cuda.current_stream().cuda_stream
        for i in range(5):
            lib.atk_copy(dst.data_ptr(), xl.data_ptr(), M * n_long * 4, st)
        for i in range(5):
            lib.atk_read_ceiling(xl.data_ptr(), M * n_long * 4, sink.data_ptr(), st)
        for b in (64, 1024):
            for i in range(20):
                rc = lib.approx_topk(xl.data_ptr(), M, n_long, K, b, 1, atk.ATK_F32, ov.data_ptr(), oi.data_ptr(), st)
                if rc != 0:
                    raise RuntimeError("approx_topk failed: %s" % atk.strerror(rc))
        torch.cuda.synchronize()
        print(json.dumps({"probe": "done", "copy_bytes": M * n_long * 4, "launches_each": 20, "b": [64, 1024]}))
        return

    # ---- inputs resident in HBM before anything is timed
    ring = [workloads.normal_rows(M, N, seed=s).to(dev) for s in range(RING)]
    out_v = torch.empty((M, K), dtype=torch.float32, device=dev)
    out_i = torch.empty((M, K), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    calls = 0

    def launch(x, b):
        rc = atk.approx_topk_raw(x.data_ptr(), M, N, K, b, 1, atk.ATK_F32, out_v.data_ptr(), out_i.data_ptr(), stream)
        if rc != 0:
            raise RuntimeError("approx_topk failed: %s" % atk.strerror(rc))

    def step(i, cold=True):
        for j, b in enumerate(SWEEP_B):
            launch(ring[(i * len(SWEEP_B) + j) % RING] if cold else ring[0], b)

    if args.probe:
        dst = torch.empty_like(ring[0])
        sink = torch.zeros(65536 // 8, dtype=torch.int64, device=dev)
        for i in range(20):
            lib.atk_copy(dst.data_ptr(), ring[i % RING].data_ptr(), M * N * 4, stream)
        for i in range(20):
            lib.atk_read_ceiling(ring[i % RING].data_ptr(), M * N * 4, sink.data_ptr(), stream)
        for b in SWEEP_B:
            for i in range(20):
                launch(ring[i % RING], b)
        torch.cuda.synchronize()
        print(json.dumps({"probe": "done", "copy_bytes": M * N * 4, "launches_each": 20, "b": SWEEP_B}))
        return

    if args.timeline:
        print(json.dumps(timeline(atk, lib, torch, dev, ring, out_v, out_i, stream)))
        return

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- the timed region: exactly `steps` steps
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = ev0.elapsed_time(ev1)
    ms_per_step = wall * 1e3 / args.steps
    step_bytes = len(SWEEP_B) * min_bytes(M, N, K)
    value = step_bytes / (wall / args.steps) / 1e9

    # ---- per-b timings (cold ring and warm single buffer), back-to-back launches between two events
    def time_case(b, cold, reps=300):
        for i in range(10):
            launch(ring[i % RING] if cold else ring[0], b)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            launch(ring[i % RING] if cold else ring[0], b)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps  # us per launch

    cases = {}
    for b in SWEEP_B:
        us_c, us_w = time_case(b, True), time_case(b, False)
        cases["b=%d" % b] = {
            "us_cold": round(us_c, 3), "GBps_cold": round(min_bytes(M, N, K) / us_c / 1e3, 1),
            "us_warm": round(us_w, 3), "GBps_warm": round(min_bytes(M, N, K) / us_w / 1e3, 1),
            "plan": atk.plan_describe(M, N, K, b, 1),
        }

    # ---- empirical ceiling: a read-only kernel over the same buffers
    sink = torch.zeros(65536 // 8, dtype=torch.int64, device=dev)  # ATK_CEILING_SINK_BYTES

    def ceiling(cold, reps=300):
        for i in range(10):
            lib.atk_read_ceiling(ring[i % RING].data_ptr(), M * N * 4, sink.data_ptr(), stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            lib.atk_read_ceiling((ring[i % RING] if cold else ring[0]).data_ptr(), M * N * 4, sink.data_ptr(), stream)
        e1.record()
        torch.cuda.synchronize()
        return M * N * 4 / (e0.elapsed_time(e1) * 1e-3 / reps) / 1e9

    ceil_cold, ceil_warm = ceiling(True), ceiling(False)

    # ---- roofline of the dominant kernel (the fused streaming kernel; HBM-bound):
    # algorithmic bytes per launch = m*n*4 read + m*k*8 written; average launch duration from HIP
    # events over the timed region (5 launches per step).
    launches = args.steps * len(SWEEP_B)
    avg_launch_s = ev_ms * 1e-3 / launches
    achieved = min_bytes(M, N, K) / avg_launch_s / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                "kernel": "lean_kernel<f32> (k_b = 1 streaming scan + fused Stage 2)", "avg_launch_us": round(avg_launch_s * 1e6, 3),
                "read_only_ceiling_GBps": {"cold": round(ceil_cold, 1), "warm": round(ceil_warm, 1)}}
    # HBM bytes per launch come from separate rocprofv3 --pmc passes (FETCH_SIZE, WRITE_SIZE scaled by a
    # copy kernel of known size); the summary of those passes records the figure.
    traffic_file = os.path.join(ROOT, "profiles", "lean_kernel_cfg2_hbm_traffic.md")
    if os.path.exists(traffic_file):
        import re

        with open(traffic_file) as f:
            hit = re.search(r"^\s*bytes_per_launch:\s*(\d+)", f.read(), flags=re.M)
        if hit:
            roofline["traffic"] = int(hit.group(1))

    # ---- CPU baseline: the oracle, untouched, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1))
        rows = 32
        xs = workloads.as_numpy_bits(workloads.normal_rows(M, N, seed=0)[:rows])
        oracle.approx_topk(xs[:2], K, 64, 1, threads=threads)  # load the library, warm the pages
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            for b in SWEEP_B:
                oracle.approx_topk(xs, K, b, 1, threads=threads)
            reps += 1
        dt = time.perf_counter() - t0
        t1 = time.perf_counter()
        for b in SWEEP_B:  # the same on one core, 4 rows
            oracle.approx_topk(xs[:4], K, b, 1, threads=1)
        dt1 = time.perf_counter() - t1
        cpu = {"value": round(reps * len(SWEEP_B) * min_bytes(rows, N, K) / dt / 1e9, 4), "unit": "GB/s",
               "cores": threads, "kind": "oracle",
               "sample": "%d of the %d rows, the same 5-value b sweep, %d repetitions in %.1f s" % (rows, M, reps, dt),
               "single_core_value": round(len(SWEEP_B) * min_bytes(4, N, K) / dt1 / 1e9, 4)}

    out = {
        "metric": "total bandwidth GB/s (min bytes / runtime), m=128 float32",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "cfg2: m=128 n=65536 f32 N(0,1) k=64 k_b=1, b in {64,128,256,512,1024}, "
                               "Stage 2 for b>64; one step = the 5 calls; inputs rotate over a 403 MB ring (HBM-cold)",
                   "m": M, "n": N, "k": K, "k_b": 1, "b": SWEEP_B},
        "frac_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "event_ms_per_step": round(ev_ms / args.steps, 5),
        "cases": cases,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    del ring
    torch.cuda.empty_cache()
    out["secondary"] = secondary(atk, workloads, torch, dev)
    if args.detail:
        out["detail"] = detail(atk, workloads, torch, dev)
    print(json.dumps(out))


PHASES = [(0, "start"), (1, "own share of the row read"), (2, "own lists merged / handed on"),
          (10, "last ticket drawn"), (11, "other workgroups' lists merged"), (3, "Stage 2 begins"),
          (4, "key range known"), (5, "histogram"), (6, "prefix sums"), (7, "winners filed"), (8, "outputs written"),
          (9, "end")]


def timeline(atk, lib, torch, dev, ring, out_v, out_i, stream, reps=30):
    """Microseconds after the first wavefront's start at which the first / median / last wavefront passed
    each phase boundary, averaged over `reps` traced launches per b (100 MHz device wall clock)."""
    import numpy as np

    res = {}
    for b in SWEEP_B:
        nbytes = lib.atk_trace_bytes(M, N, K, b, 1, atk.ATK_F32)
        assert nbytes > 0, nbytes
        tr = torch.zeros(nbytes // 8, dtype=torch.int64, device=dev)
        acc = {}
        for rep in range(reps):
            tr.zero_()
            rc = atk.approx_topk_raw(ring[(2 * rep) % RING].data_ptr(), M, N, K, b, 1, atk.ATK_F32, out_v.data_ptr(),
                                     out_i.data_ptr(), stream)
            assert rc == 0, atk.strerror(rc)
            rc = lib.atk_trace_approx(ring[(2 * rep + 1) % RING].data_ptr(), M, N, K, b, 1, atk.ATK_F32, out_v.data_ptr(),
                                      out_i.data_ptr(), tr.data_ptr(), nbytes, stream)
            assert rc == 0, atk.strerror(rc)
            torch.cuda.synchronize()
            t = tr.cpu().numpy().reshape(-1, 16).astype(np.int64)
            t = t[t[:, 0] != 0]  # wavefronts that ran
            t0 = t[:, 0].min()
            for ph, _ in PHASES:
                v = t[:, ph]
                v = v[v != 0]
                if v.size:
                    us = (v - t0) / 100.0
                    acc.setdefault(ph, []).append((float(us.min()), float(np.median(us)), float(us.max()), int(v.size)))
        rows = {}
        for ph, name in PHASES:
            if ph in acc:
                a = np.array(acc[ph])
                rows[name] = {"first_us": round(a[:, 0].mean(), 2), "median_us": round(a[:, 1].mean(), 2),
                              "last_us": round(a[:, 2].mean(), 2), "wavefronts": int(a[:, 3].mean())}
        res["b=%d" % b] = {"plan": atk.plan_describe(M, N, K, b, 1), "phases": rows}
    return {"timeline": res, "reps": reps, "clock": "100 MHz device wall clock, 10 ns steps",
            "workload": "cfg2: m=128 n=65536 f32 k=64 k_b=1, inputs from a 403 MB ring (HBM-cold)"}


def _time_us(torch, launch, reps, warm=5):
    """Average microseconds per launch of `reps` back-to-back launch(i) calls between two events."""
    for i in range(warm):
        launch(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        launch(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def _approx_entry(atk, torch, dev, ring, m, n, k, b, k_b, dt, es, reps, assignment=None):
    ov = torch.empty((m, k), dtype=ring[0].dtype, device=dev)
    oi = torch.empty((m, k), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    def launch(i):
        x = ring[i % len(ring)]
        if assignment is None:
            rc = atk.approx_topk_raw(x.data_ptr(), m, n, k, b, k_b, dt, ov.data_ptr(), oi.data_ptr(), stream)
        else:
            rc = atk.approx_topk_assign_raw(x.data_ptr(), m, n, k, b, k_b, dt, assignment, ov.data_ptr(), oi.data_ptr(),
                                            stream)
        assert rc == 0, atk.strerror(rc)

    us = _time_us(torch, launch, reps)
    nbytes = m * n * es + m * k * (es + 4)
    return {"us": round(us, 2), "est_us": round(atk.estimate_us(m, n, k, b, k_b, dt), 2) if assignment is None else None,
            "GBps": round(nbytes / us / 1e3, 1), "frac_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4),
            "plan": atk.plan_describe(m, n, k, b, k_b, dt, assignment if assignment is not None else atk.ATK_INTERLEAVED)}


def secondary(atk, workloads, torch, dev):
    """The other configurations, in every default run: microseconds per launch (inputs cold where a ring
    fits), total bandwidth and its fraction of the HBM peak.  Figure 1 right (k = n/4, k_b = 1 and 8), the long
    rows of 2^20 elements at k = 64 (one bucket per output, and 16 per output with Stage 2), the attention-score
    shape in bf16, and the row-length sweep at the headline setting (k = 64, k_b = 1, b = 64)."""
    res = {}

    def run(tag, ring, m, n, k, b, k_b, dt, es, reps):
        e = _approx_entry(atk, torch, dev, ring, m, n, k, b, k_b, dt, es, reps)
        res[tag] = {"us": e["us"], "GBps": e["GBps"], "frac_hbm_peak": e["frac_hbm_peak"], "plan": e["plan"]}

    ring = [workloads.normal_rows(M, N, seed=s).to(dev) for s in range(RING)]
    run("cfg3 k=16384 b=16384 k_b=1", ring, M, N, 16384, 16384, 1, atk.ATK_F32, 4, 200)
    run("cfg3 k=16384 b=2048 k_b=8", ring, M, N, 16384, 2048, 8, atk.ATK_F32, 4, 200)
    run("n=2^16 m=128 k=64 b=64 k_b=1", ring, M, N, 64, 64, 1, atk.ATK_F32, 4, 200)
    del ring
    torch.cuda.empty_cache()
    ring = [workloads.attention_scores(seed=s).to(dev) for s in range(RING)]
    run("cfg5 bf16 2048x8192 k=512 b=512 k_b=1", ring, 2048, 8192, 512, 512, 1, atk.ATK_BF16, 2, 200)
    del ring
    torch.cuda.empty_cache()
    for lg in (17, 18, 19, 20):
        n = 1 << lg
        nring = max(1, min(12, (420 << 20) // (M * n * 4)))
        ring = [workloads.normal_rows(M, n, seed=s).to(dev) for s in range(nring)]
        run("n=2^%d m=128 k=64 b=64 k_b=1" % lg, ring, M, n, 64, 64, 1, atk.ATK_F32, 4, 100)
        if lg == 20:  # = cfg4, k = 64
            res["cfg4 k=64 b=64 k_b=1"] = res["n=2^20 m=128 k=64 b=64 k_b=1"]
            run("cfg4 k=64 b=1024 k_b=1", ring, M, n, 64, 1024, 1, atk.ATK_F32, 4, 100)
        del ring
        torch.cuda.empty_cache()
    return res


def detail(atk, workloads, torch, dev):
    """Every configuration of the other sweeps: us per launch (cold where a ring fits), GB/s."""
    res = {}
    stream = torch.cuda.current_stream().cuda_stream
    for name in ["cfg3", "cfg4", "cfg5", "vocab", "kg"]:
        c = workloads.CONFIGS[name]
        m, n = c["m"], c["n"]
        es = 4 if c["dtype"] == "f32" else 2
        dt = atk.ATK_F32 if c["dtype"] == "f32" else atk.ATK_BF16
        nring = 1 if name in ("cfg4", "kg") else 10  # 537 MB / 679 MB inputs are cold by size
        if name == "vocab":
            nring = 20  # 16 MB each
        if name == "cfg5":
            ring = [workloads.attention_scores(seed=s).to(dev) for s in range(nring)]
        else:
            ring = [workloads.normal_rows(m, n, seed=s, dtype=c["dtype"]).to(dev) for s in range(nring)]
        reps = 50 if name in ("cfg4", "kg") else 200
        for (k, b, k_b) in c["cases"]:
            res["%s k=%d b=%d k_b=%d" % (name, k, b, k_b)] = _approx_entry(atk, torch, dev, ring, m, n, k, b, k_b, dt, es, reps)
        if name == "cfg4":
            # the exact comparison point on the same rows (Section 4.1 compares against exact top-k)
            for k in (64, 1 << 18):
                ov = torch.empty((m, k), dtype=ring[0].dtype, device=dev)
                oi = torch.empty((m, k), dtype=torch.int32, device=dev)

                def launch(i):
                    assert atk.exact_topk_raw(ring[0].data_ptr(), m, n, k, dt, ov.data_ptr(), oi.data_ptr(), stream) == 0

                us = _time_us(torch, launch, 10, warm=2)
                nbytes = m * n * es + m * k * (es + 4)
                res["cfg4 exact_topk k=%d" % k] = {"us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                                                   "frac_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4), "plan": "exact"}
        del ring
        torch.cuda.empty_cache()

    # ---- row length sweep at the headline setting (Figure 1 left: k=64, k_b=1, b*k_b/k = 1 and 16)
    for lg in (16, 17, 18, 19, 20):
        n = 1 << lg
        nring = max(1, min(12, (420 << 20) // (M * n * 4)))
        ring = [workloads.normal_rows(M, n, seed=s).to(dev) for s in range(nring)]
        for b in (64, 1024):
            res["n=2^%d m=128 k=64 b=%d k_b=1" % (lg, b)] = _approx_entry(atk, torch, dev, ring, M, n, 64, b, 1, atk.ATK_F32, 4, 100)
        del ring
        torch.cuda.empty_cache()

    # ---- small batches (Section 5 leaves the batch size open; SparQ decodes with m = 1)
    for m in (1, 8, 32):
        for n in (1 << 16, 1 << 20):
            nring = max(2, min(64, (420 << 20) // (m * n * 4)))
            ring = [workloads.normal_rows(m, n, seed=s).to(dev) for s in range(nring)]
            for (k, b, k_b) in [(64, 64, 1), (64, 1024, 1), (n // 8, n // 8, 1), (n // 8, n // 16, 2)]:
                res["m=%d n=%d k=%d b=%d k_b=%d" % (m, n, k, b, k_b)] = _approx_entry(
                    atk, torch, dev, ring, m, n, k, b, k_b, atk.ATK_F32, 4, 100)
            del ring
            torch.cuda.empty_cache()

    # ---- bf16 versions of the two 128 x 65536 sweeps (Appendix B.1, bfloat16 figure)
    ring = [workloads.normal_rows(M, N, seed=s, dtype="bf16").to(dev) for s in range(24)]
    for (k, b, k_b) in workloads.CONFIGS["cfg2"]["cases"] + workloads.CONFIGS["cfg3"]["cases"]:
        res["bf16 m=128 n=65536 k=%d b=%d k_b=%d" % (k, b, k_b)] = _approx_entry(
            atk, torch, dev, ring, M, N, k, b, k_b, atk.ATK_BF16, 2, 200)
    del ring
    torch.cuda.empty_cache()

    # ---- contiguous against interleaved buckets (Appendix A.1 reports a runtime edge for contiguous)
    ring = [workloads.normal_rows(M, N, seed=s).to(dev) for s in range(RING)]
    for (k, b, k_b) in [(64, 64, 1), (64, 1024, 1), (16384, 16384, 1), (16384, 4096, 4)]:
        res["contiguous m=128 n=65536 k=%d b=%d k_b=%d" % (k, b, k_b)] = _approx_entry(
            atk, torch, dev, ring, M, N, k, b, k_b, atk.ATK_F32, 4, 200, assignment=atk.ATK_CONTIGUOUS)

    # ---- the paper's timing protocol (Appendix B.1): per launch a sleep kernel, a start event, the call,
    # a stop event, all queued; 16 warm-up and 512 timed launches; median, minimum and standard error
    lib = atk.load_library()
    ov = torch.empty((M, K), dtype=torch.float32, device=dev)
    oi = torch.empty((M, K), dtype=torch.int32, device=dev)
    for b in SWEEP_B:
        def call(i):
            assert atk.approx_topk_raw(ring[i % RING].data_ptr(), M, N, K, b, 1, atk.ATK_F32, ov.data_ptr(), oi.data_ptr(),
                                       stream) == 0
        for i in range(16):
            call(i)
        torch.cuda.synchronize()
        times = []
        for chunk in range(8):  # 8 x 64 launches, each chunk queued behind its sleep kernels
            evs = []
            for i in range(64):
                lib.atk_sleep(20, stream)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                call(chunk * 64 + i)
                e1.record()
                evs.append((e0, e1))
            torch.cuda.synchronize()
            times += [a.elapsed_time(z) * 1e3 for a, z in evs]
        times.sort()
        mean = sum(times) / len(times)
        var = sum((t - mean) ** 2 for t in times) / (len(times) - 1)
        res["protocol b=%d" % b] = {"launches": len(times), "median_us": round(times[len(times) // 2], 2),
                                    "min_us": round(times[0], 2), "mean_us": round(mean, 2),
                                    "se_over_mean": round((var / len(times)) ** 0.5 / mean, 5)}

    # ---- the step replayed from a HIP graph (the paper's CUDA-graph variant): launch gaps removed
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        cs = side.cuda_stream
        for b in SWEEP_B:  # the scratch pool must have its size before capture starts
            assert atk.approx_topk_raw(ring[0].data_ptr(), M, N, K, b, 1, atk.ATK_F32, ov.data_ptr(), oi.data_ptr(), cs) == 0
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            for rep in range(2):
                for j, b in enumerate(SWEEP_B):
                    assert atk.approx_topk_raw(ring[(rep * 5 + j) % RING].data_ptr(), M, N, K, b, 1, atk.ATK_F32,
                                               ov.data_ptr(), oi.data_ptr(), side.cuda_stream) == 0
    ref = None
    for rep in range(3):  # every replay gives the last call's result again
        g.replay()
        torch.cuda.synchronize()
        cur = (ov.clone(), oi.clone())
        assert ref is None or (torch.equal(ref[0], cur[0]) and torch.equal(ref[1], cur[1]))
        ref = cur
    us = _time_us(torch, lambda i: g.replay(), 100)
    res["graph replay"] = {"launches_per_replay": 10, "us_per_launch": round(us / 10, 2),
                           "GBps": round(min_bytes(M, N, K) / (us / 10) / 1e3, 1)}
    return res


if __name__ == "__main__":
    main()
