#!/usr/bin/env python3
"""Benchmark of the TACOS synthesis hot path on one MI355X.

One "step" = one complete synthesis (link costs, precondition init, every TEN span:
arrivals + matching + next-event reduction, schedule statistics) of the workload through
the C ABI.  Default workload: All-Gather on the 32x32x40 3D torus (40,960 NPUs, 245,760
links, 1 chunk of 1 MiB per NPU, seed 4).  Prints ONE JSON line.

  value      = link-chunk matches per second of the whole synthesis call (wall clock,
               inputs are a few MB of topology arrays uploaded inside the call)
  roofline   = matching kernel: algorithmic (cache-blind) bytes per launch / mean launch
               duration (HIP events on the launch stream, one extra instrumented step after
               the timed ones) against the 8 TB/s HBM peak; roofline.l2 = the bytes the
               wavefronts ask L2 for / the same duration against the rate a no-arithmetic
               probe of the same request pattern reaches on this device, measured now
               (the ceiling that binds: a fraction <= 1)
  cpu_baseline = the CPU oracle timed on this machine's host cores on a bounded prefix of
               the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PROFILES = os.path.join(ROOT, "profiles")


def algorithmic_bytes(n_matches, n_npus, n_links, n_chunks):
    """Bytes the word-wise candidate computation must move per match: one held[src] row
    per matched link plus held[dst] and inflight[dst] once per destination and span,
    i.e. Wb * (1 + 2 / mean in-degree) with Wb = 8 * ceil(C / 64)."""
    wb = 8 * ((n_chunks + 63) // 64)
    deg = n_links / n_npus
    return n_matches * wb * (1.0 + 2.0 / deg)


def library_source_hash():
    import hashlib
    h = hashlib.sha256()
    for rel in ("paper_2304_05301_amd/csrc/tacos_kernels.hip", "paper_2304_05301_amd/csrc/tacos_api.cpp",
                "paper_2304_05301_amd/csrc/tacos_report.hip",
                "paper_2304_05301_amd/csrc/tacos_internal.h"):
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(kernel, workload_name, matching):
    """Counter summary of the matching kernel written by bench_profile.py from rocprofv3 --pmc
    runs: bytes beyond L2 per launch (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy of known
    size) and bytes asked of L2 (TCC_REQ_sum x 128 B).  Returns {} when there is none, or
    when it was measured on other library sources than the ones in the tree (stale)."""
    variant = f"_matching{matching}" if matching else ""
    path = os.path.join(PROFILES, f"{kernel}_{workload_name}{variant}_traffic.txt")
    if not os.path.exists(path):
        return {}
    vals = {}
    with open(path) as f:
        for line in f:
            if "=" in line and not line.startswith("#"):
                k, v = line.split("=", 1)
                vals[k.strip()] = v.strip()
    if vals.get("workload") != workload_name:
        return {}
    if vals.get("library_sources_sha256") != library_source_hash():
        print(f"bench.py: {os.path.relpath(path, ROOT)} was measured on other library sources: "
              "roofline.traffic = null (run bench_profile.py again)", file=sys.stderr)
        return {}
    return vals


class Probes:
    """ctypes access to libbench_probe.so (bench_probe.hip): no-arithmetic memory probes."""

    def __init__(self):
        import ctypes
        path = os.path.join(ROOT, "libbench_probe.so")
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: python -c 'import __graft_entry__ as g; g.build()'")
        L = ctypes.CDLL(path)
        d = ctypes.POINTER(ctypes.c_double)
        L.probe_row_stream.restype = ctypes.c_int
        L.probe_row_stream.argtypes = [ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32,
                                       ctypes.c_uint32, d, d]
        for f in (L.probe_read_stream, L.probe_copy):
            f.restype = ctypes.c_int
            f.argtypes = [ctypes.c_uint64, ctypes.c_uint32, d]
        self.L = L
        self.ctypes = ctypes

    def row_stream(self, topo, row_bytes, iters=200):
        import numpy as np
        c = self.ctypes
        rp = np.ascontiguousarray(topo.row_ptr, dtype=np.uint32)
        ci = np.ascontiguousarray(topo.col_idx, dtype=np.uint32)
        us, req = c.c_double(0), c.c_double(0)
        rc = self.L.probe_row_stream(topo.n_npus, rp.ctypes.data, ci.ctypes.data, int(row_bytes), iters,
                                     c.byref(us), c.byref(req))
        if rc != 0:
            raise RuntimeError(f"probe_row_stream: hipError {rc}")
        return us.value, req.value

    def read_stream(self, nbytes=2 << 30, iters=10):
        v = self.ctypes.c_double(0)
        rc = self.L.probe_read_stream(nbytes, iters, self.ctypes.byref(v))
        if rc != 0:
            raise RuntimeError(f"probe_read_stream: hipError {rc}")
        return v.value

    def copy(self, nbytes=1 << 30, iters=10):
        v = self.ctypes.c_double(0)
        rc = self.L.probe_copy(nbytes, iters, self.ctypes.byref(v))
        if rc != 0:
            raise RuntimeError(f"probe_copy: hipError {rc}")
        return v.value


def cpu_baseline(w, target_s=15.0):
    """The CPU oracle on a bounded sample of the workload: the whole workload if that takes
    about target_s or less, else the first spans of its All-Gather pass (the reversed pass
    of a Reduce-Scatter does the same work per span on the transposed topology)."""
    import oracle
    threads = min(oracle.max_threads(), 16)
    t = w.topo

    def run(coll, n_events):
        t0 = time.perf_counter()
        r = oracle.synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B,
                              w.chunks_per_npu, w.chunk_bytes, coll, w.seed,
                              max_events=n_events, keep_xfers=0, n_threads=threads)
        return time.perf_counter() - t0, r

    dt2, _ = run(0, 2)
    dt6, r6 = run(0, 6)
    per_event = max((dt6 - dt2) / 4, 1e-7)   # set-up time cancels
    n = int(max(6, target_s / per_event))
    oracle.set_progress(max(1, int(20.0 / per_event)))  # a line about every 20 s
    try:
        small = t.n_npus * w.chunks_per_npu <= 2048
        if small and w.collective != 0:
            t0 = time.perf_counter()
            r = oracle.synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B,
                                  w.chunks_per_npu, w.chunk_bytes, w.collective, w.seed,
                                  keep_xfers=0, n_threads=threads)
            dt = time.perf_counter() - t0
            sample = f"whole workload ({r.n_xfers} matches)"
            complete = True
        else:
            dt, r = run(0, n)
            complete = r.n_events < n and w.collective == 0
            what = "whole workload" if complete else f"first {r.n_events} TEN spans of the All-Gather pass"
            sample = f"{what} ({r.n_xfers} matches)"
    finally:
        oracle.set_progress(0)
    return {"value": r.n_xfers / dt, "unit": "matches/s", "cores": threads, "kind": "oracle",
            "sample": sample, "seconds": dt, "complete": complete}


def report_all(binding, T, stream, with_cpu):
    """One timed synthesis of every workload (after a warm-up run, except workload 4), one more
    with the matching kernel's launches bracketed by events, and the oracle beside it; prints
    a markdown table."""
    rows = []
    for idx in (1, 2, 3, 4, 5, 6, 7):
        w = T.workload(idx)
        topo = w.topo
        n_chunks = topo.n_npus * w.chunks_per_npu
        if idx != 4:
            binding.synthesize_workload(w, stream=stream).free()
        t0 = time.perf_counter()
        r0 = binding.synthesize_workload(w, stream=stream)
        wall = time.perf_counter() - t0   # uninstrumented; the kernel times come from one more run
        r0.free()
        r = binding.synthesize_workload(w, stream=stream, time_kernels=True)
        alg = algorithmic_bytes(r.num_xfers, topo.n_npus, topo.n_links, n_chunks)
        k_s = r.kernel_ms * 1e-3
        # the paper's Ideal, bandwidth term only (collective size over the bandwidth of the worst-
        # connected NPU; the latency diameter is left out): efficiency = Ideal / collective time
        ideal = binding.tacos_ideal_bound(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B,
                                          w.chunks_per_npu, w.chunk_bytes, w.collective,
                                          with_diameter=False)["bandwidth_term_ps"]
        row = {"idx": idx, "name": w.name, "npus": topo.n_npus, "links": topo.n_links, "spans": r.num_events,
               "eff": ideal / r.collective_time_ps,
               "matches": r.num_xfers, "T_ps": r.collective_time_ps, "wall_s": wall, "kernel_s": k_s,
               "matches_per_s": r.num_xfers / wall, "alg_GBps": alg / k_s / 1e9 if k_s > 0 else 0.0}
        r.free()
        if with_cpu:
            cb = cpu_baseline(w, target_s=10.0)
            row["cpu"] = cb
        rows.append(row)
        print(f"[report] workload {idx} done", file=sys.stderr, flush=True)
    print("| # | workload | NPUs | links | TEN spans | matches | collective time (ps) | Ideal (bandwidth term) / time | GPU synthesis (s) | "
          "matches/s | matching kernel (s) | algorithmic GB/s in the matching kernel | fraction of 8 TB/s | "
          "oracle matches/s (host threads; sample) |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    for r in rows:
        cpu = "-"
        if "cpu" in r:
            c = r["cpu"]
            cpu = f"{c['value']:.3g} ({c['cores']}; {c['sample']}, {c['seconds']:.1f} s)"
        print(f"| {r['idx']} | {r['name']} | {r['npus']} | {r['links']} | {r['spans']} | {r['matches']} | {r['T_ps']} | "
              f"{r['eff']:.4f} | {r['wall_s']:.4f} | {r['matches_per_s']:.3g} | {r['kernel_s']:.4f} | {r['alg_GBps']:.1f} | "
              f"{r['alg_GBps'] / HBM_PEAK_GBS:.4f} | {cpu} |")


def report_seed_search(binding, T, stream):
    """Best-of-K seeds on the workloads that fit the single-workgroup kernel: K single
    syntheses' worth of spans in about the time of one."""
    import numpy as np
    print()
    print("| workload | matching | seeds | search (s) | spans swept | spans/s | one synthesis (s) | best T (ps) | "
          "median T (ps) | worst T (ps) |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for idx, k, matching in ((2, 1024, 0), (3, 1024, 0), (3, 1024, 1), (4, 256, 0)):
        w = T.workload(idx)
        seeds = np.arange(k, dtype=np.uint64)
        binding.seed_search_workload(w, seeds[:2], stream=stream, matching=matching)
        t0 = time.perf_counter()
        times, events, best = binding.seed_search_workload(w, seeds, stream=stream, matching=matching)
        dt = time.perf_counter() - t0
        t0 = time.perf_counter()
        binding.tacos_seed_search(w.topo.n_npus, w.topo.row_ptr, w.topo.col_idx, w.topo.alpha_ps,
                                  w.topo.beta_fs_per_B, w.chunks_per_npu, w.chunk_bytes, w.collective,
                                  seeds[best:best + 1], stream=stream, matching=matching)
        one = time.perf_counter() - t0
        print(f"| {w.name} | {matching} | {k} | {dt:.3f} | {int(events.sum())} | {events.sum() / dt:.3g} | {one:.3f} | "
              f"{int(times.min())} | {int(np.median(times))} | {int(times.max())} |")
        print(f"[report] seed search on workload {idx} done", file=sys.stderr, flush=True)


def report_modes(binding, T, stream):
    """The launch forms against each other on shapes between the benchmark workloads: what the
    automatic choice (launch_mode 0) picks and what the other forms would have cost.  Wall-clock
    of one tacos_synthesize call (best of two), All-Gather unless named, 1 MiB chunks, seed 3."""
    MiB = 1 << 20
    h3 = ([300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000])
    h2 = ([300_000, 700_000], [5_000, 20_000])
    ag = T.ALL_GATHER
    cases = [
        ("mesh8x8, 4 chunks per NPU", T.mesh2d(8, 8), 4, ag, {}),
        ("mesh8x8, 32 chunks per NPU", T.mesh2d(8, 8), 32, ag, {}),
        ("mesh16x16", T.mesh2d(16, 16), 1, ag, {}),
        ("mesh16x16, 8 chunks per NPU", T.mesh2d(16, 16), 8, ag, {}),
        ("mesh16x16, 8 chunks per NPU, matching 1", T.mesh2d(16, 16), 8, ag, dict(matching=1)),
        ("heterogeneous mesh16x16, 8 chunks per NPU", T.grid([16, 16], False, *h2), 8, ag, {}),
        ("heterogeneous torus4x4x8, 4 chunks per NPU, All-Reduce", T.workload(3).topo, 4, T.ALL_REDUCE, {}),
        ("heterogeneous torus4x4x8, 16 chunks per NPU", T.workload(3).topo, 16, ag, {}),
        ("torus8x8x8", T.torus3d(8, 8, 8), 1, ag, {}),
        ("torus8x8x8, 3 chunks per NPU", T.torus3d(8, 8, 8), 3, ag, {}),
        ("heterogeneous torus8x8x8", T.grid([8, 8, 8], True, *h3), 1, ag, {}),
        ("unwound switch, 256 ports, degree 4, 4 chunks per NPU", T.switch_unwound(256, 4), 4, ag, {}),
        ("random 256 NPUs, out-degree 4, every link its own cost, 4 chunks per NPU",
         T.random_regular_out(256, 4, seed=3)[0], 4, ag, {}),
        ("torus16x16x16", T.torus3d(16, 16, 16), 1, ag, {}),
        ("torus64x64", T.grid([64, 64], True), 1, ag, {}),
        ("mesh64x64", T.mesh2d(64, 64), 1, ag, {}),
        ("torus32x32x16", T.torus3d(32, 32, 16), 1, ag, {}),
        ("mesh128x128", T.mesh2d(128, 128), 1, ag, {}),
        ("torus32x32x32", T.torus3d(32, 32, 32), 1, ag, {}),
    ]
    print("| topology | NPUs | links | chunks | TEN spans | matches per span | automatic (ms) | one workgroup, mode 2 (ms) | "
          "one launch per span, mode 3 (ms) | two launches per span, mode 4 (ms) |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for name, t, cpn, coll, kw in cases:
        cells, ev, nx = [], 0, 0
        binding.tacos_synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B, cpn, MiB, coll, 3,
                                 stream=stream, **kw).free()  # warm-up
        for mode in (0, 2, 3, 4):
            best = None
            try:
                for _ in range(2):
                    t0 = time.perf_counter()
                    r = binding.tacos_synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B, cpn, MiB,
                                                 coll, 3, stream=stream, launch_mode=mode, **kw)
                    dt = time.perf_counter() - t0
                    ev, nx = r.num_events, r.num_xfers
                    r.free()
                    best = dt if best is None else min(best, dt)
                cells.append(f"{best * 1e3:.2f}")
            except binding.TacosError:
                cells.append("does not apply")
        print(f"| {name} | {t.n_npus} | {t.n_links} | {t.n_npus * cpn} | {ev} | {nx // max(1, ev)} | " + " | ".join(cells) + " |")
        print(f"[report] {name} done", file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", type=int, default=5, help="1..7 (default 5: 40,960-NPU torus)")
    ap.add_argument("--matching", type=int, default=0, help="0 link-centric (default), 1 Algorithm 1's own order")
    ap.add_argument("--link-order", type=int, default=0, help="0 ascending link id (default), 1 cheapest link first")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="skip the extra instrumented step (profile runs: rocprofv3 times the kernels)")
    ap.add_argument("--no-probes", action="store_true", help="skip the memory probes (profile runs)")
    ap.add_argument("--report-all", action="store_true",
                    help="instead of the one JSON line: a table over workloads 1..7 (GPU time, spans, "
                         "matches/s, fraction of the HBM roofline, oracle time on the host cores)")
    ap.add_argument("--report-modes", action="store_true",
                    help="instead of the one JSON line: the launch forms against each other on shapes between "
                         "the benchmark workloads")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2304_05301_amd import binding, topologies as T

    if not torch.cuda.is_available():
        print("bench.py: no HIP device", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream
    if args.report_modes:
        report_modes(binding, T, stream)
        return
    if args.report_all:
        report_all(binding, T, stream, not args.no_cpu_baseline)
        report_seed_search(binding, T, stream)
        return
    w = T.workload(args.workload)
    topo = w.topo
    n_chunks = topo.n_npus * w.chunks_per_npu

    def step(timed):
        r = binding.synthesize_workload(w, stream=stream, time_kernels=timed, matching=args.matching,
                                        link_order=args.link_order)
        out = (r.num_xfers, r.num_events, r.collective_time_ps, r.kernel_ms, r.kernel_launches,
               r.digest, r.wall_ms)
        r.free()
        return out

    if args.calibrate_copy:
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        a.fill_(1)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    # the timed steps run without any instrumentation
    t0 = time.perf_counter()
    results = [step(False) for _ in range(args.steps)]
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    n_xfers, n_events, T_ps, _, _, digest, _ = results[0]
    assert all(r[0] == n_xfers and r[5] == digest for r in results), "non-deterministic result"
    ms_per_step = 1e3 * elapsed / args.steps

    # one extra step with HIP events around every launch of the matching kernel
    kernel_ms, launches, instrumented_wall_ms = None, None, None
    if not args.no_kernel_timing:
        k = step(True)
        assert k[0] == n_xfers and k[5] == digest, "non-deterministic result"
        kernel_ms, launches, instrumented_wall_ms = k[3], max(1, k[4]), k[6]
    alg_bytes = algorithmic_bytes(n_xfers, topo.n_npus, topo.n_links, n_chunks)
    roofline = {"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
                "traffic": None, "kernel": None,
                "note": "achieved = algorithmic (cache-blind) bytes per launch / launch duration: every source row "
                        "counted once per matched link although about 70 % of the requests hit in L2, so it may "
                        "exceed the HBM peak; the ceilings that bind are in l2 and hbm_side"}
    if kernel_ms:
        mean_launch_s = kernel_ms * 1e-3 / launches
        achieved = alg_bytes / launches / mean_launch_s / 1e9
        # small topologies run in the single-workgroup kernel: a few launches, each many spans
        kernel = "small_sweep_kernel" if launches < n_events else "match_kernel"
        tr = measured_traffic(kernel, w.name, args.matching)
        traffic = float(tr["hbm_bytes_per_launch"]) if tr else None
        roofline.update({"achieved": achieved, "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "kernel": kernel,
                         "algorithmic_bytes_per_launch": alg_bytes / launches, "mean_launch_us": mean_launch_s * 1e6})
        probes = None
        if not args.no_probes:
            try:
                probes = Probes()
            except ImportError as e:
                print(f"bench.py: {e}", file=sys.stderr)
        if probes and kernel == "match_kernel" and n_chunks <= 65536:
            row_bytes = 1024 * ((n_chunks + 8191) // 8192)
            probe_us, probe_req = probes.row_stream(topo, row_bytes)
            read_peak, copy_rate = probes.read_stream(), probes.copy()
            # bytes the wavefronts ask L2 for per launch: counted (TCC_REQ_sum x 128 B, committed
            # summary of the same sources) or else the rows the kernel must request when every
            # incoming link is idle: (1 + in-degree) rows per destination
            if tr and "l2_request_bytes_per_launch" in tr:
                l2_req, l2_src = float(tr["l2_request_bytes_per_launch"]), "rocprofv3 TCC_REQ_sum x 128 B"
            else:
                l2_req, l2_src = probe_req, "(NPUs + links) x row bytes"
            ceiling = probe_req / (probe_us * 1e-6) / 1e9
            l2_rate = l2_req / mean_launch_s / 1e9
            roofline["l2"] = {"bound": "l2", "request_bytes_per_launch": l2_req, "request_bytes_source": l2_src,
                              "achieved": l2_rate, "ceiling": ceiling, "unit": "GB/s", "frac": l2_rate / ceiling,
                              "ceiling_source": "bench_probe.hip probe_row_stream: the same rows in the same order, "
                                                "no arithmetic, measured in this run",
                              "probe_launch_us": probe_us, "probe_request_bytes_per_launch": probe_req}
            roofline["hbm_side"] = {"measured_read_stream_GBps": read_peak, "measured_copy_GBps": copy_rate,
                                    "traffic_GBps": traffic / mean_launch_s / 1e9 if traffic else None,
                                    "frac_of_peak": traffic / mean_launch_s / 1e9 / HBM_PEAK_GBS if traffic else None,
                                    "frac_of_measured_read_stream": traffic / mean_launch_s / 1e9 / read_peak
                                    if traffic else None}

    line = {
        "metric": "ten_link_chunk_matches_per_sec",
        "value": n_xfers / (ms_per_step * 1e-3),
        "unit": "matches/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64",
        "data": "synthetic",
        "config": {"workload": w.name, "topology": topo.name, "n_npus": topo.n_npus,
                   "n_links": topo.n_links, "chunks": n_chunks, "chunk_bytes": w.chunk_bytes,
                   "collective": ["all_gather", "reduce_scatter", "all_reduce"][w.collective],
                   "seed": w.seed, "matching": args.matching, "link_order": args.link_order},
        "synthesis_wall_s": ms_per_step * 1e-3,
        "synthesis_wall_s_median": sorted(r[6] for r in results)[len(results) // 2] * 1e-3,
        "matches": n_xfers,
        "ten_spans": n_events,
        "collective_time_ps": T_ps,
        "schedule_digest": digest,
        "match_kernel_ms_per_step": kernel_ms,
        "match_kernel_launches": launches,
        "match_kernel_matches_per_s": n_xfers / (kernel_ms * 1e-3) if kernel_ms else None,
        "instrumented_step_wall_ms": instrumented_wall_ms,
        "roofline": roofline,
        "paper_context": "paper reports wall-clock only: 128-NPU All-Reduce synthesized in 1.08 s, "
                         "40K-NPU 2D mesh All-Reduce in 2.52 h (Xeon E5-2699v3, 64 threads)",
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
