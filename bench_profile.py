#!/usr/bin/env python3
"""Turns rocprofv3 output of bench.py runs into the short text summaries under profiles/.

Runs on the GPU machine after the rocprofv3 commands it prints with --commands (each of them
runs committed files only), e.g. for the default workload:

  python3 bench_profile.py --workload 5 --commands          # prints the four commands
  ... run them (cd /tmp && export TMPDIR=/tmp first; one rocprofv3 run per counter set) ...
  python3 bench_profile.py --workload 5 --dir rocprof_out   # writes profiles/<kernel>_<workload>[_<variant>].txt
                                                            # and ..._traffic.txt

The traffic file records the SHA-256 of the library sources it was measured on; bench.py
ignores it (roofline.traffic = null, with a warning) when the sources have changed since.
"""
import argparse
import collections
import csv
import hashlib
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
PROFILES = os.path.join(ROOT, "profiles")
LIB_SOURCES = ["paper_2304_05301_amd/csrc/tacos_kernels.hip", "paper_2304_05301_amd/csrc/tacos_api.cpp",
                "paper_2304_05301_amd/csrc/tacos_report.hip",
               "paper_2304_05301_amd/csrc/tacos_internal.h"]


def library_source_hash():
    h = hashlib.sha256()
    for rel in LIB_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def tag(workload, matching):
    return f"w{workload}" + (f"_m{matching}" if matching else "")


def commands(workload, matching, out_dir):
    b = f"python3 bench.py --workload {workload} --steps 1 --warmup 0 --no-cpu-baseline --no-kernel-timing --no-probes"
    if matching:
        b += f" --matching {matching}"
    t = tag(workload, matching)
    return {
        "stats": f"rocprofv3 --kernel-trace --stats --output-format csv -d {out_dir}/prof_{t}_stats -o bench -- {b}",
        "fetch": f"rocprofv3 --pmc FETCH_SIZE --output-format csv -d {out_dir}/prof_{t}_fetch -o bench -- {b} --calibrate-copy",
        "write": f"rocprofv3 --pmc WRITE_SIZE --output-format csv -d {out_dir}/prof_{t}_write -o bench -- {b} --calibrate-copy",
        "tcc": f"rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum --output-format csv -d {out_dir}/prof_{t}_tcc -o bench -- {b}",
    }


def find_csv(d, suffix):
    for base, _, files in os.walk(d):
        for f in files:
            if f.endswith(suffix):
                return os.path.join(base, f)
    raise FileNotFoundError(f"no *{suffix} under {d}")


def short(name):
    return name.replace("tacos::(anonymous namespace)::", "").split("(")[0]


def counters(d):
    """{counter: {kernel: [calls, sum, max]}} of one rocprofv3 --pmc run."""
    agg = collections.defaultdict(lambda: collections.defaultdict(lambda: [0, 0.0, 0.0]))
    with open(find_csv(d, "counter_collection.csv")) as f:
        for row in csv.DictReader(f):
            a = agg[row["Counter_Name"]][short(row["Kernel_Name"])]
            v = float(row["Counter_Value"])
            a[0] += 1
            a[1] += v
            a[2] = max(a[2], v)
    return agg


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=5)
    ap.add_argument("--matching", type=int, default=0)
    ap.add_argument("--dir", default="rocprof_out", help="where the rocprofv3 output folders are")
    ap.add_argument("--commands", action="store_true", help="print the rocprofv3 commands and exit")
    ap.add_argument("--out-dir", default=None,
                    help="where to write the summaries (default: profiles/; on a box from which only one "
                         "folder comes back, write there and copy the files into profiles/)")
    args = ap.parse_args()
    cmds = commands(args.workload, args.matching, args.dir)
    out_dir = args.out_dir or PROFILES
    os.makedirs(out_dir, exist_ok=True)
    if args.commands:
        for c in cmds.values():
            print(c)
        return
    sys.path.insert(0, ROOT)
    from paper_2304_05301_amd import topologies as T
    w = T.workload(args.workload)
    t = tag(args.workload, args.matching)
    variant = f"_matching{args.matching}" if args.matching else ""

    # ---- kernel trace: durations of the working launches and the gaps between kernels
    trace = []
    with open(find_csv(os.path.join(args.dir, f"prof_{t}_stats"), "kernel_trace.csv")) as f:
        for r in csv.DictReader(f):
            trace.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), short(r["Kernel_Name"])))
    trace.sort()
    names = collections.Counter(n for _, _, n in trace)
    kernel = "small_sweep_kernel" if any("small_sweep_kernel" in n for n in names) else "match_kernel"
    durs = [e - s for s, e, n in trace if kernel in n]
    # spans of the run: launches queued past a pass's end return at once (a few us)
    spans = None
    bench_json = os.path.join(args.dir, f"prof_{t}_stats.json")
    if os.path.exists(bench_json):
        with open(bench_json) as f:
            spans = json.loads(f.read().strip().splitlines()[-1])["ten_spans"]
    # tail_sweep_kernel: one workgroup sweeping the last stretch of a pass, many spans per launch
    tail = [e - s for s, e, n in trace if "tail_sweep_kernel" in n]
    # match_uniform_kernel: one launch per span, which a large pass on equal link costs goes over to
    # once few destinations are left (before the tail launches)
    late = [e - s for s, e, n in trace if "match_uniform_kernel" in n] if kernel == "match_kernel" else []
    if kernel == "match_kernel":
        if spans is None:
            spans = sum(1 for d in durs if d > 0.3 * max(durs))
        # (a pass that ends inside a tail launch queues no launch of the other kernels past its end)
        work = list(durs) if tail else sorted(durs, reverse=True)[:spans]
    else:
        work = durs
    # launches, a tail launch counted once per span it swept (as tacos_result_kernel_launches does)
    n_units = spans if tail else len(work)
    mean_us = (sum(work) + sum(late) + sum(tail)) / n_units / 1e3
    out = [f"rocprofv3 summary: {kernel} on workload {w.name}{' (matching = %d)' % args.matching if args.matching else ''} "
           f"({w.topo.n_npus} NPUs, {w.topo.n_links} links, {w.topo.n_npus * w.chunks_per_npu} chunks of {w.chunk_bytes} B, seed {w.seed})",
           "device: AMD Instinct MI355X (gfx950, 256 CUs), ROCm 7.2.0; automatic launch mode",
           f"library sources sha256 = {library_source_hash()}", "", "command (kernel stats):", "  " + cmds["stats"], "",
           "Name | Calls | TotalDurationNs | AverageNs | Percentage | MinNs | MaxNs"]
    with open(find_csv(os.path.join(args.dir, f"prof_{t}_stats"), "kernel_stats.csv")) as f:
        for row in csv.DictReader(f):
            n = short(row["Name"])[:90]
            out.append(f"{n} | {row['Calls']} | {row['TotalDurationNs']} | {float(row['AverageNs']):.1f} | "
                       f"{row['Percentage']} | {row['MinNs']} | {row['MaxNs']}")
    out.append("")
    if tail:
        n_tail = spans - len(work) - len(late)
        out.append(f"{kernel}: {len(durs)} launches, all of them did work ({sum(work) / 1e6:.1f} ms); match_uniform_kernel "
                   f"(one launch per span once at most 2,048 destinations are left): {len(late)} launches "
                   f"({sum(late) / 1e6:.1f} ms, {sum(late) / max(1, len(late)) / 1e3:.2f} us each); tail_sweep_kernel: "
                   f"{len(tail)} launches sweeping the other {n_tail} spans ({sum(tail) / 1e6:.1f} ms, "
                   f"{sum(tail) / max(1, n_tail) / 1e3:.2f} us per span); per span over all {spans}: mean "
                   f"{mean_us:.2f} us; {kernel} alone: mean {sum(work) / len(work) / 1e3:.2f} us, "
                   f"median {sorted(work)[len(work) // 2] / 1e3:.2f} us")
    else:
        out.append(f"{kernel}: {len(durs)} launches, {len(work)} of them did work; working launches: mean {mean_us:.2f} us, "
                   f"median {sorted(work)[len(work) // 2] / 1e3:.2f} us")
    if kernel == "match_kernel":
        # per span: arrive -> (gap) -> match -> (gap) -> next arrive, over the working spans
        thr = sorted(durs, reverse=True)[len(work) - 1]
        g_am, g_ma, arr = [], [], []
        for i in range(1, len(trace) - 1):
            s, e, n = trace[i]
            if kernel in n and e - s >= thr and trace[i - 1][2].startswith("arrive_") and trace[i + 1][2].startswith("arrive_"):
                g_am.append(s - trace[i - 1][1])
                g_ma.append(trace[i + 1][0] - e)
                arr.append(trace[i - 1][1] - trace[i - 1][0])
        if arr:
            a, g1, g2 = (sum(x) / len(x) / 1e3 for x in (arr, g_am, g_ma))
            m_us = sum(work) / len(work) / 1e3
            span = m_us + a + g1 + g2
            out.append(f"per span with two launches ({len(arr)} spans): arrivals kernel {a:.2f} us + gap {g1:.2f} us + {kernel} "
                       f"{m_us:.2f} us + gap {g2:.2f} us = {span:.2f} us; outside {kernel}: {100 * (span - m_us) / span:.1f} %")
    n_chunks = w.topo.n_npus * w.chunks_per_npu
    wb = 8 * ((n_chunks + 63) // 64)
    out.append("")

    # ---- counters
    have = all(os.path.isdir(os.path.join(args.dir, f"prof_{t}_{k}")) for k in ("fetch", "write"))
    if have and kernel == "match_kernel":
        fe, wr = counters(os.path.join(args.dir, f"prof_{t}_fetch")), counters(os.path.join(args.dir, f"prof_{t}_write"))
        cp_f = fe["FETCH_SIZE"]["__amd_rocclr_copyBuffer"][2]
        cp_w = wr["WRITE_SIZE"]["__amd_rocclr_copyBuffer"][2]
        fs, ws = 1048576 / cp_f, 1048576 / cp_w
        mk = [k for k in fe["FETCH_SIZE"] if kernel in k][0]
        # counted with the launches they replace
        tk = [k for k in fe["FETCH_SIZE"] if "tail_sweep_kernel" in k or "match_uniform_kernel" in k]
        total = lambda table: table[mk][1] + sum(table[k][1] for k in tk)
        fb = total(fe["FETCH_SIZE"]) * fs * 1024 / n_units
        wbytes = total(wr["WRITE_SIZE"]) * ws * 1024 / n_units
        out += ["commands (counters, one run each; --calibrate-copy adds one plain 1 GiB device copy as reference dispatch):",
                "  " + cmds["fetch"], "  " + cmds["write"], "  " + cmds["tcc"],
                f"reference: plain device copy of 1 GiB: FETCH_SIZE reads {cp_f:.1f} (KiB units) -> scale {fs:.4f}; "
                f"WRITE_SIZE reads {cp_w:.1f} -> scale {ws:.4f}",
                f"{kernel}: per working launch read {fb / 1e6:.1f} MB, written {wbytes / 1e6:.1f} MB beyond L2 -> "
                f"{(fb + wbytes) / 1e6:.1f} MB per launch ({(fb + wbytes) / mean_us / 1e6:.2f} TB/s)"]
        vals = {"workload": w.name, "matching": args.matching, "hbm_bytes_per_launch": f"{fb + wbytes:.0f}",
                "mean_launch_us_rocprof": f"{mean_us:.2f}", "library_sources_sha256": library_source_hash()}
        tcc_dir = os.path.join(args.dir, f"prof_{t}_tcc")
        if os.path.isdir(tcc_dir):
            tc = counters(tcc_dir)
            hit, miss, req = (total(tc[c]) for c in ("TCC_HIT_sum", "TCC_MISS_sum", "TCC_REQ_sum"))
            out.append(f"  L2 (TCC) per working launch: {req / n_units / 1e6:.2f} M requests of 128 B = "
                       f"{req / n_units * 128 / 1e6:.1f} MB asked of L2, hit rate {100 * hit / (hit + miss):.1f} %")
            vals["l2_request_bytes_per_launch"] = f"{req / n_units * 128:.0f}"
            vals["l2_hit_rate"] = f"{hit / (hit + miss):.4f}"
        with open(os.path.join(out_dir, f"{kernel}_{w.name}{variant}_traffic.txt"), "w") as f:
            f.write(f"# per working launch of {kernel}: bytes beyond L2 (FETCH_SIZE + WRITE_SIZE, each scaled by a plain 1 GiB copy)\n"
                    f"# and bytes asked of L2 (TCC_REQ_sum x 128 B); written by bench_profile.py, see {kernel}_{w.name}{variant}.txt\n")
            for k, v in vals.items():
                f.write(f"{k} = {v}\n")
    path = os.path.join(out_dir, f"{kernel}_{w.name}{variant}.txt")
    with open(path, "w") as f:
        f.write("\n".join(out) + "\n")
    print("\n".join(out))
    print("wrote", path, file=sys.stderr)


if __name__ == "__main__":
    main()
