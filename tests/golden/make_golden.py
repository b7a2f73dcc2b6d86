"""Writes tests/golden/workloads_oracle.json from the CPU oracle ONLY.

Run:  python tests/golden/make_golden.py
It calls nothing but the input generators and oracle/; the HIP path is never involved.
Stored per workload 1..4: collective time, matching sweeps, records, the schedule
digest and the SHA-256 of the canonical record array (little-endian structs of
t_ps:u64, src:u32, dst:u32, chunk:u32, link:u32).  Workload 4 takes about a minute.

    python tests/golden/make_golden.py --with-5 [--threads 8]

additionally runs the 40,960-NPU workload 5 to completion (OpenMP over destinations;
minutes) and stores its time, sweeps, records, digest and the SHA-256 of the per-sweep
(time, match count) trace in workload5_oracle.json.  Of its 1.68e9 records the first 4096 and
16 windows of 65,536 spread over the whole schedule (the last one ends it) are hashed.

    python tests/golden/make_golden.py --with-5 --matching1 [--threads 8]

the same workload with the postcondition-centric matching order (workload5_matching1_oracle.json).

    python tests/golden/make_golden.py --scalability 6 [--threads 8]      (or 7)

runs the paper's scalability workload (6: All-Reduce on the 200x200 mesh, 7: on the
35x35x35 3-D mesh) to completion, digest only (tens of minutes on 8 threads), and stores
collective time, per-pass times and sweeps, records and digest in workload<N>_oracle.json.

    python tests/golden/make_golden.py --seed-search

runs workload 4's topology with three other seeds, one after the other (a minute), and
stores their collective times and sweep counts in seed_search_oracle.json.
"""
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_2304_05301_amd import topologies as T  # noqa: E402


W5_XFERS = 40_960 * 40_959          # records of the 40,960-NPU All-Gather
W5_BLOCK = 65_536                   # records per sampled window
W5_STRIDE = 104_857_600             # distance between windows: 16 of them, the last one ends the schedule


def workload5_matching1(threads):
    """Workload 5 with Algorithm 1's own (postcondition-centric) order: digest, trace and the
    first 4096 records."""
    w = T.workload(5)
    oracle.set_progress(500)
    r = oracle.synthesize_workload(w, keep_first=0, keep_xfers=4096, n_threads=threads, matching=1)
    out = {
        "name": w.name, "topology": w.topo.name, "matching": 1,
        "collective_time_ps": r.collective_time_ps, "n_events": r.n_events, "n_xfers": r.n_xfers, "digest": r.digest,
        "sha256_event_trace": hashlib.sha256(r.event_times.tobytes() + r.event_matches.tobytes()).hexdigest(),
        "sha256_first_4096_xfers": hashlib.sha256(r.xfers.tobytes()).hexdigest(),
    }
    print("5 matching 1", out, flush=True)
    with open(os.path.join(HERE, "workload5_matching1_oracle.json"), "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
        f.write("\n")


def workload5(threads):
    w = T.workload(5)
    oracle.set_progress(500)
    first = (W5_XFERS - W5_BLOCK) % W5_STRIDE
    # one run keeps the first 4096 records; a second one the windows spread over the schedule
    r = oracle.synthesize_workload(w, keep_first=0, keep_xfers=4096, n_threads=threads)
    oracle.set_keep_windows(W5_STRIDE, W5_BLOCK)
    try:
        rw = oracle.synthesize_workload(w, keep_first=first, n_threads=threads)
    finally:
        oracle.set_keep_windows(0, 0)
    assert rw.digest == r.digest and rw.n_xfers == r.n_xfers == W5_XFERS and len(rw.xfers) % W5_BLOCK == 0
    windows = [hashlib.sha256(rw.xfers[i:i + W5_BLOCK].tobytes()).hexdigest() for i in range(0, len(rw.xfers), W5_BLOCK)]
    trace = hashlib.sha256(r.event_times.tobytes() + r.event_matches.tobytes()).hexdigest()
    out = {
        "windows": {"first": first, "stride": W5_STRIDE, "block": W5_BLOCK, "sha256": windows},
        "name": w.name,
        "topology": w.topo.name,
        "collective_time_ps": r.collective_time_ps,
        "n_events": r.n_events,
        "n_xfers": r.n_xfers,
        "digest": r.digest,
        "sha256_event_trace": trace,
        "sha256_first_4096_xfers": hashlib.sha256(r.xfers.tobytes()).hexdigest(),
    }
    print(5, out, flush=True)
    with open(os.path.join(HERE, "workload5_oracle.json"), "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
        f.write("\n")


SEARCH_SEEDS = [3, 0x5EED5EED5EED5EED, 2**64 - 59]


def seed_search():
    w = T.workload(4)
    t = w.topo
    times, events = [], []
    for seed in SEARCH_SEEDS:
        r = oracle.synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B, w.chunks_per_npu,
                              w.chunk_bytes, w.collective, seed, keep_xfers=0)
        times.append(r.collective_time_ps)
        events.append(r.n_events)
        print(seed, r.collective_time_ps, r.n_events, flush=True)
    out = {"workload": w.name, "seeds": SEARCH_SEEDS, "collective_time_ps": times, "n_events": events}
    with open(os.path.join(HERE, "seed_search_oracle.json"), "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
        f.write("\n")


def scalability(idx, threads):
    w = T.workload(idx)
    oracle.set_progress(2000)
    r = oracle.synthesize_workload(w, keep_xfers=0, n_threads=threads)
    out = {
        "name": w.name,
        "topology": w.topo.name,
        "collective_time_ps": r.collective_time_ps,
        "n_events": r.n_events,
        "n_xfers": r.n_xfers,
        "pass_time_ps": list(r.pass_time_ps)[:2],
        "pass_events": list(r.pass_events)[:2],
        "digest": r.digest,
    }
    print(idx, out, flush=True)
    with open(os.path.join(HERE, f"workload{idx}_oracle.json"), "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
        f.write("\n")


def main():
    if "--scalability" in sys.argv:
        threads = int(sys.argv[sys.argv.index("--threads") + 1]) if "--threads" in sys.argv else 8
        scalability(int(sys.argv[sys.argv.index("--scalability") + 1]), threads)
        return
    if "--seed-search" in sys.argv:
        seed_search()
        return
    if "--with-5" in sys.argv:
        threads = int(sys.argv[sys.argv.index("--threads") + 1]) if "--threads" in sys.argv else 8
        if "--matching1" in sys.argv:
            workload5_matching1(threads)
        else:
            workload5(threads)
        return
    out = {}
    for idx in (1, 2, 3, 4):
        w = T.workload(idx)
        r = oracle.synthesize_workload(w)
        out[str(idx)] = {
            "name": w.name,
            "topology": w.topo.name,
            "collective_time_ps": r.collective_time_ps,
            "n_events": r.n_events,
            "n_xfers": r.n_xfers,
            "pass_time_ps": list(r.pass_time_ps),
            "pass_events": list(r.pass_events),
            "digest": r.digest,
            "sha256_xfers": hashlib.sha256(r.xfers.tobytes()).hexdigest(),
        }
        print(idx, out[str(idx)], flush=True)
    with open(os.path.join(HERE, "workloads_oracle.json"), "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
        f.write("\n")


if __name__ == "__main__":
    main()
