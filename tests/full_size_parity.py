"""One-off full-size parity run (not collected by pytest: it takes minutes).

    python tests/full_size_parity.py [--threads 16] [--workload N] [--collective ag|rs|ar]
                                     [--matching 0|1] [--link-order 0|1]

Runs the 40,960-NPU torus All-Gather (workload 5) to completion on the GPU through the
C ABI and in the CPU oracle (OpenMP over destinations), and compares collective time,
number of TEN spans, number of matches, the per-span match counts and the schedule
digest over all 1.68e9 transfers.  The oracle prints its own progress lines.
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2304_05301_amd import binding, topologies as T  # noqa: E402


def reversed_run(w, threads, opt):
    """Reduce-Scatter / All-Reduce at full size: the oracle digests its records without
    materialising them (keep_xfers=0), so collective time, per-pass times and spans, the
    number of transfers and the digest over all of them are compared."""
    t0 = time.time()
    r = binding.synthesize_workload(w, **opt)
    gpu = dict(T=r.collective_time_ps, events=r.num_events, xfers=r.num_xfers, digest=r.digest,
               pass_T=[r.pass_time_ps(i) for i in range(r.num_passes)],
               pass_events=[r.pass_events(i) for i in range(r.num_passes)])
    r.free()
    print(f"gpu   {gpu} in {time.time() - t0:.1f} s", flush=True)
    oracle.set_progress(1000)
    t0 = time.time()
    ref = oracle.synthesize_workload(w, keep_xfers=0, n_threads=threads, **opt)
    n_pass = len(gpu["pass_T"])
    print(f"oracle T={ref.collective_time_ps} events={ref.n_events} xfers={ref.n_xfers} digest={ref.digest} "
          f"pass_T={ref.pass_time_ps[:n_pass]} in {time.time() - t0:.1f} s with {threads} threads", flush=True)
    ok = (gpu["T"] == ref.collective_time_ps and gpu["events"] == ref.n_events and
          gpu["xfers"] == ref.n_xfers and gpu["digest"] == ref.digest and
          gpu["pass_T"] == list(ref.pass_time_ps[:n_pass]) and
          gpu["pass_events"] == list(ref.pass_events[:n_pass]))
    print("FULL-SIZE PARITY:", "PASS" if ok else "FAIL", flush=True)
    sys.exit(0 if ok else 1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--threads", type=int, default=16)
    ap.add_argument("--workload", type=int, default=5)
    ap.add_argument("--collective", choices=["ag", "rs", "ar"], default=None,
                    help="override the workload's collective (rs/ar: digest, times and counts only)")
    ap.add_argument("--cpn", type=int, default=0,
                    help="override chunks per NPU (the collective size stays: chunk bytes are divided)")
    ap.add_argument("--matching", type=int, default=0, help="0 link-centric, 1 postcondition-centric")
    ap.add_argument("--link-order", type=int, default=0, help="0 by link id, 1 cheapest first")
    args = ap.parse_args()
    opt = dict(matching=args.matching, link_order=args.link_order)
    w = T.workload(args.workload)
    if args.cpn:
        w = T.Workload(f"{w.name}_cpn{args.cpn}", w.topo, args.cpn,
                       w.chunk_bytes * w.chunks_per_npu // args.cpn, w.collective, w.seed)
    if args.collective:
        coll = {"ag": T.ALL_GATHER, "rs": T.REDUCE_SCATTER, "ar": T.ALL_REDUCE}[args.collective]
        w = T.Workload(w.name + "_" + args.collective, w.topo, w.chunks_per_npu, w.chunk_bytes, coll, w.seed)
    if w.collective != T.ALL_GATHER:
        return reversed_run(w, args.threads, opt)
    t0 = time.time()
    r = binding.synthesize_workload(w, **opt)
    gpu = dict(T=r.collective_time_ps, events=r.num_events, xfers=r.num_xfers, digest=r.digest)
    gt, gm = r.event_trace(0)
    first = r.read(0, 1000)
    last = r.read(r.num_xfers - 1000, 1000)
    r.free()
    print(f"gpu   {gpu} in {time.time() - t0:.1f} s", flush=True)
    oracle.set_progress(500)
    t0 = time.time()
    ref = oracle.synthesize_workload(w, keep_first=0, keep_xfers=1000, n_threads=args.threads, **opt)
    print(f"oracle T={ref.collective_time_ps} events={ref.n_events} xfers={ref.n_xfers} "
          f"digest={ref.digest} in {time.time() - t0:.1f} s with {args.threads} threads", flush=True)
    ok = (gpu["T"] == ref.collective_time_ps and gpu["events"] == ref.n_events and
          gpu["xfers"] == ref.n_xfers and gpu["digest"] == ref.digest and
          np.array_equal(gt, ref.event_times) and np.array_equal(gm, ref.event_matches) and
          np.array_equal(first, ref.xfers))
    print("first-1000 records equal:", np.array_equal(first, ref.xfers))
    print("per-span times equal:", np.array_equal(gt, ref.event_times),
          " per-span match counts equal:", np.array_equal(gm, ref.event_matches))
    print("last GPU record:", last[-1])
    print("FULL-SIZE PARITY:", "PASS" if ok else "FAIL", flush=True)
    sys.exit(0 if ok else 1)


if __name__ == "__main__":
    main()
