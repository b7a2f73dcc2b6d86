"""Writes tests/golden/workloads_oracle.json from the CPU oracle ONLY.

Run:  python tests/golden/make_golden.py
It calls nothing but the input generators and oracle/; the HIP path is never involved.
Stored per workload 1..4: collective time, matching sweeps, records, the schedule
digest and the SHA-256 of the canonical record array (little-endian structs of
t_ps:u64, src:u32, dst:u32, chunk:u32, link:u32).  Workload 4 takes about a minute.
"""
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_2304_05301_amd import topologies as T  # noqa: E402


def main():
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
