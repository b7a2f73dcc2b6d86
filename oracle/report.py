"""TEST INFRASTRUCTURE: plain CPU oracle of the quantities around the synthesis (exact
python integers and fractions; pure-python loops, so for small inputs).

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this module;
it imports nothing from the product package and shares no code with the HIP path.

  unwind_switch  paper, section "TACOS for Switch-based Networks": an N-NPU switch unwound with
                 degree d gives NPU i the d outgoing links to NPUs i+1 .. i+d (mod N); alpha stays,
                 beta is multiplied by d.
  link_busy_ps   busy time of every link in one pass = sum of the costs of the transfers it
                 carries (link utilisation = busy time / pass time; section "Analysis of
                 TACOS-Synthesized Algorithms").
  ideal_bound    paper, section "Baseline Collective Algorithms and Synthesizers":
                 Ideal = CollectiveSize * 2(n-1)/n / min_NPU(BW_NPU) + Diameter.

Readings (the paper gives the formula for All-Reduce only): CollectiveSize = n * chunks per
NPU * chunk bytes.  An All-Gather makes every NPU RECEIVE CollectiveSize*(n-1)/n bytes, so its
bandwidth term divides by the smallest ingress bandwidth (sum of 1/beta over the incoming
links); a Reduce-Scatter makes every NPU SEND as much: smallest egress bandwidth; All-Reduce =
Reduce-Scatter term + All-Gather term (the factor 2 of the formula when both sides are equal).
Each term is rounded up to a whole picosecond.  Diameter = largest over ordered pairs of the
smallest sum of alpha along a path.

Pins (tests/test_report_oracle.py): the unwound link lists of the paper's 4-NPU figure
(degrees 1..3), closed forms on ring / complete graph / unwound switch, the one-way ring whose
synthesized All-Gather meets the Ideal exactly, brute-force path enumeration for the diameter.
"""
from __future__ import annotations

import heapq
from fractions import Fraction

ALL_GATHER, REDUCE_SCATTER, ALL_REDUCE = 0, 1, 2


def unwind_switch(n_npus: int, degree: int, alpha_ps: int, beta_fs_per_B: int):
    """(row_ptr, col_idx, alpha, beta) python lists: CSR by source, ascending destination."""
    n, d = int(n_npus), int(degree)
    if n < 2 or not 1 <= d <= n - 1:
        raise ValueError("need n >= 2 and 1 <= degree <= n - 1")
    row_ptr, col, al, be = [0], [], [], []
    for i in range(n):
        for dst in sorted((i + k) % n for k in range(1, d + 1)):
            col.append(dst)
            al.append(int(alpha_ps))
            be.append(int(beta_fs_per_B) * d)
        row_ptr.append(len(col))
    return row_ptr, col, al, be


def link_busy_ps(xfer_links, cost_ps, n_links: int):
    """busy[l] = sum of cost[l] over the transfers on link l (python ints)."""
    busy = [0] * int(n_links)
    for l in xfer_links:
        busy[int(l)] += int(cost_ps[int(l)])
    return busy


def _per_byte_fs(betas):
    """Femtoseconds per byte through links of reciprocal bandwidths `betas` used together."""
    if not betas:
        raise ValueError("an NPU without a link on this side")
    if any(b == 0 for b in betas):
        return Fraction(0)
    return 1 / sum(Fraction(1, int(b)) for b in betas)


def latency_diameter_ps(n_npus, link_src, link_dst, alpha_ps) -> int:
    n = int(n_npus)
    adj = [[] for _ in range(n)]
    for s, d, a in zip(link_src, link_dst, alpha_ps):
        adj[int(s)].append((int(d), int(a)))
    worst = 0
    for s in range(n):
        dist = {s: 0}
        pq = [(0, s)]
        while pq:
            du, u = heapq.heappop(pq)
            if du > dist[u]:
                continue
            for v, a in adj[u]:
                if v not in dist or du + a < dist[v]:
                    dist[v] = du + a
                    heapq.heappush(pq, (du + a, v))
        if len(dist) != n:
            raise ValueError("not strongly connected")
        worst = max(worst, max(dist.values()))
    return worst


def ideal_bound(n_npus, link_src, link_dst, alpha_ps, beta_fs_per_B, chunks_per_npu, chunk_bytes, collective,
                with_diameter=True) -> dict:
    n = int(n_npus)
    size = n * int(chunks_per_npu) * int(chunk_bytes)
    moved = (n - 1) * int(chunks_per_npu) * int(chunk_bytes)      # = size * (n - 1) / n
    ingress = [[] for _ in range(n)]
    egress = [[] for _ in range(n)]
    for s, d, b in zip(link_src, link_dst, beta_fs_per_B):
        egress[int(s)].append(int(b))
        ingress[int(d)].append(int(b))

    def term(side):
        per_byte = [_per_byte_fs(x) for x in side]
        worst = max(per_byte)
        npu = per_byte.index(worst)                               # lowest id on ties
        fs = worst * moved
        ps = -((-fs.numerator) // (fs.denominator * 1000))        # ceil(fs / 1000)
        return ps, npu

    passes = {ALL_GATHER: [ingress], REDUCE_SCATTER: [egress], ALL_REDUCE: [egress, ingress]}[int(collective)]
    terms = [term(side) for side in passes] if n > 1 else []
    diam = latency_diameter_ps(n, link_src, link_dst, alpha_ps) if (with_diameter and n > 1) else 0
    bw = sum(t for t, _ in terms)
    return {"collective_bytes": size, "bandwidth_term_ps": bw, "diameter_ps": diam, "ideal_ps": bw + diam,
            "pass_bandwidth_term_ps": [t for t, _ in terms], "pass_bottleneck_npu": [i for _, i in terms]}
