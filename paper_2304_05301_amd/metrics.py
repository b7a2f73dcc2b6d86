"""Reporting on a synthesized schedule: the quantities the paper uses to judge a
collective algorithm (collective bandwidth, link utilisation, efficiency against the
theoretical ideal).  Pure numpy on numbers read through the C ABI (collective time,
per-link transfer counts, link costs); nothing here takes part in the synthesis.

Paper, section "Baseline Collective Algorithms and Synthesizers":
    Ideal = CollectiveSize * 2(n-1)/n / min_N(BW_N) + Diameter          (All-Reduce)
with the bandwidth term halved for All-Gather / Reduce-Scatter alone; BW_N is the
bandwidth of the worst-connected NPU and Diameter the latency between the two
farthest NPUs.  Section "Topology Exploration": bandwidth = collective size / time.
"""
from __future__ import annotations

import heapq
from typing import Optional

import numpy as np

ALL_GATHER, REDUCE_SCATTER, ALL_REDUCE = 0, 1, 2


def npu_ingress_bandwidth_Bps(n_npus, link_dst, beta_fs_per_B) -> np.ndarray:
    """Sum over an NPU's incoming links of 1/beta, in bytes per second."""
    bw = np.zeros(int(n_npus), dtype=np.float64)
    beta = np.asarray(beta_fs_per_B, dtype=np.float64)
    with np.errstate(divide="ignore"):
        per_link = np.where(beta > 0, 1.0e15 / beta, np.inf)
    np.add.at(bw, np.asarray(link_dst, dtype=np.int64), per_link)
    return bw


def latency_diameter_ps(n_npus, link_src, link_dst, alpha_ps) -> int:
    """Largest shortest-path latency (alpha only) between two NPUs; Dijkstra from every
    NPU, so meant for topologies of up to a few thousand NPUs."""
    n = int(n_npus)
    adj = [[] for _ in range(n)]
    for s, d, a in zip(link_src, link_dst, alpha_ps):
        adj[int(s)].append((int(d), int(a)))
    worst = 0
    for s in range(n):
        dist = [None] * n
        dist[s] = 0
        pq = [(0, s)]
        while pq:
            du, u = heapq.heappop(pq)
            if du > dist[u]:
                continue
            for v, a in adj[u]:
                nd = du + a
                if dist[v] is None or nd < dist[v]:
                    dist[v] = nd
                    heapq.heappush(pq, (nd, v))
        if any(x is None for x in dist):
            raise ValueError("topology is not strongly connected")
        worst = max(worst, max(dist))
    return worst


def ideal_time_ps(n_npus, chunks_per_npu, chunk_bytes, collective, link_src, link_dst, alpha_ps,
                  beta_fs_per_B, with_diameter: bool = True) -> float:
    """The paper's 'Ideal' collective time in picoseconds."""
    n = int(n_npus)
    size = n * int(chunks_per_npu) * int(chunk_bytes)          # bytes every NPU ends up with
    factor = 2.0 if collective == ALL_REDUCE else 1.0
    bw = npu_ingress_bandwidth_Bps(n, link_dst, beta_fs_per_B).min()
    t = factor * size * (n - 1) / n / bw * 1.0e12
    if with_diameter:
        t += latency_diameter_ps(n, link_src, link_dst, alpha_ps)
    return t


def schedule_metrics(collective_time_ps, pass_times_ps, link_counts_per_pass, cost_ps, n_npus,
                     chunks_per_npu, chunk_bytes, collective, ideal_ps: Optional[float] = None) -> dict:
    """Bandwidth, utilisation and efficiency of a schedule.

    link_counts_per_pass: one array [n_links] per pass (transfers carried by each link).
    Link utilisation of a pass = busy time / pass time = count * cost / pass time."""
    cost = np.asarray(cost_ps, dtype=np.float64)
    size = int(n_npus) * int(chunks_per_npu) * int(chunk_bytes)
    util = []
    for T, counts in zip(pass_times_ps, link_counts_per_pass):
        busy = np.asarray(counts, dtype=np.float64) * cost
        util.append(busy / float(T) if T else np.zeros_like(busy))
    out = {
        "collective_bytes": size,
        "collective_time_us": collective_time_ps / 1.0e6,
        "bandwidth_GBps": (size / (collective_time_ps * 1.0e-12) / 1.0e9) if collective_time_ps else float("inf"),
        "mean_link_utilisation": float(np.mean([u.mean() for u in util])) if util else 0.0,
        "min_link_utilisation": float(min(u.min() for u in util)) if util else 0.0,
        "max_link_utilisation": float(max(u.max() for u in util)) if util else 0.0,
        "link_utilisation_per_pass": util,
    }
    if ideal_ps is not None:
        out["ideal_time_us"] = ideal_ps / 1.0e6
        out["efficiency_vs_ideal"] = (ideal_ps / collective_time_ps) if collective_time_ps else 1.0
    return out
