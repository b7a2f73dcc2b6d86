"""Formatting of the library's schedule metrics for reports: ratios of the exact integers
the C ABI returns (tacos_result_link_busy, tacos_ideal_bound, pass and collective times).
Nothing here computes a metric from a schedule or a topology; that is done on the device.

Paper: bandwidth = collective size / collective time (section "Topology Exploration"); link
utilisation = busy time / execution time (section "Analysis of TACOS-Synthesized
Algorithms"); efficiency = Ideal / collective time (section "Baseline Collective Algorithms and
Synthesizers").
"""
from __future__ import annotations

from typing import Optional, Sequence


def bandwidth_GBps(collective_bytes: int, collective_time_ps: int) -> float:
    return float("inf") if not collective_time_ps else collective_bytes / (collective_time_ps * 1.0e-12) / 1.0e9


def efficiency(ideal_ps: int, collective_time_ps: int) -> float:
    return 1.0 if not collective_time_ps else ideal_ps / collective_time_ps


def utilisation(busy_sum_ps: int, n_links: int, pass_time_ps: int) -> float:
    """Mean link utilisation of a pass = sum of the link busy times / (links * pass time)."""
    return 0.0 if not (n_links and pass_time_ps) else busy_sum_ps / (n_links * pass_time_ps)


def summary(collective_bytes: int, collective_time_ps: int, pass_times_ps: Sequence[int],
            pass_busy: Sequence[tuple], n_links: int, ideal_ps: Optional[int] = None) -> dict:
    """pass_busy: per pass (sum, min, max) of the link busy times in ps."""
    out = {
        "collective_bytes": collective_bytes,
        "collective_time_us": collective_time_ps / 1.0e6,
        "bandwidth_GBps": bandwidth_GBps(collective_bytes, collective_time_ps),
        "mean_link_utilisation_per_pass": [utilisation(s, n_links, T) for (s, _, _), T in zip(pass_busy, pass_times_ps)],
        "min_link_utilisation_per_pass": [mn / T if T else 0.0 for (_, mn, _), T in zip(pass_busy, pass_times_ps)],
        "max_link_utilisation_per_pass": [mx / T if T else 0.0 for (_, _, mx), T in zip(pass_busy, pass_times_ps)],
    }
    if ideal_ps is not None:
        out["ideal_time_us"] = ideal_ps / 1.0e6
        out["efficiency_vs_ideal"] = efficiency(ideal_ps, collective_time_ps)
    return out
