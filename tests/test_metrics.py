"""Schedule metrics (reporting only): closed forms on topologies whose ideal is known."""
import numpy as np
import pytest

import checker
import oracle
from paper_2304_05301_amd import metrics, topologies as T

MiB = 1 << 20


def _counts(xfers, n_links):
    return np.bincount(xfers["link"].astype(np.int64), minlength=n_links)


@pytest.mark.parametrize("n", [4, 8])
def test_unidirectional_ring_is_ideal_and_fully_utilised(n):
    """Ring All-Gather on a unidirectional ring: every link busy all the time, and the
    collective time equals the paper's Ideal: (n-1) chunks through one 50 GB/s port
    plus a diameter of (n-1) hops."""
    topo = T.ring(n, 500_000, 20_000)
    r = oracle.synthesize(n, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B, 1, MiB, 0, 0)
    cost = checker.link_costs_ps(topo.alpha_ps, topo.beta_fs_per_B, MiB)
    ideal = metrics.ideal_time_ps(n, 1, MiB, metrics.ALL_GATHER, topo.link_src, topo.link_dst,
                                  topo.alpha_ps, topo.beta_fs_per_B)
    m = metrics.schedule_metrics(r.collective_time_ps, [r.collective_time_ps], [_counts(r.xfers, n)],
                                 cost, n, 1, MiB, metrics.ALL_GATHER, ideal)
    assert m["mean_link_utilisation"] == pytest.approx(1.0)
    assert m["efficiency_vs_ideal"] == pytest.approx(1.0)
    assert m["bandwidth_GBps"] == pytest.approx(n * MiB / (r.collective_time_ps * 1e-12) / 1e9)


def test_ideal_terms():
    topo = T.fully_connected(4, 1_000_000, 10_000)  # 100 GB/s links, 1 us
    # every NPU has 3 incoming links of 100 GB/s; diameter = 1 hop
    bw = metrics.npu_ingress_bandwidth_Bps(4, topo.link_dst, topo.beta_fs_per_B)
    assert np.allclose(bw, 300e9)
    assert metrics.latency_diameter_ps(4, topo.link_src, topo.link_dst, topo.alpha_ps) == 1_000_000
    ag = metrics.ideal_time_ps(4, 1, MiB, metrics.ALL_GATHER, topo.link_src, topo.link_dst, topo.alpha_ps,
                               topo.beta_fs_per_B)
    ar = metrics.ideal_time_ps(4, 1, MiB, metrics.ALL_REDUCE, topo.link_src, topo.link_dst, topo.alpha_ps,
                               topo.beta_fs_per_B)
    size = 4 * MiB
    assert ag == pytest.approx(size * 0.75 / 300e9 * 1e12 + 1_000_000)
    assert ar == pytest.approx(2 * size * 0.75 / 300e9 * 1e12 + 1_000_000)


def test_efficiency_never_above_one_on_valid_schedules():
    topo = T.torus3d(4, 4, 4, 500_000, 10_000)
    r = oracle.synthesize(64, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B, 2, MiB, 2, 3)
    cost = checker.link_costs_ps(topo.alpha_ps, topo.beta_fs_per_B, MiB)
    n = len(r.xfers) // 2
    ideal = metrics.ideal_time_ps(64, 2, MiB, metrics.ALL_REDUCE, topo.link_src, topo.link_dst, topo.alpha_ps,
                                  topo.beta_fs_per_B)
    m = metrics.schedule_metrics(r.collective_time_ps, list(r.pass_time_ps),
                                 [_counts(r.xfers[:n], topo.n_links), _counts(r.xfers[n:], topo.n_links)],
                                 cost, 64, 2, MiB, metrics.ALL_REDUCE, ideal)
    assert 0.5 < m["efficiency_vs_ideal"] <= 1.0
    assert 0.5 < m["mean_link_utilisation"] <= 1.0
