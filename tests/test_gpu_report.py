"""The reporting / pre-processing entry points of the C ABI (switch unwinding, link busy times,
the paper's Ideal) against the CPU oracle (oracle/report.py), value by value."""
import numpy as np
import pytest

import checker
import oracle
from oracle import report
from paper_2304_05301_amd import binding, topologies as T

pytestmark = pytest.mark.gpu
MiB = 1 << 20


@pytest.mark.parametrize("n,d", [(2, 1), (4, 1), (4, 2), (4, 3), (9, 8), (12, 3), (64, 17), (257, 100), (4096, 6),
                                 (40_000, 5)])
def test_switch_unwinding_equals_oracle(n, d):
    rp, col, al, be = binding.tacos_unwind_switch(n, d, 700_000, 20_000)
    wrp, wcol, wal, wbe = report.unwind_switch(n, d, 700_000, 20_000)
    assert rp.tolist() == wrp and col.tolist() == wcol and al.tolist() == wal and be.tolist() == wbe


def test_switch_unwinding_errors_and_use_as_a_topology():
    for n, d in ((1, 1), (4, 0), (4, 4), (0, 0)):
        with pytest.raises(binding.TacosError) as e:
            binding.tacos_unwind_switch(n, d, 1, 1)
        assert e.value.code == binding.TACOS_E_INVAL
    with pytest.raises(binding.TacosError) as e:
        binding.tacos_unwind_switch(8, 3, 1, (1 << 64) - 1)
    assert e.value.code == binding.TACOS_E_OVERFLOW
    # the unwound switch goes straight into the synthesis: bit-exact against the oracle
    rp, col, al, be = binding.tacos_unwind_switch(12, 3, 500_000, 20_000)
    ref = oracle.synthesize(12, rp, col, al, be, 2, MiB, T.ALL_REDUCE, 5)
    with binding.tacos_synthesize(12, rp, col, al, be, 2, MiB, T.ALL_REDUCE, 5) as r:
        assert r.collective_time_ps == ref.collective_time_ps and np.array_equal(r.read(), ref.xfers)


IDEAL = [
    ("ring8", lambda: T.ring(8), 1),
    ("fc16", lambda: T.fully_connected(16), 2),
    ("mesh5x4", lambda: T.mesh2d(5, 4), 3),
    ("hetero_torus", lambda: T.grid([3, 2, 3], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000]), 2),
    ("random40", lambda: T.random_regular_out(40, 3, seed=7)[0], 1),
    ("random300", lambda: T.random_regular_out(300, 4, seed=1)[0], 5),
    ("switch12d3", lambda: T.switch_unwound(12, 3), 1),
    ("odd_betas", lambda: T.from_edge_list(3, [(0, 1, 10, 7), (0, 2, 11, 13), (1, 0, 12, 7919), (1, 2, 13, 3),
                                               (2, 0, 14, 104_729), (2, 1, 15, 0)]), 1),
    ("torus16x16x16", lambda: T.torus3d(16, 16, 16), 1),
]


@pytest.mark.parametrize("name,mk,cpn", IDEAL, ids=[c[0] for c in IDEAL])
@pytest.mark.parametrize("coll", [T.ALL_GATHER, T.REDUCE_SCATTER, T.ALL_REDUCE])
def test_ideal_bound_equals_oracle(name, mk, cpn, coll):
    topo = mk()
    for cb in (1, 192 << 10, (1 << 30) + 7):
        with_diam = topo.n_npus <= 512
        got = binding.tacos_ideal_bound(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B,
                                        cpn, cb, coll, with_diameter=with_diam)
        want = report.ideal_bound(topo.n_npus, topo.link_src, topo.link_dst, topo.alpha_ps, topo.beta_fs_per_B,
                                  cpn, cb, coll, with_diameter=with_diam)
        assert got == want, (name, cb)
    if name == "torus16x16x16" and coll == T.ALL_GATHER:   # 4,096 NPUs: diameter 3 * 8 hops
        got = binding.tacos_ideal_bound(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B,
                                        1, MiB, coll)
        assert got["diameter_ps"] == 24 * 500_000


def test_ideal_bound_errors():
    topo = T.mesh2d(4, 4)
    args = (topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B, 1, MiB)
    with pytest.raises(binding.TacosError) as e:
        binding.tacos_ideal_bound(*args, T.BROADCAST)
    assert e.value.code == binding.TACOS_E_INVAL
    big = T.workload(5).topo
    with pytest.raises(binding.TacosError) as e:   # the diameter is for at most 8,192 NPUs
        binding.tacos_ideal_bound(big.n_npus, big.row_ptr, big.col_idx, big.alpha_ps, big.beta_fs_per_B, 1, MiB, 0)
    assert e.value.code == binding.TACOS_E_INVAL
    got = binding.tacos_ideal_bound(big.n_npus, big.row_ptr, big.col_idx, big.alpha_ps, big.beta_fs_per_B, 1, MiB, 0,
                                    with_diameter=False)
    assert got["bandwidth_term_ps"] == -(-(40_959 * MiB * 10_000) // (6 * 1000)) and got["diameter_ps"] == 0
    # NPU 2 sends but never receives: no ingress bandwidth; and it is not reached
    broken = T.from_edge_list(3, [(0, 1, 5, 10), (1, 0, 5, 10), (2, 0, 5, 10)])
    with pytest.raises(binding.TacosError) as e:
        binding.tacos_ideal_bound(3, broken.row_ptr, broken.col_idx, broken.alpha_ps, broken.beta_fs_per_B, 1, MiB, 0)
    assert e.value.code == binding.TACOS_E_UNREACHABLE
    huge = T.from_edge_list(2, [(0, 1, 5, (1 << 63) + 1), (1, 0, 5, 3)])
    with pytest.raises(binding.TacosError) as e:
        binding.tacos_ideal_bound(2, huge.row_ptr, huge.col_idx, huge.alpha_ps, huge.beta_fs_per_B, 1, 1 << 40, 0)
    assert e.value.code == binding.TACOS_E_OVERFLOW


BUSY = [
    ("ring8_ag", lambda: T.ring(8), 1, T.ALL_GATHER),
    ("mesh5x4_ag", lambda: T.mesh2d(5, 4), 3, T.ALL_GATHER),
    ("hetero_torus_ar", lambda: T.grid([3, 3, 2], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000]), 3, T.ALL_REDUCE),
    ("random40_rs", lambda: T.random_regular_out(40, 3, seed=7)[0], 2, T.REDUCE_SCATTER),
    ("torus8x8x8_ag_per_span_launches", lambda: T.torus3d(8, 8, 8), 20, T.ALL_GATHER),
]


@pytest.mark.parametrize("name,mk,cpn,coll", BUSY, ids=[c[0] for c in BUSY])
def test_link_busy_times_equal_oracle(name, mk, cpn, coll):
    topo = mk()
    cb = 192 << 10
    ref = oracle.synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B, cpn, cb, coll, 3)
    cost = checker.link_costs_ps(topo.alpha_ps, topo.beta_fs_per_B, cb)
    n_pass = 2 if coll == T.ALL_REDUCE else 1
    n = len(ref.xfers) // n_pass
    with binding.tacos_synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B, cpn, cb,
                                  coll, 3) as r:
        for k in range(n_pass):
            want = report.link_busy_ps(ref.xfers["link"][k * n:(k + 1) * n], cost, topo.n_links)
            busy, s, mn, mx = r.link_busy(k, topo.n_links)
            assert busy.tolist() == want and (s, mn, mx) == (sum(want), min(want), max(want)), (name, k)
            assert mx <= r.pass_time_ps(k)
