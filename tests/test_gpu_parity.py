"""Parity of the HIP path (through the C ABI) with the CPU oracle: bit-exact schedules,
collective times, event traces and digests on the same seeded inputs."""
import hashlib
import json
import os

import numpy as np
import pytest

import checker
import oracle
from paper_2304_05301_amd import binding, topologies as T

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "workloads_oracle.json")
MiB = 1 << 20


@pytest.fixture(scope="module")
def stream():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a HIP device"
    torch.cuda.set_device(0)
    return torch.cuda.current_stream().cuda_stream


def gpu(topo, cpn, cb, coll, seed, stream, **kw):
    return binding.tacos_synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps,
                                    topo.beta_fs_per_B, cpn, cb, coll, seed, stream=stream, **kw)


def cpu(topo, cpn, cb, coll, seed, **kw):
    return oracle.synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps,
                             topo.beta_fs_per_B, cpn, cb, coll, seed, **kw)


def assert_same(r, ref, name=""):
    assert r.collective_time_ps == ref.collective_time_ps, name
    assert r.num_events == ref.n_events, name
    assert r.num_xfers == ref.n_xfers, name
    got = r.read()
    assert got.shape == ref.xfers.shape, name
    if not np.array_equal(got, ref.xfers):
        bad = np.nonzero(got != ref.xfers)[0]
        i = int(bad[0])
        raise AssertionError(f"{name}: first difference at record {i}: gpu {got[i]} oracle {ref.xfers[i]} "
                             f"({len(bad)} differ)")
    assert r.digest == ref.digest, name


def test_link_costs_match_alpha_beta_model(stream):
    """a1: alpha + beta*n in integer ps, against python integers."""
    rng = np.random.default_rng(0)
    L = 1000
    edges = [(0, 1, int(a), int(b)) for a, b in zip(rng.integers(0, 5_000_000, L), rng.integers(0, 80_000, L))]
    topo = T.from_edge_list(2, edges)
    for cb in (1, 999, MiB, 4 * MiB, (1 << 40) + 12345):
        got = binding.tacos_link_costs(2, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B, cb)
        want = checker.link_costs_ps(topo.alpha_ps, topo.beta_fs_per_B, cb)
        assert got.tolist() == want
    big = T.from_edge_list(2, [(0, 1, 0, (1 << 64) - 1), (1, 0, (1 << 64) - 1, 1000)])
    with pytest.raises(binding.TacosError) as e:
        binding.tacos_link_costs(2, big.row_ptr, big.col_idx, big.alpha_ps, big.beta_fs_per_B, 1 << 30)
    assert e.value.code == binding.TACOS_E_OVERFLOW


SMALL = [
    ("uniring2", lambda: T.ring(2), 1, T.ALL_GATHER),
    ("uniring13", lambda: T.ring(13), 1, T.ALL_GATHER),
    ("biring9_cpn3", lambda: T.ring(9, bidirectional=True), 3, T.ALL_GATHER),
    ("fc16", lambda: T.fully_connected(16), 1, T.ALL_GATHER),
    ("fc70_indeg_over_64", lambda: T.fully_connected(70), 2, T.ALL_GATHER),
    ("mesh5x4_cpn7", lambda: T.mesh2d(5, 4), 7, T.ALL_GATHER),
    ("torus2x3_parallel_links", lambda: T.grid([2, 3], True), 2, T.ALL_GATHER),
    ("hetero_torus_rs", lambda: T.grid([3, 2, 3], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000]), 2, T.REDUCE_SCATTER),
    ("hetero_torus_ar", lambda: T.grid([3, 3, 2], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000]), 3, T.ALL_REDUCE),
    ("random40_ag", lambda: T.random_regular_out(40, 3, seed=7)[0], 2, T.ALL_GATHER),
    ("random40_ar", lambda: T.random_regular_out(40, 3, seed=7)[0], 1, T.ALL_REDUCE),
    ("switch12d3_rs", lambda: T.switch_unwound(12, 3), 1, T.REDUCE_SCATTER),
]


@pytest.mark.parametrize("name,mk,cpn,coll", SMALL, ids=[c[0] for c in SMALL])
@pytest.mark.parametrize("seed", [0, 0xDEADBEEFCAFE])
def test_small_cases_bit_exact(name, mk, cpn, coll, seed, stream):
    topo = mk()
    cb = 192 << 10
    ref = cpu(topo, cpn, cb, coll, seed)
    with gpu(topo, cpn, cb, coll, seed, stream) as r:
        assert_same(r, ref, name)
        assert r.num_passes == (2 if coll == T.ALL_REDUCE else 1)
        # per-span trace (times and matches made) of the LAST pass is what the oracle keeps; the
        # Reduce-Scatter half of an All-Reduce equals the Reduce-Scatter alone
        last = r.num_passes - 1
        t, m = r.event_trace(last)
        assert np.array_equal(t, ref.event_times) and np.array_equal(m, ref.event_matches), name
        assert int(m.sum()) == r.num_xfers // r.num_passes
        if coll == T.ALL_REDUCE:
            rs = cpu(topo, cpn, cb, T.REDUCE_SCATTER, seed)
            t, m = r.event_trace(0)
            assert np.array_equal(t, rs.event_times) and np.array_equal(m, rs.event_matches), name


def test_event_trace_of_a_reversed_pass_two_npus(stream):
    """Two NPUs, one chunk each, links of cost 7 and 3: the reversed pass of the
    Reduce-Scatter matches both links in its sweep at t = 0, sweeps again (matching nothing)
    when the faster link has delivered at t = 3, and ends at t = 7."""
    topo = T.from_edge_list(2, [(0, 1, 7, 0), (1, 0, 3, 0)])
    ref = cpu(topo, 1, 1, T.REDUCE_SCATTER, 0)
    assert ref.event_times.tolist() == [0, 3] and ref.event_matches.tolist() == [2, 0]
    for mode in (1, 2):
        with gpu(topo, 1, 1, T.REDUCE_SCATTER, 0, stream, launch_mode=mode) as r:
            assert r.collective_time_ps == 7
            t, m = r.event_trace(0)
            assert t.tolist() == [0, 3] and m.tolist() == [2, 0]


def test_single_npu(stream):
    topo = T.from_edge_list(1, [])
    for coll in (T.ALL_GATHER, T.REDUCE_SCATTER, T.ALL_REDUCE):
        with gpu(topo, 3, MiB, coll, 0, stream) as r:
            assert (r.collective_time_ps, r.num_events, r.num_xfers, r.digest) == (0, 0, 0, 0)
            assert len(r.read()) == 0


def test_unreachable_is_an_error(stream):
    topo = T.from_edge_list(3, [(0, 1, 1, 0), (1, 2, 1, 0)])
    with pytest.raises(binding.TacosError) as e:
        gpu(topo, 1, 1, T.ALL_GATHER, 0, stream)
    assert e.value.code == binding.TACOS_E_UNREACHABLE
    nolinks = T.from_edge_list(2, [])
    with pytest.raises(binding.TacosError) as e:
        gpu(nolinks, 1, 1, T.ALL_GATHER, 0, stream)
    assert e.value.code == binding.TACOS_E_UNREACHABLE


NOT_STRONGLY_CONNECTED = [
    ("never_receives", lambda: T.from_edge_list(3, [(0, 1, 500_000, 20_000), (1, 0, 500_000, 20_000), (2, 0, 500_000, 20_000)])),
    ("never_sends", lambda: T.from_edge_list(3, [(0, 1, 1000, 10), (1, 0, 1000, 10), (0, 2, 1000, 10)])),
    ("two_islands", lambda: T.from_edge_list(4, [(0, 1, 1000, 10), (1, 0, 1000, 10), (2, 3, 1000, 10), (3, 2, 1000, 10)])),
    ("path", lambda: T.from_edge_list(3, [(0, 1, 1, 0), (1, 2, 1, 0)])),
]


@pytest.mark.parametrize("mode", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("name,mk", NOT_STRONGLY_CONNECTED, ids=[c[0] for c in NOT_STRONGLY_CONNECTED])
def test_not_strongly_connected_is_an_error_in_every_launch_mode(name, mk, mode, stream):
    """Postconditions left and nothing in flight (Algorithm 2 would expand the TEN for ever): an
    error from the oracle and from every launch mode, for every collective and both matching
    orders, also when the NPU that cannot be served has no incoming link at all."""
    topo = mk()
    for coll in (T.ALL_GATHER, T.REDUCE_SCATTER, T.ALL_REDUCE):
        for matching in (0, 1):
            if mode == 3 and matching == 1:
                continue  # one launch per span is link-centric only
            with pytest.raises(oracle.OracleError) as e2:
                cpu(topo, 2, MiB, coll, 5, matching=matching)
            assert e2.value.code == oracle.E_UNREACHABLE, (name, coll, matching)
            with pytest.raises(binding.TacosError) as e:
                gpu(topo, 2, MiB, coll, 5, stream, launch_mode=mode, matching=matching)
            assert e.value.code == binding.TACOS_E_UNREACHABLE, (name, coll, matching)


def test_large_topology_with_an_npu_nothing_reaches_is_an_error(stream):
    """The same on a topology of the size the per-span launches take automatically: a 70 x 70
    mesh plus one NPU that sends into it and never receives."""
    m = T.mesh2d(70, 70)
    src = np.repeat(np.arange(m.n_npus), np.diff(m.row_ptr))
    edges = [(int(a), int(b), 500_000, 10_000) for a, b in zip(src, m.col_idx)] + [(m.n_npus, 0, 500_000, 10_000)]
    topo = T.from_edge_list(m.n_npus + 1, edges)
    for coll in (T.ALL_GATHER, T.REDUCE_SCATTER):
        with pytest.raises(binding.TacosError) as e:
            gpu(topo, 1, MiB, coll, 0, stream)
        assert e.value.code == binding.TACOS_E_UNREACHABLE


@pytest.mark.parametrize("mode", [0, 1, 2, 4])
def test_broadcast_root_needs_no_incoming_link(mode, stream):
    """A root that nothing reaches is fine for a Broadcast (it holds every chunk) and for the
    Reduce towards it in the reversed orientation only if it can be reached there: record by
    record against the oracle, and the error where the oracle gives one."""
    topo = T.from_edge_list(3, [(0, 1, 500_000, 20_000), (1, 0, 500_000, 20_000), (2, 0, 300_000, 10_000)])
    ref = cpu(topo, 9, MiB, T.BROADCAST, 3, root=2)
    with gpu(topo, 9, MiB, T.BROADCAST, 3, stream, root=2, launch_mode=mode) as r:
        assert_same(r, ref, "broadcast from an NPU without incoming links")
    with pytest.raises(oracle.OracleError) as e2:
        cpu(topo, 9, MiB, T.BROADCAST, 3, root=0)
    assert e2.value.code == oracle.E_UNREACHABLE
    with pytest.raises(binding.TacosError) as e:
        gpu(topo, 9, MiB, T.BROADCAST, 3, stream, root=0, launch_mode=mode)
    assert e.value.code == binding.TACOS_E_UNREACHABLE


def test_time_overflow_is_an_error(stream):
    # two hops of cost 2^63 each: the second transfer would end beyond 2^64
    big = (1 << 63)
    topo = T.from_edge_list(3, [(0, 1, big, 0), (1, 2, big, 0), (2, 0, 1, 0), (1, 0, 1, 0), (2, 1, 1, 0)])
    with pytest.raises(binding.TacosError) as e:
        gpu(topo, 1, 1, T.ALL_GATHER, 0, stream)
    assert e.value.code == binding.TACOS_E_OVERFLOW
    with pytest.raises(oracle.OracleError) as e2:
        cpu(topo, 1, 1, T.ALL_GATHER, 0)
    assert e2.value.code == oracle.E_OVERFLOW


@pytest.mark.parametrize("C_npus,cpn", [(128, 65), (96, 171), (64, 1024)])
def test_several_pieces_and_ragged_tail(C_npus, cpn, stream):
    """Chunk counts that span 2, 3 and 8 one-KiB pieces per row, the first two with a
    ragged last word."""
    topo = T.torus3d(4, 4, C_npus // 16)
    ref = cpu(topo, cpn, MiB, T.ALL_GATHER, 21, max_events=40)
    with gpu(topo, cpn, MiB, T.ALL_GATHER, 21, stream, max_events=40) as r:
        assert_same(r, ref, f"C={C_npus * cpn}")


def test_windowed_read_and_errors(stream):
    topo = T.mesh2d(6, 5)
    ref = cpu(topo, 2, MiB, T.ALL_REDUCE, 4)
    with gpu(topo, 2, MiB, T.ALL_REDUCE, 4, stream) as r:
        n = r.num_xfers
        for first, count in ((0, 1), (n - 1, 1), (17, 1000), (n // 2 - 50, 100), (0, 0), (n, 0)):
            assert np.array_equal(r.read(first, count), ref.xfers[first:first + count])
        with pytest.raises(binding.TacosError) as e:
            r.read(n - 1, 2)
        assert e.value.code == binding.TACOS_E_INVAL


def _golden():
    with open(GOLDEN) as f:
        return json.load(f)


@pytest.mark.parametrize("idx", [1, 2, 3])
def test_workloads_1_to_3_bit_exact(idx, stream):
    w = T.workload(idx)
    ref = oracle.synthesize_workload(w)
    g = _golden()[str(idx)]
    assert ref.collective_time_ps == g["collective_time_ps"] and ref.digest == g["digest"]
    with binding.synthesize_workload(w, stream=stream) as r:
        assert_same(r, ref, w.name)
        for i in range(r.num_passes):
            assert r.pass_time_ps(i) == g["pass_time_ps"][i] and r.pass_events(i) == g["pass_events"][i]


def test_workload_4_against_stored_oracle_result(stream):
    """Random 1024-NPU topology, 1.05 M spans.  The oracle needs about a minute for it, so
    the comparison is with the values tests/golden/make_golden.py stored from the oracle:
    time, spans, records, digest and the SHA-256 of the canonical record array."""
    w = T.workload(4)
    g = _golden()["4"]
    with binding.synthesize_workload(w, stream=stream) as r:
        assert r.collective_time_ps == g["collective_time_ps"]
        assert r.num_events == g["n_events"] and r.num_xfers == g["n_xfers"]
        assert r.digest == g["digest"]
        got = r.read()
        assert hashlib.sha256(got.tobytes()).hexdigest() == g["sha256_xfers"]


def test_same_seed_same_digest_and_stream_independence(stream):
    import torch
    topo = T.torus3d(5, 4, 3)
    with gpu(topo, 2, MiB, T.ALL_GATHER, 77, stream) as a:
        side = torch.cuda.Stream()
        with gpu(topo, 2, MiB, T.ALL_GATHER, 77, side.cuda_stream) as b:
            assert a.digest == b.digest and a.collective_time_ps == b.collective_time_ps
            assert np.array_equal(a.read(), b.read())
        with gpu(topo, 2, MiB, T.ALL_GATHER, 78, stream) as c:
            assert c.digest != a.digest


def test_kernel_timing_is_reported(stream):
    topo = T.torus3d(6, 6, 4)
    with gpu(topo, 1, MiB, T.ALL_GATHER, 1, stream, time_kernels=True, launch_mode=1) as r:
        assert r.kernel_launches == r.num_events      # one matching launch per span
        assert 0.0 < r.kernel_ms < r.wall_ms
    with gpu(topo, 1, MiB, T.ALL_GATHER, 1, stream, time_kernels=True, launch_mode=2) as r:
        assert 1 <= r.kernel_launches < r.num_events  # single-workgroup sweeps
        assert 0.0 < r.kernel_ms < r.wall_ms


@pytest.mark.parametrize("name,mk,cpn,coll", SMALL, ids=[c[0] for c in SMALL])
@pytest.mark.parametrize("mode", [1, 2, 4])
def test_explicit_launch_modes_bit_exact(name, mk, cpn, coll, mode, stream):
    """launch_mode 1 (two launches per span, one workgroup sweeping the last stretch of a pass),
    4 (two launches per span to the end) and 2 (one workgroup sweeping many spans with the link
    state in LDS) give the schedule of the oracle, like the automatic mode the other tests use."""
    topo = mk()
    cb = 192 << 10
    ref = cpu(topo, cpn, cb, coll, 5)
    with gpu(topo, cpn, cb, coll, 5, stream, launch_mode=mode) as r:
        assert_same(r, ref, name)


HOMOGENEOUS = [
    ("uniring13", lambda: T.ring(13), 1, T.ALL_GATHER),
    ("biring9_cpn3", lambda: T.ring(9, bidirectional=True), 3, T.ALL_GATHER),
    ("fc70_indeg_over_64", lambda: T.fully_connected(70), 2, T.ALL_GATHER),
    ("mesh5x4_cpn7", lambda: T.mesh2d(5, 4), 7, T.ALL_GATHER),
    ("torus2x3_parallel_links", lambda: T.grid([2, 3], True), 2, T.ALL_GATHER),
    ("mesh6x5_rs", lambda: T.mesh2d(6, 5), 3, T.REDUCE_SCATTER),
    ("torus3x3x3_ar", lambda: T.torus3d(3, 3, 3), 2, T.ALL_REDUCE),
    ("switch12d3_rs", lambda: T.switch_unwound(12, 3), 1, T.REDUCE_SCATTER),
    ("random40_equal_cost_ar", lambda: _equal_cost(T.random_regular_out(40, 3, seed=7)[0]), 2, T.ALL_REDUCE),
    ("torus4x4x4_three_piece_rows", lambda: T.torus3d(4, 4, 4), 300, T.ALL_GATHER),
]


def _equal_cost(topo):
    """The same graph with the paper's default link (0.5 us, 50 GB/s) on every link."""
    return T.Topology(topo.n_npus, topo.row_ptr, topo.col_idx, np.full_like(topo.alpha_ps, 500_000),
                      np.full_like(topo.beta_fs_per_B, 20_000), topo.name + "_equal")


@pytest.mark.parametrize("name,mk,cpn,coll", HOMOGENEOUS, ids=[c[0] for c in HOMOGENEOUS])
def test_homogeneous_ten_one_launch_per_span_bit_exact(name, mk, cpn, coll, stream):
    """launch_mode 3 (links of equal cost: one launch per span on the double-buffered held
    table) gives the oracle's schedule and trace, record by record; so does launch_mode 1 on
    the same input (two launches per span)."""
    topo = mk()
    cb = 192 << 10
    ref = cpu(topo, cpn, cb, coll, 9)
    for mode in (3, 1):
        with gpu(topo, cpn, cb, coll, 9, stream, launch_mode=mode) as r:
            assert_same(r, ref, f"{name} mode {mode}")
            t, m = r.event_trace(r.num_passes - 1)
            assert np.array_equal(t, ref.event_times) and np.array_equal(m, ref.event_matches)


def test_homogeneous_ten_mode_limits_and_errors(stream):
    het = T.grid([3, 2, 3], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000])
    with pytest.raises(binding.TacosError) as e:   # link costs differ
        gpu(het, 1, MiB, T.ALL_GATHER, 0, stream, launch_mode=3)
    assert e.value.code == binding.TACOS_E_INVAL
    topo = T.mesh2d(4, 4)
    for kw in ({"matching": 1}, {"max_events": 3}):
        with pytest.raises(binding.TacosError) as e:
            gpu(topo, 1, MiB, T.ALL_GATHER, 0, stream, launch_mode=3, **kw)
        assert e.value.code == binding.TACOS_E_INVAL
    # not strongly connected: NPU 2 can send but never receives
    broken = T.from_edge_list(3, [(0, 1, 500_000, 20_000), (1, 0, 500_000, 20_000), (2, 0, 500_000, 20_000)])
    with pytest.raises(binding.TacosError) as e:
        gpu(broken, 1, MiB, T.ALL_GATHER, 0, stream, launch_mode=3)
    assert e.value.code == binding.TACOS_E_UNREACHABLE
    # rooted collectives take the path as well
    ring = T.ring(7)
    for coll in (T.BROADCAST, T.REDUCE):
        ref = cpu(ring, 5, MiB, coll, 8, root=3)
        with gpu(ring, 5, MiB, coll, 8, stream, root=3, launch_mode=3) as r:
            assert_same(r, ref, f"rooted {coll}")


def test_both_launch_modes_on_prefix_runs(stream):
    topo = T.torus3d(4, 4, 8)
    ref = cpu(topo, 65, MiB, T.ALL_GATHER, 3, max_events=37)
    for mode in (0, 1, 2):
        with gpu(topo, 65, MiB, T.ALL_GATHER, 3, stream, max_events=37, launch_mode=mode) as r:
            assert_same(r, ref, f"mode {mode}")


def test_small_topology_mode_limits(stream):
    big = T.torus3d(16, 16, 20)  # 30,720 links do not fit one workgroup's LDS
    with pytest.raises(binding.TacosError) as e:
        gpu(big, 1, MiB, T.ALL_GATHER, 0, stream, launch_mode=2, max_events=2)
    assert e.value.code == binding.TACOS_E_INVAL
    with gpu(big, 1, MiB, T.ALL_GATHER, 0, stream, launch_mode=0, max_events=2) as r:  # automatic: per-span
        assert r.num_events == 2


def test_five_piece_rows_full_run(stream):
    """512 NPUs x 72 chunks = 36,864 chunks: rows of 5 one-KiB pieces like the 40,960-NPU
    workload, run to completion (18.8 M transfers, ~6.1 k spans) and compared record by
    record."""
    topo = T.torus3d(8, 8, 8)
    cpn = 72
    ref = cpu(topo, cpn, MiB, T.ALL_GATHER, 31, n_threads=min(16, oracle.max_threads()))
    with gpu(topo, cpn, MiB, T.ALL_GATHER, 31, stream) as r:
        assert r.collective_time_ps == ref.collective_time_ps
        assert r.num_events == ref.n_events and r.num_xfers == ref.n_xfers == 36_864 * 511
        assert r.digest == ref.digest
        t, m = r.event_trace(0)
        assert np.array_equal(t, ref.event_times) and np.array_equal(m, ref.event_matches)
        n = r.num_xfers
        step = 1 << 21
        for first in range(0, n, step):
            cnt = min(step, n - first)
            assert np.array_equal(r.read(first, cnt), ref.xfers[first:first + cnt]), first


def test_workload_5_prefix_bit_exact(stream):
    """40,960-NPU torus in the launch configuration bench.py times: the first 48 TEN spans
    (11.8 M transfers) record by record.  The complete run is compared with the oracle's stored
    result by the next test."""
    w = T.workload(5)
    n_ev = 48
    ref = oracle.synthesize_workload(w, max_events=n_ev, n_threads=min(16, oracle.max_threads()))
    with binding.synthesize_workload(w, stream=stream, max_events=n_ev) as r:
        assert r.collective_time_ps == ref.collective_time_ps == n_ev * 10_985_760
        assert r.num_events == n_ev and r.num_xfers == ref.n_xfers
        assert r.digest == ref.digest
        n = r.num_xfers
        step = 1 << 21
        for first in range(0, n, step):
            cnt = min(step, n - first)
            assert np.array_equal(r.read(first, cnt), ref.xfers[first:first + cnt]), first


def test_workload_5_full_run_against_stored_oracle_result(stream):
    """The complete 40,960-NPU All-Gather (1.68e9 transfers) against what the oracle
    stored in tests/golden/workload5_oracle.json (make_golden.py --with-5, minutes of CPU
    time): collective time, spans, transfers, the digest over every transfer, the per-span
    (time, match count) trace and the first 4096 records."""
    with open(os.path.join(os.path.dirname(GOLDEN), "workload5_oracle.json")) as f:
        g = json.load(f)
    w = T.workload(5)
    with binding.synthesize_workload(w, stream=stream) as r:
        assert r.collective_time_ps == g["collective_time_ps"]
        assert r.num_events == g["n_events"] and r.num_xfers == g["n_xfers"]
        assert r.digest == g["digest"]
        t, m = r.event_trace(0)
        assert hashlib.sha256(t.tobytes() + m.tobytes()).hexdigest() == g["sha256_event_trace"]
        assert hashlib.sha256(r.read(0, 4096).tobytes()).hexdigest() == g["sha256_first_4096_xfers"]
        # the last record of the canonical order ends exactly at the collective time
        last = r.read(r.num_xfers - 1, 1)[0]
        assert int(last["t_ps"]) + 10_985_760 == g["collective_time_ps"]
        # records, not only their digest: 16 windows of 65,536 records spread over the whole
        # schedule (the last one ends it), each against the SHA-256 of the oracle's records
        win = g["windows"]
        assert win["first"] + (len(win["sha256"]) - 1) * win["stride"] + win["block"] == r.num_xfers
        for k, want in enumerate(win["sha256"]):
            got = r.read(win["first"] + k * win["stride"], win["block"])
            assert hashlib.sha256(got.tobytes()).hexdigest() == want, f"window {k}"


def test_workload_5_full_run_postcondition_centric_against_stored_oracle_result(stream):
    """The complete 40,960-NPU All-Gather in Algorithm 1's own order (matching = 1, rows of the
    free links in register planes) against tests/golden/workload5_matching1_oracle.json
    (make_golden.py --with-5 --matching1): time, spans, transfers, digest over every transfer,
    per-span trace and the first 4096 records.  The time equals the ingress lower bound."""
    with open(os.path.join(os.path.dirname(GOLDEN), "workload5_matching1_oracle.json")) as f:
        g = json.load(f)
    w = T.workload(5)
    with binding.synthesize_workload(w, stream=stream, matching=1) as r:
        assert r.collective_time_ps == g["collective_time_ps"] == 6_827 * 10_985_760
        assert r.num_events == g["n_events"] and r.num_xfers == g["n_xfers"]
        assert r.digest == g["digest"]
        t, m = r.event_trace(0)
        assert hashlib.sha256(t.tobytes() + m.tobytes()).hexdigest() == g["sha256_event_trace"]
        assert hashlib.sha256(r.read(0, 4096).tobytes()).hexdigest() == g["sha256_first_4096_xfers"]


@pytest.mark.parametrize("idx", [6, 7])
def test_scalability_workloads_full_run_against_stored_oracle_result(idx, stream):
    """The paper's scalability workloads at full size (All-Reduce on the 200x200 mesh and
    on the 35x35x35 3-D mesh: 3.2e9 / 3.7e9 transfers, a Reduce-Scatter and an All-Gather
    pass) against what the oracle stored in tests/golden/workload<N>_oracle.json
    (make_golden.py --scalability N): collective time, per-pass times and spans, transfers
    and the digest over every transfer.  Also the launches that drop complete destinations
    at full size (most NPUs are complete for the second half of each pass)."""
    with open(os.path.join(os.path.dirname(GOLDEN), f"workload{idx}_oracle.json")) as f:
        g = json.load(f)
    w = T.workload(idx)
    assert w.name == g["name"]
    with binding.synthesize_workload(w, stream=stream) as r:
        assert r.collective_time_ps == g["collective_time_ps"]
        assert r.num_events == g["n_events"] and r.num_xfers == g["n_xfers"]
        assert [r.pass_time_ps(i) for i in range(2)] == g["pass_time_ps"]
        assert [r.pass_events(i) for i in range(2)] == g["pass_events"]
        assert r.digest == g["digest"]


@pytest.mark.parametrize("coll", [T.ALL_GATHER, T.ALL_REDUCE])
def test_lower_cost_link_priority_bit_exact(coll, stream):
    """link_order = cheapest first ('Prioritizing Lower-cost Links') against the oracle
    with the same option, on heterogeneous inputs where the order matters."""
    for topo, cpn in ((T.grid([3, 3, 4], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000]), 3),
                      (T.random_regular_out(64, 4, seed=12)[0], 2),
                      (T.from_edge_list(2, [(0, 1, 10, 0), (0, 1, 1, 0), (1, 0, 1, 0)]), 1)):
        ref = cpu(topo, cpn, 64 << 10, coll, 17, link_order=1)
        with gpu(topo, cpn, 64 << 10, coll, 17, stream, link_order=1) as r:
            assert_same(r, ref, topo.name)
    # the option matters on the torus (coincident events, several idle links per NPU)
    topo = T.grid([3, 3, 4], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000])
    assert cpu(topo, 3, 64 << 10, coll, 17, link_order=1).digest != cpu(topo, 3, 64 << 10, coll, 17).digest


@pytest.mark.parametrize("coll", [T.ALL_GATHER, T.REDUCE_SCATTER])
def test_one_launch_per_span_hands_over_to_the_last_stretch_sweep(coll, stream):
    """Automatic mode on a homogeneous mesh too large for the single-workgroup kernel: one launch
    per span while many destinations are left, then (16 left: the corners and their neighbours)
    the link state is rebuilt from the chunks matched in the last span and one workgroup sweeps
    the rest.  Record by record against the oracle; launch_mode 3 (one launch per span to the
    end) and 4 (two launches per span to the end) give the same digest."""
    topo = T.mesh2d(58, 58)
    ref = cpu(topo, 1, MiB, coll, 12, n_threads=min(16, oracle.max_threads()))
    with gpu(topo, 1, MiB, coll, 12, stream, time_kernels=True) as r:
        assert_same(r, ref, "mesh58x58")
        assert r.kernel_launches == r.num_events  # a launch that sweeps several spans counts once per span
        for mode in (3, 4):
            with gpu(topo, 1, MiB, coll, 12, stream, launch_mode=mode) as q:
                assert q.digest == r.digest and q.collective_time_ps == r.collective_time_ps
                assert q.num_events == r.num_events


@pytest.mark.parametrize("coll", [T.ALL_GATHER, T.REDUCE_SCATTER])
def test_large_mesh_changes_launch_form_twice(coll, stream):
    """Automatic mode on a homogeneous mesh whose two held tables would not fit the Infinity Cache
    (182 x 182: 2 x 170 MB): two launches per span while most destinations are left, one launch
    per span from 2,048 destinations on (the link state becomes the arrivals of the next span),
    one workgroup for the last 16.  Same digest, times and span count as two launches per span
    to the end (launch_mode 4) and as one launch per span from the start (launch_mode 3); the
    full-size workloads 6 and 7 take the same route against the oracle's stored results."""
    topo = T.mesh2d(182, 182)
    with gpu(topo, 1, MiB, coll, 21, stream, time_kernels=True) as r:
        assert r.kernel_launches == r.num_events  # every span counted once, whichever form swept it
        for mode in (4, 3):
            with gpu(topo, 1, MiB, coll, 21, stream, launch_mode=mode) as q:
                assert q.digest == r.digest and q.collective_time_ps == r.collective_time_ps
                assert q.num_events == r.num_events and q.num_xfers == r.num_xfers
                t0, m0 = r.event_trace(0)
                t1, m1 = q.event_trace(0)
                assert np.array_equal(t0, t1) and np.array_equal(m0, m1)


@pytest.mark.parametrize("name,mk", [("mesh64x64", lambda: T.mesh2d(64, 64, 500_000, 20_000)),
                                     ("mesh3d_12", lambda: T.grid([12, 12, 12], False, 500_000, 20_000))])
def test_scalability_shapes_all_reduce_full(name, mk, stream):
    """Scaled-down shapes of the paper's scalability experiment (All-Reduce on a 2D mesh
    and on a 3D mesh without wrap-around; in-degree 2..6), run to completion: Reduce-
    Scatter and All-Gather halves record by record."""
    topo = mk()
    ref = cpu(topo, 1, MiB, T.ALL_REDUCE, 6, n_threads=min(16, oracle.max_threads()))
    with gpu(topo, 1, MiB, T.ALL_REDUCE, 6, stream) as r:
        assert r.collective_time_ps == ref.collective_time_ps and r.digest == ref.digest
        assert [r.pass_time_ps(i) for i in range(2)] == list(ref.pass_time_ps)
        assert [r.pass_events(i) for i in range(2)] == list(ref.pass_events)
        n = r.num_xfers
        assert n == ref.n_xfers
        step = 1 << 21
        for first in range(0, n, step):
            cnt = min(step, n - first)
            assert np.array_equal(r.read(first, cnt), ref.xfers[first:first + cnt]), (name, first)


def _every_link_its_own_cost(n, deg, seed):
    topo = T.random_regular_out(n, deg, seed=seed)[0]
    rng = np.random.default_rng(seed)
    topo.alpha_ps[:] = rng.integers(200_000, 2_000_000, size=topo.n_links)
    topo.beta_fs_per_B[:] = rng.choice([5_000, 10_000, 20_000, 40_000], size=topo.n_links)
    return topo


@pytest.mark.parametrize("n,deg,cpn,coll,matching,link_order,seed", [
    (60, 3, 2, T.ALL_GATHER, 0, 0, 1), (60, 3, 2, T.REDUCE_SCATTER, 0, 0, 2), (90, 4, 1, T.ALL_REDUCE, 1, 0, 4),
    (40, 5, 3, T.ALL_GATHER, 0, 1, 6), (200, 4, 1, T.ALL_REDUCE, 0, 0, 7), (64, 3, 40, T.REDUCE, 1, 0, 9)])
def test_per_span_launches_keep_compact_records_when_every_link_has_its_own_cost(n, deg, cpn, coll, matching,
                                                                                link_order, seed, stream):
    """Links that nearly all cost differently: about one transfer starts per span, and the
    per-span launches keep (link, chunk) records instead of one row of n_links entries per
    span.  Records, per-span traces of forward and reversed passes, link counts; the device
    memory held stays proportional to the transfers."""
    topo = _every_link_its_own_cost(n, deg, seed)
    kw = dict(matching=matching, link_order=link_order, root=3)
    ref = cpu(topo, cpn, MiB, coll, seed, **kw)
    with gpu(topo, cpn, MiB, coll, seed, stream, launch_mode=1, **kw) as r:
        assert_same(r, ref, "own costs")
        t, m = r.event_trace(r.num_passes - 1)
        assert np.array_equal(t, ref.event_times) and np.array_equal(m, ref.event_matches)
        if coll == T.ALL_REDUCE:
            rs = cpu(topo, cpn, MiB, T.REDUCE_SCATTER, seed, **kw)
            t, m = r.event_trace(0)
            assert np.array_equal(t, rs.event_times) and np.array_equal(m, rs.event_matches)
        per_pass = r.num_xfers // r.num_passes
        for ps in range(r.num_passes):
            first = ps * per_pass
            want = np.bincount(ref.xfers["link"][first:first + per_pass], minlength=topo.n_links)
            assert np.array_equal(r.link_counts(ps, topo.n_links), want)
        assert r.device_bytes <= 24 * r.num_xfers + 4096        # 8 B per transfer + 12 B per span
        assert r.device_bytes < r.num_events * topo.n_links * 4  # what dense rows would take


def test_workload_4_prefix_through_the_per_span_launches(stream):
    """The 1,024-NPU heterogeneous workload through two launches per span (compact records),
    first 20,000 spans: record by record against the oracle's prefix."""
    w = T.workload(4)
    t = w.topo
    ref = oracle.synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B, w.chunks_per_npu,
                            w.chunk_bytes, w.collective, w.seed, max_events=20_000,
                            n_threads=min(16, oracle.max_threads()))
    with binding.tacos_synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B, w.chunks_per_npu,
                                  w.chunk_bytes, w.collective, w.seed, stream=stream, launch_mode=1,
                                  max_events=20_000) as r:
        assert_same(r, ref, "workload 4 prefix")
        assert r.device_bytes < 64 << 20


@pytest.mark.parametrize("mode", [1, 4])
@pytest.mark.parametrize("coll", [T.ALL_GATHER, T.REDUCE_SCATTER, T.ALL_REDUCE])
def test_heterogeneous_mesh_with_few_destinations_left(coll, mode, stream):
    """A mesh with different link classes per dimension through the per-span launches:
    the interior completes long before the corners, the host drops complete destinations
    from the launches, and the arrivals are then looked for in the remaining in-lists
    only; spans sit on many distinct times, forward and reversed passes.  With launch_mode 1
    the last stretch (at most 16 destinations left) is swept by one workgroup, many spans per
    launch; with 4 every span keeps its two launches.  Record by record."""
    topo = T.grid([14, 11], False, [300_000, 700_000], [5_000, 20_000])
    ref = cpu(topo, 2, 96 << 10, coll, 23, n_threads=min(16, oracle.max_threads()))
    with gpu(topo, 2, 96 << 10, coll, 23, stream, launch_mode=mode) as r:
        assert_same(r, ref, "hetero mesh 14x11")
        n_pass = 2 if coll == T.ALL_REDUCE else 1
        assert [r.pass_events(i) for i in range(n_pass)] == list(ref.pass_events)[:n_pass]


TAIL = [
    # at most 16 NPUs: the whole pass is swept by the single-workgroup tail launches, 1,024 spans each
    ("biring12_cpn150", lambda: T.grid([12], True, [300_000], [5_000]), 150, T.ALL_GATHER, 96 << 10),
    ("mesh4x4_hetero_cpn200_ar", lambda: T.grid([4, 4], False, [300_000, 700_000], [5_000, 20_000]), 200, T.ALL_REDUCE, 64 << 10),
    ("uniring16_rs_two_piece_rows", lambda: T.ring(16), 700, T.REDUCE_SCATTER, MiB),
    # rows of 3, 5, 6 and 8 pieces (every row width is its own instantiation of the kernel)
    ("biring8_three_piece_rows", lambda: T.grid([8], True), 2500, T.ALL_GATHER, MiB),
    ("mesh3x3_hetero_five_piece_rows", lambda: T.grid([3, 3], False, [300_000, 700_000], [5_000, 20_000]), 4400,
     T.ALL_GATHER, 64 << 10),
    ("torus2x2x3_parallel_links_six_piece_rows_rs", lambda: T.grid([2, 2, 3], True), 3800, T.REDUCE_SCATTER, MiB),
    ("uniring5_eight_piece_rows", lambda: T.ring(5), 13000, T.ALL_GATHER, MiB),
    # larger: two launches per span first, the tail launches take over when 16 destinations are left
    ("mesh9x7_corners_last_ar", lambda: T.mesh2d(9, 7), 40, T.ALL_REDUCE, MiB),
    ("mesh3d_5x4x3_hetero_ag", lambda: T.grid([5, 4, 3], False, [300_000, 500_000, 900_000], [5_000, 10_000, 20_000]), 30,
     T.ALL_GATHER, 256 << 10),
]


@pytest.mark.parametrize("name,mk,cpn,coll,cb", TAIL, ids=[c[0] for c in TAIL])
def test_last_stretch_of_a_pass_in_one_workgroup(name, mk, cpn, coll, cb, stream):
    """launch_mode 1 once at most 16 destinations still miss chunks: one workgroup sweeps the
    remaining spans, many per launch, with the link state in registers and the need rows in LDS;
    it takes over from the two launches per span (or runs the whole pass), hands over from one
    launch to the next, and ends the pass.  Record by record against the oracle, and the same
    digest, times and span counts as launch_mode 4 (two launches for every span); with kernel
    timing one launch is counted per span."""
    topo = mk()
    ref = cpu(topo, cpn, cb, coll, 41, n_threads=min(16, oracle.max_threads()))
    with gpu(topo, cpn, cb, coll, 41, stream, launch_mode=1, time_kernels=True) as r:
        assert_same(r, ref, name)
        assert r.kernel_launches == r.num_events
        with gpu(topo, cpn, cb, coll, 41, stream, launch_mode=4) as q:
            assert q.digest == r.digest and q.collective_time_ps == r.collective_time_ps
            assert q.num_events == r.num_events and q.num_xfers == r.num_xfers


@pytest.mark.parametrize("idx,n_ev", [(6, 40), (7, 40)])
def test_scalability_workloads_prefix_bit_exact(idx, n_ev, stream):
    """Full-size shapes of the paper's scalability experiment (40,000-NPU 2D mesh and
    42,875-NPU 3D mesh): the first spans of the All-Gather pass record by record."""
    w = T.workload(idx)
    t = w.topo
    ref = oracle.synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B, 1, w.chunk_bytes,
                            T.ALL_GATHER, w.seed, max_events=n_ev, n_threads=min(16, oracle.max_threads()))
    with gpu(t, 1, w.chunk_bytes, T.ALL_GATHER, w.seed, stream, max_events=n_ev) as r:
        assert r.collective_time_ps == ref.collective_time_ps and r.num_xfers == ref.n_xfers
        assert r.digest == ref.digest
        n = r.num_xfers
        step = 1 << 21
        for first in range(0, n, step):
            cnt = min(step, n - first)
            assert np.array_equal(r.read(first, cnt), ref.xfers[first:first + cnt]), first


def test_link_counts_match_oracle_records(stream):
    """tacos_result_link_counts (device column sums of the schedule) against a bincount of
    the oracle's records, per pass of an All-Reduce."""
    topo = T.grid([4, 3, 3], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000])
    ref = cpu(topo, 2, MiB, T.ALL_REDUCE, 9)
    n = len(ref.xfers) // 2
    with gpu(topo, 2, MiB, T.ALL_REDUCE, 9, stream) as r:
        for p, part in enumerate((ref.xfers[:n], ref.xfers[n:])):
            want = np.bincount(part["link"].astype(np.int64), minlength=topo.n_links)
            assert np.array_equal(r.link_counts(p, topo.n_links), want.astype(np.uint64))


PAIR_CASES = [
    ("mesh5x4_cpn7", lambda: T.mesh2d(5, 4), 7, T.ALL_GATHER),
    ("biring9_cpn3", lambda: T.ring(9, bidirectional=True), 3, T.ALL_REDUCE),
    ("fc16", lambda: T.fully_connected(16), 2, T.ALL_GATHER),
    ("torus2x3_parallel_links", lambda: T.grid([2, 3], True), 2, T.REDUCE_SCATTER),
    ("hetero_torus", lambda: T.grid([3, 3, 4], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000]), 3, T.ALL_REDUCE),
    ("random40", lambda: T.random_regular_out(40, 3, seed=7)[0], 2, T.ALL_GATHER),
    ("torus4x4x8_c8320", lambda: T.torus3d(4, 4, 8), 65, T.ALL_GATHER),
]


@pytest.mark.parametrize("name,mk,cpn,coll", PAIR_CASES, ids=[c[0] for c in PAIR_CASES])
@pytest.mark.parametrize("link_order", [0, 1])
@pytest.mark.parametrize("launch_mode", [1, 2])
def test_postcondition_centric_matching_bit_exact(name, mk, cpn, coll, link_order, launch_mode, stream):
    """matching = 1 (Algorithm 1 in the order the paper prints it) against the oracle's
    same mode, with random and with cheapest-first holder links, through the per-span
    launches and through the single-workgroup kernel."""
    topo = mk()
    cb = 96 << 10
    kw = dict(max_events=60) if cpn == 65 else {}
    ref = cpu(topo, cpn, cb, coll, 23, matching=1, link_order=link_order, **kw)
    with gpu(topo, cpn, cb, coll, 23, stream, matching=1, link_order=link_order, launch_mode=launch_mode,
             **kw) as r:
        assert_same(r, ref, name)


def test_postcondition_centric_limits(stream):
    fc70 = T.fully_connected(70)  # in-degree 69 > 64
    with pytest.raises(binding.TacosError) as e:
        gpu(fc70, 1, MiB, T.ALL_GATHER, 0, stream, matching=1)
    assert e.value.code == binding.TACOS_E_INVAL


def test_postcondition_centric_workload_5_prefix(stream):
    """Algorithm 1's own order on the 40,960-NPU torus: first 16 spans record by record."""
    w = T.workload(5)
    n_ev = 16
    ref = oracle.synthesize_workload(w, max_events=n_ev, matching=1, n_threads=min(16, oracle.max_threads()))
    with binding.synthesize_workload(w, stream=stream, max_events=n_ev, matching=1) as r:
        assert r.num_xfers == ref.n_xfers and r.digest == ref.digest
        assert np.array_equal(r.read(0, 1 << 20), ref.xfers[:1 << 20])
        assert np.array_equal(r.read(r.num_xfers - (1 << 20), 1 << 20), ref.xfers[-(1 << 20):])


# ---------------------------------------------------------------- best of several seeds

def search(topo, cpn, cb, coll, seeds, stream, **kw):
    return binding.tacos_seed_search(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps,
                                     topo.beta_fs_per_B, cpn, cb, coll, seeds, stream=stream, **kw)


def oracle_times(topo, cpn, cb, coll, seeds, **kw):
    out = [cpu(topo, cpn, cb, coll, int(s), keep_xfers=0, **kw) for s in seeds]
    return (np.array([o.collective_time_ps for o in out], dtype=np.uint64),
            np.array([o.n_events for o in out], dtype=np.uint64))


SEARCH_CASES = [
    ("ring8_ag", lambda: T.ring(8), 1, T.ALL_GATHER),
    ("mesh5x4_ar", lambda: T.mesh2d(5, 4), 3, T.ALL_REDUCE),
    ("hetero_torus_ar", lambda: T.grid([3, 3, 4], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000]), 3, T.ALL_REDUCE),
    ("random40_rs", lambda: T.random_regular_out(40, 3, seed=7)[0], 2, T.REDUCE_SCATTER),
    ("torus4x4x8_c8320_ag", lambda: T.torus3d(4, 4, 8), 65, T.ALL_GATHER),
]


@pytest.mark.parametrize("name,mk,cpn,coll", SEARCH_CASES, ids=[c[0] for c in SEARCH_CASES])
@pytest.mark.parametrize("matching,link_order", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_seed_search_equals_one_oracle_run_per_seed(name, mk, cpn, coll, matching, link_order, stream):
    """Every seed's collective time and span count from the concurrent search are the
    oracle's for that seed; the best index is the first minimum."""
    topo = mk()
    cb = 200 << 10
    seeds = np.arange(100, 100 + (5 if cpn == 65 else 19), dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)
    want_t, want_e = oracle_times(topo, cpn, cb, coll, seeds, matching=matching, link_order=link_order)
    times, events, best = search(topo, cpn, cb, coll, seeds, stream, matching=matching, link_order=link_order)
    assert np.array_equal(times, want_t), name
    assert np.array_equal(events, want_e), name
    assert best == int(np.argmin(want_t))


def test_seed_search_more_passes_than_compute_units(stream):
    """600 seeds of an All-Reduce = 1200 single-workgroup passes in one launch (256 CUs)."""
    topo = T.grid([3, 3], True, [300_000, 700_000], [5_000, 20_000])
    seeds = np.arange(600, dtype=np.uint64)
    want_t, want_e = oracle_times(topo, 2, MiB, T.ALL_REDUCE, seeds)
    times, events, best = search(topo, 2, MiB, T.ALL_REDUCE, seeds, stream)
    assert np.array_equal(times, want_t) and np.array_equal(events, want_e)
    assert best == int(np.argmin(want_t))
    assert len(set(times.tolist())) > 1  # the seeds do differ in quality


def test_seed_search_sequential_path_and_single_run_agree(stream):
    topo = T.random_regular_out(24, 3, seed=5)[0]
    seeds = np.array([7, 7, 1 << 63, 0], dtype=np.uint64)
    a = search(topo, 2, MiB, T.ALL_REDUCE, seeds, stream, launch_mode=1)
    b = search(topo, 2, MiB, T.ALL_REDUCE, seeds, stream, launch_mode=2)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and a[2] == b[2]
    assert a[0][0] == a[0][1]
    with gpu(topo, 2, MiB, T.ALL_REDUCE, int(seeds[a[2]]), stream) as r:
        assert r.collective_time_ps == int(a[0][a[2]]) and r.num_events == int(a[1][a[2]])


def test_seed_search_workload_4_against_stored_oracle_values(stream):
    """Three seeds of the 1024-NPU heterogeneous workload (about a million spans each),
    against values written by tests/golden/make_golden.py from the oracle."""
    with open(os.path.join(os.path.dirname(GOLDEN), "seed_search_oracle.json")) as f:
        g = json.load(f)
    w = T.workload(4)
    seeds = np.array(g["seeds"], dtype=np.uint64)
    times, events, best = binding.seed_search_workload(w, seeds, stream=stream)
    assert times.tolist() == g["collective_time_ps"]
    assert events.tolist() == g["n_events"]
    assert best == int(np.argmin(np.array(g["collective_time_ps"], dtype=np.uint64)))


def test_seed_search_errors_and_degenerate_inputs(stream):
    ring = T.ring(6)
    with pytest.raises(binding.TacosError) as e:
        search(ring, 1, MiB, T.ALL_GATHER, [], stream)
    assert e.value.code == binding.TACOS_E_INVAL
    big = T.torus3d(16, 16, 16)  # 24,576 links do not fit the LDS of one workgroup
    with pytest.raises(binding.TacosError) as e:
        search(big, 1, MiB, T.ALL_GATHER, [1, 2], stream, launch_mode=2)
    assert e.value.code == binding.TACOS_E_INVAL
    one = T.from_edge_list(1, [])
    times, events, best = search(one, 4, MiB, T.ALL_REDUCE, [3, 4, 5], stream)
    assert times.tolist() == [0, 0, 0] and events.tolist() == [0, 0, 0] and best == 0
    broken = T.from_edge_list(3, [(0, 1, 1000, 10), (1, 0, 1000, 10), (0, 2, 1000, 10)])  # 2 cannot send
    with pytest.raises(binding.TacosError) as e:
        search(broken, 1, MiB, T.ALL_GATHER, [1, 2, 3], stream)
    assert e.value.code == binding.TACOS_E_UNREACHABLE


@pytest.mark.parametrize("coll", [T.ALL_GATHER, T.ALL_REDUCE, T.BROADCAST])
def test_seed_search_beyond_one_workgroup_runs_seeds_on_several_streams(coll, stream):
    """Per-span launches (here forced with launch_mode 1; a topology too large for the single-
    workgroup kernel takes them by itself) on a topology small enough to leave the GPU mostly
    idle: the seeds are synthesized whole, several at a time on streams of the library's own
    from several host threads (an All-Reduce additionally sweeps its two passes at once).  Times
    and span counts of the oracle for every seed, and of a single synthesis with each seed; an
    unreachable NPU is reported from whichever thread finds it."""
    topo = T.grid([24, 24], False, [300_000, 700_000], [5_000, 20_000])
    seeds = np.array([11, 12, 13, 14, 15, 16, 17], dtype=np.uint64)
    kw = dict(root=77) if coll == T.BROADCAST else {}
    cpn = 600 if coll == T.BROADCAST else 1
    want_t, want_e = oracle_times(topo, cpn, MiB, coll, seeds, n_threads=min(16, oracle.max_threads()), **kw)
    times, events, best = search(topo, cpn, MiB, coll, seeds, stream, launch_mode=1, **kw)
    assert np.array_equal(times, want_t) and np.array_equal(events, want_e)
    assert best == int(np.argmin(want_t))
    for i in (0, 6):
        with gpu(topo, cpn, MiB, coll, int(seeds[i]), stream, **kw) as r:
            assert r.collective_time_ps == int(times[i]) and r.num_events == int(events[i])
    big = T.mesh2d(58, 58)  # beyond the single-workgroup kernel: the same path in automatic mode
    times, events, best = search(big, 1, MiB, coll if coll != T.BROADCAST else T.ALL_GATHER, seeds[:5], stream)
    for i in (1, 4):
        with gpu(big, 1, MiB, coll if coll != T.BROADCAST else T.ALL_GATHER, int(seeds[i]), stream) as r:
            assert r.collective_time_ps == int(times[i]) and r.num_events == int(events[i])
    src = np.repeat(np.arange(topo.n_npus), np.diff(topo.row_ptr))
    edges = [(int(a), int(b), int(al), int(be)) for a, b, al, be in zip(src, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B)]
    broken = T.from_edge_list(topo.n_npus + 1, edges + [(topo.n_npus, 0, 500_000, 10_000)])  # the new NPU never receives
    if coll != T.BROADCAST:
        with pytest.raises(binding.TacosError) as e:
            search(broken, 1, MiB, coll, seeds, stream, launch_mode=1)
        assert e.value.code == binding.TACOS_E_UNREACHABLE


def test_best_of_seeds_returns_the_winning_schedule(stream):
    w = T.workload(3)
    seeds = np.arange(50, 90, dtype=np.uint64)
    r, seed, times = binding.synthesize_best_of(w, seeds, stream=stream)
    with r:
        assert r.collective_time_ps == int(times.min()) and seed == int(seeds[int(np.argmin(times))])
        ref = oracle.synthesize_workload(T.Workload(w.name, w.topo, w.chunks_per_npu, w.chunk_bytes,
                                                    w.collective, seed))
        assert_same(r, ref, "best of 40 seeds")


# ---------------------------------------------------------------- Broadcast / Reduce

ROOTED = [
    ("ring7_k5", lambda: T.ring(7), 5, 3),
    ("biring10_k1", lambda: T.ring(10, bidirectional=True), 1, 9),
    ("fc12_k40", lambda: T.fully_connected(12), 40, 0),
    ("mesh6x5_k300", lambda: T.mesh2d(6, 5), 300, 14),
    ("hetero_torus_k77", lambda: T.grid([3, 3, 4], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000]), 77, 35),
    ("random50_k9000_two_piece_rows", lambda: T.random_regular_out(50, 3, seed=21)[0], 9000, 17),
    ("switch9d2_k13", lambda: T.switch_unwound(9, 2), 13, 8),
]


@pytest.mark.parametrize("name,mk,k,root", ROOTED, ids=[c[0] for c in ROOTED])
@pytest.mark.parametrize("coll", [T.BROADCAST, T.REDUCE])
@pytest.mark.parametrize("mode", [1, 2])
def test_broadcast_and_reduce_bit_exact(name, mk, k, root, coll, mode, stream):
    """Rooted collectives (the root's k chunks to every NPU; Reduce = the reverse) against
    the oracle, through the per-span launches and the single-workgroup kernel."""
    topo = mk()
    cb = 256 << 10
    ref = cpu(topo, k, cb, coll, 31, root=root)
    with gpu(topo, k, cb, coll, 31, stream, root=root, launch_mode=mode) as r:
        assert_same(r, ref, name)
        assert r.num_passes == 1 and r.num_xfers == k * (topo.n_npus - 1)


@pytest.mark.parametrize("coll", [T.BROADCAST, T.REDUCE])
def test_rooted_collectives_with_both_matching_orders_and_link_orders(coll, stream):
    topo = T.grid([4, 3, 3], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000])
    for matching in (0, 1):
        for link_order in (0, 1):
            ref = cpu(topo, 50, MiB, coll, 8, root=20, matching=matching, link_order=link_order)
            with gpu(topo, 50, MiB, coll, 8, stream, root=20, matching=matching, link_order=link_order) as r:
                assert_same(r, ref, f"matching {matching} link_order {link_order}")


def test_broadcast_on_the_40960_npu_torus(stream):
    """Broadcast of 4,096 chunks from one corner of the 32x32x40 torus, record by record."""
    topo = T.workload(5).topo
    ref = oracle.synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B,
                            64, MiB, T.BROADCAST, 12, root=0, max_events=60, n_threads=min(16, oracle.max_threads()))
    with gpu(topo, 64, MiB, T.BROADCAST, 12, stream, root=0, max_events=60) as r:
        assert_same(r, ref, "prefix of 60 spans")


def test_rooted_seed_search_and_limits(stream):
    topo = T.mesh2d(5, 5)
    seeds = np.arange(30, dtype=np.uint64)
    for coll in (T.BROADCAST, T.REDUCE):
        want_t, want_e = oracle_times(topo, 20, MiB, coll, seeds, root=12)
        times, events, best = search(topo, 20, MiB, coll, seeds, stream, root=12)
        assert np.array_equal(times, want_t) and np.array_equal(events, want_e) and best == int(np.argmin(want_t))
    with pytest.raises(binding.TacosError) as e:
        gpu(topo, 3, MiB, T.BROADCAST, 0, stream, root=25)
    assert e.value.code == binding.TACOS_E_INVAL
    with gpu(T.from_edge_list(1, []), 5, MiB, T.BROADCAST, 0, stream, root=0) as r:
        assert r.num_xfers == 0 and r.collective_time_ps == 0


@pytest.mark.parametrize("coll", [T.ALL_GATHER, T.ALL_REDUCE])
def test_heterogeneous_4096_npu_torus_through_the_per_span_launches(coll, stream):
    """16x16x16 torus with three link classes (24,576 links: too many for the single-workgroup
    kernel): spans at many distinct times, several events at one time, complete destinations
    dropped from the launches.  Times, spans, transfers, digest over all 16.8 M (33.5 M)
    transfers, the per-span trace and the first and last 100,000 records."""
    topo = T.grid([16, 16, 16], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000])
    nt = min(16, oracle.max_threads())
    ref = cpu(topo, 1, MiB, coll, 77, keep_first=0, keep_xfers=100_000, n_threads=nt)
    with gpu(topo, 1, MiB, coll, 77, stream) as r:
        assert r.collective_time_ps == ref.collective_time_ps and r.num_events == ref.n_events
        assert r.num_xfers == ref.n_xfers and r.digest == ref.digest
        if coll == T.ALL_GATHER:
            t, m = r.event_trace(0)
            assert np.array_equal(t, ref.event_times) and np.array_equal(m, ref.event_matches)
            assert np.array_equal(r.read(0, 100_000), ref.xfers)
            tail = cpu(topo, 1, MiB, coll, 77, keep_first=ref.n_xfers - 100_000, keep_xfers=100_000, n_threads=nt)
            assert np.array_equal(r.read(ref.n_xfers - 100_000, 100_000), tail.xfers)


# ---------------------------------------------------------------- more than 65,536 chunks

BIG_ROWS = [
    ("fc12_c70000_9_pieces", lambda: T.fully_connected(12), 5834, T.ALL_GATHER, {}),
    ("torus3x3x2_c131076_17_pieces", lambda: T.torus3d(3, 3, 2), 7282, T.ALL_REDUCE, {}),
    ("hetero_mesh4x4_c262144_32_pieces", lambda: T.grid([4, 4], False, [300_000, 700_000], [5_000, 20_000]), 16384,
     T.ALL_GATHER, dict(max_events=400)),
    ("broadcast_c200001_25_pieces", lambda: T.random_regular_out(20, 3, seed=3)[0], 200_001, T.BROADCAST, dict(root=7, max_events=3000)),
    ("reduce_c65537_9_pieces", lambda: T.mesh2d(4, 3), 65_537, T.REDUCE, dict(root=5)),
    ("fc70_indeg69_c70000_9_pieces", lambda: T.fully_connected(70), 1000, T.ALL_GATHER, dict(link_order=1)),
    # 10 to 15 pieces: the last row widths matched with whole rows in registers; 16: the first streamed one
    ("mesh3x3_c81000_10_pieces", lambda: T.mesh2d(3, 3), 9000, T.ALL_GATHER, {}),
    ("biring8_c88000_11_pieces_rs", lambda: T.ring(8, bidirectional=True), 11000, T.REDUCE_SCATTER, {}),
    ("fc12_c96000_12_pieces", lambda: T.fully_connected(12), 8000, T.ALL_GATHER, dict(link_order=1)),
    ("torus2x5_c100000_13_pieces", lambda: T.grid([2, 5], True), 10000, T.ALL_GATHER, {}),
    ("mesh5x2_c110000_14_pieces", lambda: T.mesh2d(5, 2), 11000, T.ALL_GATHER, {}),
    ("fc8_c120000_15_pieces_ar", lambda: T.fully_connected(8), 15000, T.ALL_REDUCE, {}),
    ("biring6_c126000_16_pieces", lambda: T.ring(6, bidirectional=True), 21000, T.ALL_GATHER, {}),
]


@pytest.mark.parametrize("name,mk,cpn,coll,kw", BIG_ROWS, ids=[c[0] for c in BIG_ROWS])
def test_more_than_65536_chunks_streamed_rows(name, mk, cpn, coll, kw, stream):
    """Rows of 9 to 32 one-KiB pieces: up to 15 pieces a source's whole row is still kept in
    registers, beyond that the source rows are streamed.  Digest over all transfers, times,
    spans, the per-span trace (All-Gather), the first and the last 50,000 records."""
    topo = mk()
    nt = min(16, oracle.max_threads())
    ref = cpu(topo, cpn, MiB, coll, 13, keep_first=0, keep_xfers=50_000, n_threads=nt, **kw)
    with gpu(topo, cpn, MiB, coll, 13, stream, **kw) as r:
        assert r.collective_time_ps == ref.collective_time_ps and r.num_events == ref.n_events, name
        assert r.num_xfers == ref.n_xfers and r.digest == ref.digest, name
        if coll in (T.ALL_GATHER, T.BROADCAST):
            t, m = r.event_trace(0)
            assert np.array_equal(t, ref.event_times) and np.array_equal(m, ref.event_matches)
            n = min(50_000, ref.n_xfers)
            assert np.array_equal(r.read(0, n), ref.xfers[:n])
            tail = cpu(topo, cpn, MiB, coll, 13, keep_first=ref.n_xfers - n, keep_xfers=n, n_threads=nt, **kw)
            assert np.array_equal(r.read(ref.n_xfers - n, n), tail.xfers)


def test_chunk_count_limits(stream):
    ring = T.ring(4)
    with pytest.raises(binding.TacosError) as e:   # 262,148 chunks
        gpu(ring, 65_537, MiB, T.ALL_GATHER, 0, stream)
    assert e.value.code == binding.TACOS_E_INVAL
    with pytest.raises(binding.TacosError) as e:   # the postcondition-centric order keeps rows in registers
        gpu(ring, 16_385, MiB, T.ALL_GATHER, 0, stream, matching=1)
    assert e.value.code == binding.TACOS_E_INVAL
    with pytest.raises(binding.TacosError) as e:   # and so does the single-workgroup kernel
        gpu(ring, 16_385, MiB, T.ALL_GATHER, 0, stream, launch_mode=2)
    assert e.value.code == binding.TACOS_E_INVAL


def test_163840_chunks_on_the_40960_npu_torus_prefix(stream):
    """Four chunks per NPU on the 32x32x40 torus (163,840 chunks, rows of 20 KiB, 839 MB of
    rows): the first 10 spans record by record (2.4 M records)."""
    w = T.workload(5)
    t = w.topo
    nt = min(16, oracle.max_threads())
    ref = oracle.synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B, 4, 256 << 10,
                            T.ALL_GATHER, 21, max_events=10, n_threads=nt)
    with gpu(t, 4, 256 << 10, T.ALL_GATHER, 21, stream, max_events=10) as r:
        assert_same(r, ref, "prefix of 10 spans")
