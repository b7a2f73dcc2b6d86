"""Bounded randomized parity sweep: 48 small random workloads from a fixed seed (random
out-regular heterogeneous graphs, rings, meshes, tori, unwound switches, complete graphs;
1..70 chunks per NPU; all five collectives; both matching orders; both link orders; every
launch mode that applies), each compared with the CPU oracle record by record.  Stops at the
first difference.  A second sweep draws 300 arbitrary small digraphs, most of them not strongly
connected: the oracle's error code or its schedule, in every launch mode."""
import numpy as np
import pytest

import oracle
from paper_2304_05301_amd import binding, topologies as T

pytestmark = pytest.mark.gpu
N_CASES = 48


def draw_topology(rng):
    kind = rng.integers(0, 6)
    if kind == 0:
        n = int(rng.integers(4, 90))
        deg = int(rng.integers(2, min(6, n - 1) + 1))
        try:
            return T.random_regular_out(n, deg, seed=int(rng.integers(0, 1 << 30)))[0]
        except RuntimeError:  # no strongly connected graph in the allowed attempts
            return T.ring(n)
    if kind == 1:
        return T.ring(int(rng.integers(2, 40)), bidirectional=bool(rng.integers(0, 2)))
    if kind == 2:
        dims = [int(rng.integers(2, 7)) for _ in range(int(rng.integers(1, 4)))]
        alphas = [int(rng.integers(100_000, 2_000_000)) for _ in dims]
        betas = [int(rng.choice([5_000, 10_000, 20_000, 40_000])) for _ in dims]
        return T.grid(dims, bool(rng.integers(0, 2)), alphas, betas)
    if kind == 3:
        return T.mesh2d(int(rng.integers(2, 9)), int(rng.integers(2, 9)))
    if kind == 4:
        n = int(rng.integers(3, 30))
        return T.switch_unwound(n, int(rng.integers(1, min(5, n - 1) + 1)))
    return T.fully_connected(int(rng.integers(2, 24)))


def test_random_workloads_bit_exact():
    import torch
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(20230405)
    modes_seen = set()
    for case in range(N_CASES):
        topo = draw_topology(rng)
        cpn = int(rng.integers(1, max(1, min(70, 16_000 // topo.n_npus)) + 1))
        cb = int(rng.integers(1, 1 << 22))
        coll = int(rng.integers(0, 5))  # 3, 4: Broadcast / Reduce from / to a random root
        root = int(rng.integers(0, topo.n_npus))
        if coll >= 3:
            cpn = int(rng.integers(1, 2_000))
        seed = int(rng.integers(0, 1 << 62))
        matching = int(rng.integers(0, 2))
        link_order = int(rng.integers(0, 2))
        mode = int(rng.integers(0, 4))
        deg = max(int(np.bincount(topo.col_idx, minlength=topo.n_npus).max()), int(np.diff(topo.row_ptr).max()))
        if matching == 1 and deg > 64:
            matching = 0
        hetero = len(set(zip(topo.alpha_ps.tolist(), topo.beta_fs_per_B.tolist()))) > 1
        if mode == 3 and (hetero or matching == 1):  # one launch per span: equal costs, link-centric
            mode = 1
        if mode == 1 and case % 2 == 1:  # two launches for every span, also for the last stretch of a pass
            mode = 4
        n_chunks = cpn if coll >= 3 else cpn * topo.n_npus
        if hetero and n_chunks * topo.n_npus > 200_000:  # about one span per transfer: bound the oracle's work
            cpn = max(1, 200_000 // (topo.n_npus * (1 if coll >= 3 else topo.n_npus)))
        what = (f"case {case}: {topo.name} N={topo.n_npus} L={topo.n_links} cpn={cpn} coll={coll} matching={matching} "
                f"link_order={link_order} launch_mode={mode} seed={seed} root={root} chunk_bytes={cb}")
        print(what, flush=True)
        kw = dict(matching=matching, link_order=link_order, root=root)
        ref = oracle.synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B,
                                cpn, cb, coll, seed, **kw)
        with binding.tacos_synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B,
                                      cpn, cb, coll, seed, stream=stream, launch_mode=mode, **kw) as r:
            assert r.collective_time_ps == ref.collective_time_ps, what
            assert r.num_events == ref.n_events and r.num_xfers == ref.n_xfers, what
            assert r.digest == ref.digest, what
            assert np.array_equal(r.read(), ref.xfers), what
            t, m = r.event_trace(r.num_passes - 1)
            assert np.array_equal(t, ref.event_times) and np.array_equal(m, ref.event_matches), what
        modes_seen.add(mode)
    assert modes_seen == {0, 1, 2, 3, 4}


N_ODD_CASES = 300


def test_random_odd_inputs_agree_with_the_oracle():
    """Arbitrary small random digraphs from a fixed seed: often not strongly connected, with
    parallel links and NPUs that nothing reaches or that reach nothing; all five collectives,
    both matching orders, both link orders, every launch mode that applies.  The library gives
    the oracle's error code (postconditions left and nothing in flight) or, where the collective
    can be completed (a Broadcast needs its root to reach everyone, no more), the oracle's
    schedule record by record."""
    import torch
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(405301)
    n_feasible = n_errors = 0
    for case in range(N_ODD_CASES):
        n = int(rng.integers(2, 12))
        hetero = bool(rng.integers(0, 2))
        edges = []
        for _ in range(int(rng.integers(1, 3 * n))):
            a, b = int(rng.integers(0, n)), int(rng.integers(0, n))
            if a == b:
                continue
            cost = (int(rng.integers(1, 2_000_000)), int(rng.choice([5_000, 10_000, 20_000]))) if hetero else (500_000, 10_000)
            edges.append((a, b) + cost)
        if rng.integers(0, 2):  # a ring with a few links missing: many of these can be completed
            edges += [(i, (i + 1) % n, 500_000, 10_000) for i in range(n) if rng.integers(0, 12) != 0]
        if not edges:
            continue
        topo = T.from_edge_list(n, edges)
        cpn, coll, root = int(rng.integers(1, 40)), int(rng.integers(0, 5)), int(rng.integers(0, n))
        seed, cb = int(rng.integers(0, 1 << 62)), int(rng.integers(1, 1 << 22))
        kw = dict(matching=int(rng.integers(0, 2)), link_order=int(rng.integers(0, 2)), root=root)
        equal_costs = len(set(zip(topo.alpha_ps.tolist(), topo.beta_fs_per_B.tolist()))) == 1
        try:
            ref, ref_code = oracle.synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B,
                                              cpn, cb, coll, seed, **kw), 0
        except oracle.OracleError as e:
            ref, ref_code = None, e.code
        for mode in (0, 1, 2, 3, 4):
            if mode == 3 and (not equal_costs or kw["matching"] == 1):
                continue
            what = f"case {case}: n={n} edges={edges} cpn={cpn} coll={coll} seed={seed} chunk_bytes={cb} {kw} launch_mode={mode}"
            try:
                r = binding.tacos_synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B,
                                             cpn, cb, coll, seed, stream=stream, launch_mode=mode, **kw)
            except binding.TacosError as e:
                assert e.code == ref_code, what
                continue
            with r:
                assert ref_code == 0, what
                assert r.collective_time_ps == ref.collective_time_ps and r.num_events == ref.n_events, what
                assert r.num_xfers == ref.n_xfers and r.digest == ref.digest, what
                assert np.array_equal(r.read(), ref.xfers), what
        n_feasible += ref_code == 0
        n_errors += ref_code != 0
    assert n_feasible >= 50 and n_errors >= 50  # the sweep exercises both outcomes
