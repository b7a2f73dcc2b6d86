"""Are the oracle's pins sharp?  Plant plausible mistakes in COPIES of the oracle source
(textual patches, built to temporary libraries, CPU only) and check that for each one
at least one pin that does not depend on the oracle itself fails: published constants,
closed forms, the independent replaying checker, brute force.  The real oracle is never
modified."""
import ctypes
import os
import subprocess
import tempfile

import numpy as np
import pytest

import checker
import oracle
from paper_2304_05301_amd import topologies as T

SRC = os.path.join(os.path.dirname(oracle.__file__), "tacos_oracle.c")
MiB = 1 << 20

MUTANTS = {
    # name: (text to replace, replacement)
    "philox_wrong_multiplier": ("0xD2511F53u * c0", "0xD2511F57u * c0"),
    "philox_nine_rounds": ("round < 10", "round < 9"),
    "philox_swapped_words": ("c0 = n0; c1 = n1; c2 = n2; c3 = n3;", "c0 = n2; c1 = n1; c2 = n0; c3 = n3;"),
    "cost_drops_alpha": ("unsigned __int128 ps = fs / 1000u + alpha_ps;", "unsigned __int128 ps = fs / 1000u;"),
    "cost_truncates": ("* chunk_bytes + 500u;", "* chunk_bytes;"),
    "source_need_not_hold": ("p += (uint64_t)__builtin_popcountll(hs[w] & ~hd[w] & ~fd[w]);",
                             "p += (uint64_t)__builtin_popcountll(~hd[w] & ~fd[w]);"),
    "inflight_ignored": ("uint64_t cand = hs[w] & ~hd[w] & ~fd[w];", "uint64_t cand = hs[w] & ~hd[w];"),
    "arrival_not_applied_before_matching": ("if (carry[l] != ORC_NONE && free_at[l] == t) {",
                                            "if (carry[l] != ORC_NONE && free_at[l] < t) {"),
    "busy_links_reused": ("if (carry[l] != ORC_NONE) continue;            /* link busy */", ""),
    "kth_off_by_one": ("while (k--) w &= w - 1;", "if (k) k--; while (k--) w &= w - 1;"),
    "next_event_is_latest": ("if (carry[l] != ORC_NONE && free_at[l] < tn) tn = free_at[l];",
                             "if (carry[l] != ORC_NONE && (tn == ORC_INF || free_at[l] > tn)) tn = free_at[l];"),
    "rs_not_time_reversed": ("x.t_ps = T - r->t - cost[r->link];", "x.t_ps = r->t;"),
    "rs_direction_not_reversed": ("rc = ag_pass(n_npus, L, col_idx, src, cost, chunks_per_npu, seed, 1u, max_events,",
                                  "rc = ag_pass(n_npus, L, src, col_idx, cost, chunks_per_npu, seed, 1u, max_events,"),
    "wrong_owner": ("uint64_t c = (uint64_t)i * cpn + j;", "uint64_t c = (uint64_t)j * N + i;"),
    "priority_sorts_descending": ("cost[in_link[k - 1]] > cost[l]", "cost[in_link[k - 1]] < cost[l]"),
    "counter_link_event_swapped": ("uint32_t ctr[4] = { link, event, phase, 0u };", "uint32_t ctr[4] = { event, link, phase, 0u };"),
    "phase_ignored": ("uint32_t ctr[4] = { link, event, phase, 0u };", "uint32_t ctr[4] = { link, event, 0u, 0u };"),
    "seed_halves_swapped": ("uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };",
                            "uint32_t key[2] = { (uint32_t)(seed >> 32), (uint32_t)(seed & 0xFFFFFFFFu) };"),
    "uses_second_philox_word": ("return out[0];", "return out[1];"),
    "kth_from_the_top": ("uint32_t k = draw(seed, l, (uint32_t)event, phase) % (uint32_t)p;",
                         "uint32_t k = (uint32_t)p - 1u - draw(seed, l, (uint32_t)event, phase) % (uint32_t)p;"),
    "ar_halves_overlap": ("    t_off = T;\n", "    t_off = 0;\n"),
    "broadcast_root_ignored": ("held[(size_t)root * W + (j >> 6)] |= 1ull << (j & 63);",
                               "held[(size_t)0 * W + (j >> 6)] |= 1ull << (j & 63);"),
    "broadcast_counts_all_gather_chunks": ("(root == ORC_NONE) ? (uint64_t)N * cpn : (uint64_t)cpn;",
                                           "(uint64_t)N * cpn;"),
    "reduce_not_reversed": ("const int has_rev = collective == ORC_REDUCE_SCATTER || collective == ORC_ALL_REDUCE || collective == ORC_REDUCE;",
                            "const int has_rev = collective == ORC_REDUCE_SCATTER || collective == ORC_ALL_REDUCE;"),
}


class _Res(ctypes.Structure):
    _fields_ = oracle._CResult._fields_


def _build(name):
    text = open(SRC).read()
    old, new = MUTANTS[name]
    assert text.count(old) == 1, f"mutant {name}: pattern occurs {text.count(old)} times"
    d = tempfile.mkdtemp(prefix="orc_mut_")
    c = os.path.join(d, "m.c")
    so = os.path.join(d, "m.so")
    with open(c, "w") as f:
        f.write(text.replace(old, new))
    subprocess.check_call(["gcc", "-O1", "-mpopcnt", "-fopenmp", "-shared", "-fPIC", "-w", "-o", so, c])
    lib = ctypes.CDLL(so)
    lib.orc_synthesize.restype = ctypes.c_int
    lib.orc_synthesize.argtypes = oracle.lib().orc_synthesize.argtypes
    lib.orc_result_free.argtypes = [ctypes.POINTER(oracle._CResult)]
    lib.orc_philox4x32_10.argtypes = [ctypes.c_void_p] * 3
    lib.orc_link_cost.restype = ctypes.c_int
    lib.orc_link_cost.argtypes = oracle.lib().orc_link_cost.argtypes
    return lib


def _run(lib, topo, cpn=1, cb=MiB, coll=0, seed=0, link_order=0, matching=0, root=0):
    res = ctypes.POINTER(oracle._CResult)()
    rp = np.ascontiguousarray(topo.row_ptr, dtype=np.uint32)
    ci = np.ascontiguousarray(topo.col_idx, dtype=np.uint32)
    al = np.ascontiguousarray(topo.alpha_ps, dtype=np.uint64)
    be = np.ascontiguousarray(topo.beta_fs_per_B, dtype=np.uint64)
    rc = lib.orc_synthesize(topo.n_npus, rp.ctypes.data, ci.ctypes.data, al.ctypes.data, be.ctypes.data,
                            cpn, cb, coll, seed, 0, 0, (1 << 64) - 1, 1, link_order, matching, root, ctypes.byref(res))
    if rc != 0:
        raise RuntimeError(f"rc={rc}")
    r = res.contents
    n = int(r.n_stored)
    xf = np.frombuffer((ctypes.c_char * (n * 24)).from_address(r.xfers), dtype=oracle.XFER_DTYPE).copy() \
        if n else np.zeros(0, dtype=oracle.XFER_DTYPE)
    out = (int(r.collective_time_ps), int(r.n_events), xf)
    lib.orc_result_free(res)
    return out


def _pins(lib):
    """A subset of the pins of test_oracle_pins.py, run against `lib`.  Raises on the
    first pin that fails."""
    # Philox known answers
    c = np.array([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], dtype=np.uint32)
    k = np.array([0xa4093822, 0x299f31d0], dtype=np.uint32)
    o = np.zeros(4, dtype=np.uint32)
    lib.orc_philox4x32_10(c.ctypes.data, k.ctypes.data, o.ctypes.data)
    assert [int(x) for x in o] == [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]
    # the selection rule against the published Philox vector (counter 0, key 0)
    two = T.from_edge_list(2, [(0, 1, 1, 0), (1, 0, 1, 0)])
    for cpn in (7, 200):
        xf = _run(lib, two, cpn=cpn, cb=1, seed=0)[2]
        assert (int(xf[0]["link"]), int(xf[0]["chunk"])) == (0, 0x6627E8D5 % cpn)
    # exact replay of the 2-NPU schedule: counter/key layout, forward and reversed phase
    want = checker.two_npu_all_gather(9, 0x0123456789ABCDEF, phase=0)
    xf = _run(lib, two, cpn=9, cb=1, seed=0x0123456789ABCDEF)[2]
    assert [(int(x["t_ps"]), int(x["link"]), int(x["chunk"])) for x in xf] == want
    want1 = checker.two_npu_all_gather(9, 5, phase=1)  # reversed pass: links swap their sources
    xf = _run(lib, two, cpn=9, cb=1, coll=1, seed=5)[2]
    got1 = sorted((9 - int(x["t_ps"]) - 1, int(x["link"]), int(x["chunk"])) for x in xf)
    assert got1 == sorted((t, l, (c + 9) % 18) for (t, l, c) in want1)
    # alpha-beta cost
    v = ctypes.c_uint64(0)
    assert lib.orc_link_cost(500_000, 20_000, MiB, ctypes.byref(v)) and v.value == 21_471_520
    assert lib.orc_link_cost(0, 1500, 1, ctypes.byref(v)) and v.value == 2
    # unidirectional ring: N-1 steps, unique schedule
    ring = T.ring(6)
    Tt, ev, xf = _run(lib, ring)
    assert (Tt, ev, len(xf)) == (5 * 21_471_520, 5, 30)
    for rec in xf:
        assert int(rec["chunk"]) == (int(rec["src"]) - int(rec["t_ps"]) // 21_471_520) % 6
    # fully connected: one step
    Tt, ev, xf = _run(lib, T.fully_connected(5))
    assert ev == 1 and np.array_equal(xf["chunk"], xf["src"])
    # independent checker on heterogeneous inputs, AG and RS
    het = T.grid([3, 2, 3], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000])
    cost = checker.link_costs_ps(het.alpha_ps, het.beta_fs_per_B, 64 << 10)
    Tt, ev, xf = _run(lib, het, cpn=2, cb=64 << 10, seed=3)
    checker.check_all_gather(18, het.link_src, het.link_dst, cost, 2, xf, Tt, check_maximal=True)
    assert Tt >= checker.ingress_lower_bound(18, het.link_dst, cost, 2)
    Tt, ev, xf = _run(lib, het, cpn=1, cb=64 << 10, coll=1, seed=3)
    checker.check_reduce_scatter(18, het.link_src, het.link_dst, cost, 1, xf, Tt)
    rnd = T.random_regular_out(12, 2, seed=4)[0]
    cost = checker.link_costs_ps(rnd.alpha_ps, rnd.beta_fs_per_B, MiB)
    Tt, ev, xf = _run(lib, rnd, coll=1, seed=6)
    checker.check_reduce_scatter(12, rnd.link_src, rnd.link_dst, cost, 1, xf, Tt)
    # All-Reduce = Reduce-Scatter, then All-Gather starting when the Reduce-Scatter ends
    m = T.mesh2d(3, 3)
    cost = checker.link_costs_ps(m.alpha_ps, m.beta_fs_per_B, MiB)
    T_rs = _run(lib, m, coll=1, seed=2)[0]
    T_ar, ev, xf = _run(lib, m, coll=2, seed=2)
    half = len(xf) // 2
    checker.check_reduce_scatter(9, m.link_src, m.link_dst, cost, 1, xf[:half], T_rs)
    checker.check_all_gather(9, m.link_src, m.link_dst, cost, 1, xf[half:], T_ar, check_maximal=True, t0=T_rs)
    # brute-force optimum on a few small digraphs
    for edges in ([(0, 1), (1, 2), (2, 0)], [(0, 1), (1, 0), (1, 2), (2, 1)], [(0, 1), (1, 2), (2, 3), (3, 0), (0, 2)]):
        n = 1 + max(max(e) for e in edges)
        topo = T.from_edge_list(n, [(s, d, 1, 0) for s, d in edges])
        opt = checker.optimal_steps_unit(n, edges)
        Tt, ev, xf = _run(lib, topo, cb=1, seed=1)
        assert opt <= ev <= opt + 1 and Tt == ev
    # Broadcast from a root: pipelined on a one-way ring (N - 2 + k spans for k chunks), one
    # span on a complete graph, valid and maximal on a heterogeneous torus; Reduce = its reverse
    Tt, ev, xf = _run(lib, T.ring(7), cpn=5, coll=3, seed=8, root=3)
    assert (Tt, ev, len(xf)) == (10 * 21_471_520, 10, 30) and set(xf["chunk"].tolist()) == set(range(5))
    assert int(xf[0]["src"]) == 3 and int(xf[0]["t_ps"]) == 0
    Tt, ev, xf = _run(lib, T.fully_connected(6), cpn=1, coll=3, root=4)
    assert ev == 1 and set(xf["src"].tolist()) == {4} and len(xf) == 5
    cost = checker.link_costs_ps(het.alpha_ps, het.beta_fs_per_B, 64 << 10)
    Tt, ev, xf = _run(lib, het, cpn=6, cb=64 << 10, coll=3, seed=3, root=11)
    checker.check_all_gather(18, het.link_src, het.link_dst, cost, 6, xf, Tt, check_maximal=True, root=11)
    Tt, ev, xf = _run(lib, het, cpn=4, cb=64 << 10, coll=4, seed=3, root=7)
    checker.check_reduce_scatter(18, het.link_src, het.link_dst, cost, 4, xf, Tt, root=7)
    # lower-cost-link priority closed form
    par = T.from_edge_list(2, [(0, 1, 10, 0), (0, 1, 1, 0), (1, 0, 1, 0)])
    assert _run(lib, par, cb=1, link_order=1)[0] == 1 and _run(lib, par, cb=1, link_order=0)[0] == 10


def test_the_pins_pass_on_the_real_oracle():
    _pins(oracle.lib())


def _child(name, q):
    try:
        _pins(_build(name))
        q.put("passed")
    except BaseException as e:  # any pin failing is what we want to see
        q.put(f"caught: {type(e).__name__}")


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_mutant(name):
    """Run the pins on the mutant in a child process: a mutant may also never terminate
    (a stalled event loop), which counts as caught."""
    import multiprocessing as mp
    ctx = mp.get_context("fork")
    q = ctx.Queue()
    proc = ctx.Process(target=_child, args=(name, q))
    proc.start()
    proc.join(12)
    if proc.is_alive():
        proc.kill()
        proc.join()
        return  # did not terminate: caught
    if proc.exitcode != 0:
        return  # crashed: caught
    assert q.get(timeout=5).startswith("caught"), f"no pin notices mutant {name}"
