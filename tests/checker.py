"""Independent schedule checker (test infrastructure, pure Python/numpy).

It replays a schedule and asserts what the paper and the mathematics fix for ANY valid
result of the synthesis, whatever the random choices were:

  * every transfer uses a link of the topology between neighbouring NPUs (the paper's
    deadlock-freedom remark) and its (src, dst) are that link's;
  * a transfer is sourced from an NPU that already HOLDS the chunk at its start time;
  * every (destination, chunk) is delivered exactly once and never to the owner;
  * per link the busy intervals [t, t+cost) are disjoint (one chunk per TEN link);
  * at the end every NPU holds all chunks (All-Gather postcondition); collective time
    is the latest arrival;
  * matching is maximal: after the matching of an event no idle link has a chunk its
    source holds and its destination neither holds nor is receiving;
  * transfers start only at event times (0 or an arrival time).

It shares nothing with the oracle or with the HIP path.
"""
from __future__ import annotations

from collections import defaultdict

import numpy as np


def link_costs_ps(alpha_ps, beta_fs_per_B, chunk_bytes):
    """alpha + beta*n in integer ps, beta given in fs/B, rounded to nearest (python ints)."""
    return [int(a) + (int(b) * int(chunk_bytes) + 500) // 1000
            for a, b in zip(alpha_ps, beta_fs_per_B)]


def check_all_gather(n_npus, link_src, link_dst, cost, cpn, xfers, collective_time,
                     check_maximal=True, t0=0, root=None):
    """xfers: structured array (t_ps, src, dst, chunk, link) of ONE All-Gather pass whose
    time origin is t0.  Raises AssertionError on the first violated invariant.
    root given: a Broadcast instead (cpn chunks, all held by the root at the start)."""
    N = int(n_npus)
    C = N * int(cpn) if root is None else int(cpn)
    L = len(link_src)
    t = xfers["t_ps"].astype(object) - t0 if len(xfers) else np.zeros(0, dtype=object)
    t = [int(x) for x in t]
    src = xfers["src"].astype(np.int64)
    dst = xfers["dst"].astype(np.int64)
    chunk = xfers["chunk"].astype(np.int64)
    link = xfers["link"].astype(np.int64)
    n = len(xfers)

    assert n == C * (N - 1), f"expected {C * (N - 1)} transfers, got {n}"
    # canonical order: (t, link) strictly ascending
    for i in range(1, n):
        assert (t[i - 1], link[i - 1]) < (t[i], link[i]), f"records not in (t, link) order at {i}"
    # links of the topology
    assert np.all(link < L) and np.all(link >= 0)
    assert np.array_equal(np.asarray(link_src, dtype=np.int64)[link], src), "src is not the link's source"
    assert np.array_equal(np.asarray(link_dst, dtype=np.int64)[link], dst), "dst is not the link's destination"
    assert np.all(chunk < C) and np.all(chunk >= 0)

    arrive = {}  # (npu, chunk) -> arrival time
    if root is None:
        for i in range(N):
            for j in range(cpn):
                arrive[(i, i * cpn + j)] = 0
    else:
        for j in range(cpn):
            arrive[(int(root), j)] = 0
    order = sorted(range(n), key=lambda i: (t[i], link[i]))
    last_free = [0] * L
    # delivery uniqueness + interval disjointness
    for i in order:
        key = (int(dst[i]), int(chunk[i]))
        assert key not in arrive, f"chunk {key[1]} delivered twice to NPU {key[0]} (or to its owner)"
        arrive[key] = t[i] + cost[link[i]]
        assert t[i] >= last_free[link[i]], f"link {link[i]} carries two chunks at once at t={t[i]}"
        last_free[link[i]] = t[i] + cost[link[i]]
    # source holds the chunk when the transfer starts
    for i in range(n):
        key = (int(src[i]), int(chunk[i]))
        assert key in arrive and arrive[key] <= t[i], \
            f"transfer {i}: NPU {key[0]} sends chunk {key[1]} at {t[i]} before holding it"
    assert len(arrive) == N * C, "All-Gather postcondition not met"
    T = max(arrive.values()) if arrive else 0
    assert int(collective_time) - t0 == T, f"collective time {collective_time} != last arrival {T}"

    # transfers start only at event times
    event_times = {0} | set(arrive.values())
    for i in range(n):
        assert t[i] in event_times, f"transfer {i} starts at {t[i]}, which is no event time"

    if check_maximal:
        in_links = defaultdict(list)
        for l in range(L):
            in_links[int(link_dst[l])].append(l)
        by_link = defaultdict(list)
        for i in range(n):
            by_link[int(link[i])].append((t[i], t[i] + cost[link[i]]))
        recv = defaultdict(list)  # npu -> [(match time, arrival time, chunk)]
        for i in range(n):
            recv[int(dst[i])].append((t[i], t[i] + cost[link[i]], int(chunk[i])))
        have = defaultdict(list)
        for (npu, c), ta in arrive.items():
            have[npu].append((ta, c))
        for te in sorted(event_times):
            if te >= T:
                continue
            held = {npu: {c for (ta, c) in have[npu] if ta <= te} for npu in range(N)}
            for d in range(N):
                blocked = held[d] | {c for (tm, ta, c) in recv[d] if tm <= te < ta}
                for l in in_links[d]:
                    busy = any(a <= te < b for (a, b) in by_link[l])
                    if busy:
                        continue
                    cand = held[int(link_src[l])] - blocked
                    assert not cand, (f"matching not maximal: at t={te} link {l} "
                                      f"({link_src[l]}->{d}) is idle but could carry {sorted(cand)[:4]}")
    return T


def check_reduce_scatter(n_npus, link_src, link_dst, cost, cpn, xfers, collective_time, root=None):
    """Invariants of a Reduce-Scatter schedule obtained by reversal: for every chunk the
    transfers form an in-tree over all NPUs rooted at the owner; an NPU forwards its
    partial sum of chunk c once, and only after everything sent TO it for c has arrived;
    links carry one chunk at a time; the collective ends at the last arrival.
    root given: a Reduce instead (cpn chunks, every one of them owned by the root)."""
    N = int(n_npus)
    C = N * int(cpn) if root is None else int(cpn)

    def owner(c):
        return c // cpn if root is None else int(root)

    n = len(xfers)
    assert n == C * (N - 1)
    t = [int(x) for x in xfers["t_ps"]]
    src = xfers["src"].astype(np.int64)
    dst = xfers["dst"].astype(np.int64)
    chunk = xfers["chunk"].astype(np.int64)
    link = xfers["link"].astype(np.int64)
    for i in range(1, n):
        assert (t[i - 1], link[i - 1]) < (t[i], link[i])
    assert np.array_equal(np.asarray(link_src, dtype=np.int64)[link], src)
    assert np.array_equal(np.asarray(link_dst, dtype=np.int64)[link], dst)
    send_time = {}
    for i in range(n):
        key = (int(src[i]), int(chunk[i]))
        assert key not in send_time, f"NPU {key[0]} sends chunk {key[1]} twice"
        assert key[0] != owner(key[1]), "the owner never sends its own chunk in Reduce-Scatter"
        send_time[key] = t[i]
    assert len(send_time) == C * (N - 1)
    for i in range(n):
        d, c = int(dst[i]), int(chunk[i])
        ta = t[i] + cost[link[i]]
        if d != owner(c):
            assert ta <= send_time[(d, c)], \
                f"NPU {d} forwards chunk {c} at {send_time[(d, c)]} before a contribution arrives at {ta}"
    # every chain ends at the owner: follow parents
    parent = {(int(src[i]), int(chunk[i])): int(dst[i]) for i in range(n)}
    for (s, c), d in parent.items():
        hops = 0
        cur = s
        while cur != owner(c):
            cur = parent[(cur, c)]
            hops += 1
            assert hops <= N
    last_free = defaultdict(int)
    for i in sorted(range(n), key=lambda i: (t[i], link[i])):
        assert t[i] >= last_free[int(link[i])]
        last_free[int(link[i])] = t[i] + cost[link[i]]
    T = max(t[i] + cost[link[i]] for i in range(n)) if n else 0
    assert T == int(collective_time)
    return T


def digest(xfers) -> int:
    """Sum over records of a 64-bit mix of (t, link, chunk), modulo 2^64 (numpy retyping
    of the boundary's digest definition, used to cross-check both implementations)."""
    if len(xfers) == 0:
        return 0
    with np.errstate(over="ignore"):
        t = xfers["t_ps"].astype(np.uint64)
        lc = (xfers["link"].astype(np.uint64) << np.uint64(32)) | xfers["chunk"].astype(np.uint64)
        h = t ^ (lc * np.uint64(0x9E3779B97F4A7C15))
        h ^= h >> np.uint64(33)
        h *= np.uint64(0xFF51AFD7ED558CCD)
        h ^= h >> np.uint64(33)
        h *= np.uint64(0xC4CEB9FE1A85EC53)
        h ^= h >> np.uint64(33)
        return int(np.sum(h, dtype=np.uint64))


# ------------------------------------------------------------------ lower bounds

def ingress_lower_bound(n_npus, link_dst, cost, cpn):
    """Bandwidth term of the paper's 'Ideal': NPU d must receive C-cpn chunks over its
    incoming links; link l can deliver floor(T/cost_l) chunks by time T."""
    N = int(n_npus)
    need = N * cpn - cpn
    best = 0
    by_d = defaultdict(list)
    for l, d in enumerate(link_dst):
        by_d[int(d)].append(int(cost[l]))
    for d in range(N):
        cs = by_d[d]
        if need == 0:
            continue
        assert cs, "NPU without incoming link"
        lo, hi = 0, min(cs) * need
        while lo < hi:
            mid = (lo + hi) // 2
            if sum(mid // c for c in cs) >= need:
                hi = mid
            else:
                lo = mid + 1
        best = max(best, lo)
    return best


def diameter_lower_bound(n_npus, link_src, link_dst, cost):
    """Latency term of the paper's 'Ideal': the largest shortest-path cost between two
    NPUs (Dijkstra from every source)."""
    import heapq
    N = int(n_npus)
    adj = defaultdict(list)
    for l in range(len(link_src)):
        adj[int(link_src[l])].append((int(link_dst[l]), int(cost[l])))
    worst = 0
    for s in range(N):
        dist = {s: 0}
        pq = [(0, s)]
        while pq:
            du, u = heapq.heappop(pq)
            if du > dist.get(u, 1 << 200):
                continue
            for v, c in adj[u]:
                nd = du + c
                if nd < dist.get(v, 1 << 200):
                    dist[v] = nd
                    heapq.heappush(pq, (nd, v))
        assert len(dist) == N
        worst = max(worst, max(dist.values()))
    return worst


# ------------------------------------------------------------------ brute force

def optimal_steps_unit(n_npus, edges):
    """Exact minimum number of spans of an All-Gather (1 chunk per NPU, unit-cost links,
    one chunk per link per span) by breadth-first search over held-state vectors.
    Uses only that holding more chunks is never worse, so per destination only the
    inclusion-maximal receivable sets are expanded."""
    N = n_npus
    full = (1 << N) - 1
    start = tuple(1 << i for i in range(N))
    goal = tuple(full for _ in range(N))
    if start == goal:
        return 0
    in_nb = defaultdict(list)
    for (s, d) in edges:
        in_nb[d].append(s)
    frontier = {start}
    seen = {start}
    steps = 0
    while frontier:
        steps += 1
        nxt = set()
        for st in frontier:
            per_dest = []
            for d in range(N):
                options = {st[d]}
                for s in in_nb[d]:
                    useful = st[s] & ~st[d]
                    new_opts = set()
                    for o in options:
                        new_opts.add(o)
                        b = useful
                        while b:
                            low = b & -b
                            new_opts.add(o | low)
                            b ^= low
                    options = new_opts
                maximal = [o for o in options if not any((o | p) == p and p != o for p in options)]
                per_dest.append(maximal)
            stack = [()]
            for d in range(N):
                stack = [pre + (o,) for pre in stack for o in per_dest[d]]
            for ns in stack:
                if ns == goal:
                    return steps
                if ns not in seen:
                    seen.add(ns)
                    nxt.add(ns)
        frontier = nxt
        assert steps <= N * N, "unreachable"
    raise AssertionError("goal not reachable")


def strongly_connected_digraphs(n):
    """All labelled simple digraphs on n nodes that are strongly connected."""
    pairs = [(i, j) for i in range(n) for j in range(n) if i != j]
    out = []
    for mask in range(1 << len(pairs)):
        edges = [pairs[k] for k in range(len(pairs)) if mask >> k & 1]
        if _strong(n, edges):
            out.append(edges)
    return out


def _strong(n, edges):
    def reach(adj):
        seen = {0}
        st = [0]
        while st:
            u = st.pop()
            for v in adj[u]:
                if v not in seen:
                    seen.add(v)
                    st.append(v)
        return len(seen) == n
    fw = defaultdict(list)
    bw = defaultdict(list)
    for s, d in edges:
        fw[s].append(d)
        bw[d].append(s)
    return reach(fw) and reach(bw)


# ------------------------------------------------------------------ Philox in python

def philox4x32_10(ctr, key):
    """Philox4x32-10 of Salmon et al. (SC'11) on python integers.  Test-side only; it is
    itself checked against the published known-answer vectors before it is used to pin
    the counter/key layout of the deterministic choice."""
    M0, M1, W0, W1, MASK = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85, 0xFFFFFFFF
    c0, c1, c2, c3 = [int(x) & MASK for x in ctr]
    k0, k1 = [int(x) & MASK for x in key]
    for _ in range(10):
        p0, p1 = M0 * c0, M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & MASK, p1 & MASK, ((p0 >> 32) ^ c3 ^ k1) & MASK, p0 & MASK
        k0, k1 = (k0 + W0) & MASK, (k1 + W1) & MASK
    return (c0, c1, c2, c3)


def two_npu_all_gather(cpn, seed, phase=0):
    """Exact expected schedule of the forward pass on the 2-NPU topology with unit-cost
    links 0 -> 1 (id 0) and 1 -> 0 (id 1): every span each link sends the
    (Philox(link, span, phase, 0; seed)[0] mod p)-th smallest of the p chunks its source
    owns and has not sent yet.  Returns [(t, link, chunk)]."""
    key = (seed & 0xFFFFFFFF, seed >> 32)
    left = {0: list(range(0, cpn)), 1: list(range(cpn, 2 * cpn))}  # by link = by source
    out = []
    for span in range(cpn):
        for link in (0, 1):
            cand = left[link]
            r = philox4x32_10((link, span, phase, 0), key)[0]
            c = cand[r % len(cand)]
            cand.remove(c)
            out.append((span, link, c))
    return out


def two_npu_hetero_all_gather(cpn, seed, cost0, cost1):
    """Exact expected forward pass on two NPUs whose links 0 -> 1 (id 0, cost0) and 1 -> 0
    (id 1, cost1) differ in cost, event by event: spans sit on the arrival times, a span in
    which no idle link has anything left to send still counts in the span index (it is the
    second counter word of every later draw), and link l sends the
    (Philox(l, span, 0, 0; seed)[0] mod p)-th smallest of the p chunks its source owns and
    has not sent yet.  Returns ([(t, link, chunk)], collective time, spans, matches per span)."""
    key = (seed & 0xFFFFFFFF, seed >> 32)
    cost = (cost0, cost1)
    left = {0: list(range(0, cpn)), 1: list(range(cpn, 2 * cpn))}
    busy_until = {0: None, 1: None}
    t, span, delivered, out, per_span = 0, 0, 0, [], []
    while True:
        for link in (0, 1):
            if busy_until[link] == t:
                busy_until[link] = None
                delivered += 1
        if delivered == 2 * cpn:
            return out, t, span, per_span
        n = 0
        for link in (0, 1):
            if busy_until[link] is None and left[link]:
                r = philox4x32_10((link, span, 0, 0), key)[0]
                c = left[link][r % len(left[link])]
                left[link].remove(c)
                out.append((t, link, c))
                busy_until[link] = t + cost[link]
                n += 1
        per_span.append(n)
        t = min(v for v in busy_until.values() if v is not None)
        span += 1


def two_npu_parallel_links_pairs(cpn, n_par, seed, phase=0):
    """Exact expected forward pass of the postcondition-centric matching on two NPUs with
    unit-cost links: 0 -> 1 once (link id 0) and 1 -> 0 `n_par` times in parallel (ids
    1 .. n_par).  Every source holds all of its own chunks from the start, so at step s of
    destination d in a span the servable chunks are exactly the ones of the other NPU that d
    has not been sent yet, and every still-free link into d is a holder:
      (r0, r1) = words 0, 1 of Philox(d, span, phase + 2, s; seed);
      chunk = the (r0 mod p)-th smallest servable one; link = the (r1 mod n)-th free link
      into d in ascending link id.
    Returns [(t, link, chunk)] sorted by (t, link)."""
    key = (seed & 0xFFFFFFFF, seed >> 32)
    into = {0: list(range(1, n_par + 1)), 1: [0]}
    left = {0: list(range(cpn, 2 * cpn)), 1: list(range(0, cpn))}  # by destination
    out = []
    span = 0
    while left[0] or left[1]:
        for d in (0, 1):
            free = list(into[d])
            step = 0
            while free and left[d]:
                r = philox4x32_10((d, span, phase + 2, step), key)
                c = left[d][r[0] % len(left[d])]
                link = free[r[1] % len(free)]
                left[d].remove(c)
                free.remove(link)
                out.append((span, link, c))
                step += 1
        span += 1
    return sorted(out)


def alg1_postcondition_centric(n_npus, link_src, link_dst, cost, cpn, seed, phase=0, cheapest_first=False):
    """Second, set-based implementation (python, small inputs) of the postcondition-
    centric matching: per destination, repeatedly draw a servable missing chunk with
    Philox(d, span, phase+2, step)[0] and a free holder link with word [1] (or the
    cheapest).  Returns ([(t, link, chunk)], collective_time).  It is a cross-check of the
    C oracle's word/bit handling, written independently; the pins proper are the
    validity checker, the closed forms and the brute force."""
    N, L = int(n_npus), len(link_src)
    C = N * cpn
    key = (seed & 0xFFFFFFFF, seed >> 32)
    held = [set(range(i * cpn, (i + 1) * cpn)) for i in range(N)]
    inflight = [set() for _ in range(N)]
    carry = [None] * L
    free_at = [0] * L
    in_links = [[l for l in range(L) if link_dst[l] == d] for d in range(N)]
    if cheapest_first:
        in_links = [sorted(ls, key=lambda l: (cost[l], l)) for ls in in_links]
    remaining = N * C - C
    t, span, out = 0, 0, []
    while True:
        for l in range(L):
            if carry[l] is not None and free_at[l] == t:
                d = link_dst[l]
                held[d].add(carry[l]); inflight[d].discard(carry[l]); carry[l] = None; remaining -= 1
        if remaining == 0:
            return sorted(out), t
        new = {}
        for d in range(N):
            free = [l for l in in_links[d] if carry[l] is None]
            step = 0
            while True:
                serv = set()
                for l in free:
                    serv |= held[link_src[l]]
                serv -= held[d]
                serv -= inflight[d]
                if not serv:
                    break
                r = philox4x32_10((d, span, phase + 2, step), key)
                c = sorted(serv)[r[0] % len(serv)]
                holders = [l for l in free if c in held[link_src[l]]]
                l = holders[0] if cheapest_first else holders[r[1] % len(holders)]
                new[l] = c
                inflight[d].add(c)
                free.remove(l)
                step += 1
        for l, c in new.items():
            carry[l] = c; free_at[l] = t + cost[l]; out.append((t, l, c))
        nxt = [free_at[l] for l in range(L) if carry[l] is not None]
        assert nxt, "unreachable"
        t = min(nxt)
        span += 1
