"""Seeded synthetic input generators: topologies in CSR form with per-link alpha/beta.

This module builds INPUTS only.  It holds none of the synthesis arithmetic (no link
cost, no matching, no random choice of chunks) and imports neither the HIP binding
nor the CPU oracle, so that both can be fed from it.

Conventions (shared by every generator):
  * a topology is a directed multigraph in CSR form by SOURCE NPU; the LINK ID of a
    link is its index in ``col_idx``;
  * inside one CSR row the links are ordered by destination, ties (parallel links)
    by generation order;
  * ``alpha_ps`` is the link latency in integer picoseconds, ``beta_fs_per_B`` the
    reciprocal bandwidth in integer femtoseconds per byte (50 GB/s -> 20000), the two
    terms of the alpha-beta link model of the paper's section on heterogeneous
    networks;
  * NPU numbering: 2D mesh ``y*X + x``; 3D torus/mesh ``z*X*Y + y*X + x``.

The topology families are those of the paper's table of evaluated topologies (ring,
fully connected, 2D/3D torus, 2D mesh, 3D "hypercube" = 3D mesh without wrap-around,
switch unwound to point-to-point links); the paper's default link is alpha = 0.5 us,
1/beta = 50 GB/s.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterable, List, Sequence, Tuple

import numpy as np

ALL_GATHER = 0
REDUCE_SCATTER = 1
ALL_REDUCE = 2
BROADCAST = 3   # from a root NPU: chunks_per_npu chunks, all held by the root at the start
REDUCE = 4      # to a root NPU: the reverse of Broadcast


def gbps_to_beta_fs_per_B(gb_per_s: float) -> int:
    """Reciprocal bandwidth in fs/byte for a bandwidth in GB/s (1 GB = 1e9 bytes)."""
    beta = 1.0e6 / float(gb_per_s)
    ibeta = int(round(beta))
    if abs(beta - ibeta) > 1e-9:
        raise ValueError(f"{gb_per_s} GB/s is not an integer number of fs/byte")
    return ibeta


def us_to_ps(us: float) -> int:
    ps = float(us) * 1.0e6
    ips = int(round(ps))
    if abs(ps - ips) > 1e-6:
        raise ValueError(f"{us} us is not an integer number of ps")
    return ips


@dataclass(frozen=True)
class Topology:
    """Directed multigraph in CSR-by-source form with per-link alpha/beta."""

    n_npus: int
    row_ptr: np.ndarray        # uint32 [N+1]
    col_idx: np.ndarray        # uint32 [L]  destination of link id l
    alpha_ps: np.ndarray       # uint64 [L]
    beta_fs_per_B: np.ndarray  # uint64 [L]
    name: str = ""

    @property
    def n_links(self) -> int:
        return int(self.col_idx.shape[0])

    @property
    def link_src(self) -> np.ndarray:
        """uint32 [L]: source NPU of every link id (CSR row expansion)."""
        deg = np.diff(self.row_ptr.astype(np.int64))
        return np.repeat(np.arange(self.n_npus, dtype=np.uint32), deg)

    @property
    def link_dst(self) -> np.ndarray:
        return self.col_idx


def from_edge_list(n_npus: int,
                   edges: Iterable[Tuple[int, int, int, int]],
                   name: str = "") -> Topology:
    """Build a Topology from (src, dst, alpha_ps, beta_fs_per_B) tuples.

    Links are sorted by (src, dst); parallel links keep their generation order
    (the sort is stable)."""
    edges = list(edges)
    src = np.array([e[0] for e in edges], dtype=np.int64)
    dst = np.array([e[1] for e in edges], dtype=np.int64)
    alpha = np.array([e[2] for e in edges], dtype=np.uint64)
    beta = np.array([e[3] for e in edges], dtype=np.uint64)
    order = np.lexsort((dst, src))  # stable: primary src, secondary dst
    src, dst, alpha, beta = src[order], dst[order], alpha[order], beta[order]
    counts = np.bincount(src, minlength=n_npus) if len(src) else np.zeros(n_npus, dtype=np.int64)
    row_ptr = np.zeros(n_npus + 1, dtype=np.uint32)
    row_ptr[1:] = np.cumsum(counts)
    return Topology(
        n_npus=int(n_npus),
        row_ptr=row_ptr,
        col_idx=dst.astype(np.uint32),
        alpha_ps=alpha,
        beta_fs_per_B=beta,
        name=name,
    )


# --------------------------------------------------------------------------- families

def ring(n: int, alpha_ps: int = 500_000, beta_fs_per_B: int = 20_000,
         bidirectional: bool = False) -> Topology:
    edges = []
    for i in range(n):
        if n > 1:
            edges.append((i, (i + 1) % n, alpha_ps, beta_fs_per_B))
            if bidirectional:
                edges.append((i, (i - 1) % n, alpha_ps, beta_fs_per_B))
    return from_edge_list(n, edges, name=f"{'bi' if bidirectional else 'uni'}ring{n}")


def fully_connected(n: int, alpha_ps: int = 500_000, beta_fs_per_B: int = 20_000) -> Topology:
    edges = [(i, j, alpha_ps, beta_fs_per_B) for i in range(n) for j in range(n) if i != j]
    return from_edge_list(n, edges, name=f"fc{n}")


def grid(dims: Sequence[int], wrap: bool,
         alpha_ps: Sequence[int] | int = 500_000,
         beta_fs_per_B: Sequence[int] | int = 20_000) -> Topology:
    """k-dimensional mesh (wrap=False) or torus (wrap=True), links to +-1 in every
    dimension, one (alpha, beta) per dimension.  Dimension 0 is the fastest-varying
    NPU coordinate.  A wrapped dimension of size 2 yields two parallel links per
    direction pair (ids distinct); a dimension of size 1 yields none."""
    dims = [int(d) for d in dims]
    nd = len(dims)
    if isinstance(alpha_ps, int):
        alpha_ps = [alpha_ps] * nd
    if isinstance(beta_fs_per_B, int):
        beta_fs_per_B = [beta_fs_per_B] * nd
    n = int(np.prod(dims))
    ids = np.arange(n, dtype=np.int64)
    coords = []
    rem = ids.copy()
    for d in dims:
        coords.append(rem % d)
        rem //= d
    strides = [int(np.prod(dims[:k])) for k in range(nd)]
    srcs, dsts, als, bes = [], [], [], []
    for k in range(nd):
        if dims[k] == 1:
            continue
        for step in (+1, -1):
            c = coords[k] + step
            if wrap:
                ok = np.ones(n, dtype=bool)
                c = c % dims[k]
            else:
                ok = (c >= 0) & (c < dims[k])
            dst = ids + (c - coords[k]) * strides[k]
            srcs.append(ids[ok])
            dsts.append(dst[ok])
            als.append(np.full(int(ok.sum()), alpha_ps[k], dtype=np.int64))
            bes.append(np.full(int(ok.sum()), beta_fs_per_B[k], dtype=np.int64))
    if srcs:
        src = np.concatenate(srcs)
        dst = np.concatenate(dsts)
        al = np.concatenate(als)
        be = np.concatenate(bes)
    else:
        src = dst = al = be = np.zeros(0, dtype=np.int64)
    order = np.lexsort((dst, src))  # stable
    src, dst, al, be = src[order], dst[order], al[order], be[order]
    row_ptr = np.zeros(n + 1, dtype=np.uint32)
    row_ptr[1:] = np.cumsum(np.bincount(src, minlength=n))
    kind = "torus" if wrap else "mesh"
    return Topology(n, row_ptr, dst.astype(np.uint32), al.astype(np.uint64),
                    be.astype(np.uint64), name=f"{kind}{'x'.join(map(str, dims))}")


def mesh2d(x: int, y: int, alpha_ps: int = 500_000, beta_fs_per_B: int = 10_000) -> Topology:
    return grid([x, y], wrap=False, alpha_ps=alpha_ps, beta_fs_per_B=beta_fs_per_B)


def torus3d(x: int, y: int, z: int, alpha_ps=500_000, beta_fs_per_B=10_000) -> Topology:
    return grid([x, y, z], wrap=True, alpha_ps=alpha_ps, beta_fs_per_B=beta_fs_per_B)


def switch_unwound(n: int, degree: int, alpha_ps: int = 500_000,
                   beta_fs_per_B: int = 20_000) -> Topology:
    """An N-port switch unwound with degree d (paper, section on switch-based
    networks): NPU i gets d outgoing links to i+1 .. i+d (mod N); alpha is kept and
    beta is multiplied by d because the port bandwidth is shared."""
    if not (1 <= degree <= max(1, n - 1)):
        raise ValueError("degree must be in 1..N-1")
    edges = []
    for i in range(n):
        for k in range(1, degree + 1):
            if n > 1:
                edges.append((i, (i + k) % n, alpha_ps, beta_fs_per_B * degree))
    return from_edge_list(n, edges, name=f"switch{n}d{degree}")


# ------------------------------------------------------------------ random asymmetric

_M64 = (1 << 64) - 1


class SplitMix64:
    """Public-domain SplitMix64 sequence generator (input generation only)."""

    def __init__(self, state: int):
        self.state = state & _M64

    def next(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & _M64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
        return z ^ (z >> 31)


def is_strongly_connected(n: int, row_ptr: np.ndarray, col_idx: np.ndarray) -> bool:
    """Forward and backward reachability from NPU 0 (iterative DFS)."""
    if n <= 1:
        return True
    src = np.repeat(np.arange(n, dtype=np.int64), np.diff(row_ptr.astype(np.int64)))
    dst = col_idx.astype(np.int64)

    def reach(a: np.ndarray, b: np.ndarray) -> bool:
        order = np.argsort(a, kind="stable")
        aa, bb = a[order], b[order]
        ptr = np.zeros(n + 1, dtype=np.int64)
        ptr[1:] = np.cumsum(np.bincount(aa, minlength=n))
        seen = np.zeros(n, dtype=bool)
        seen[0] = True
        stack = [0]
        cnt = 1
        while stack:
            u = stack.pop()
            for v in bb[ptr[u]:ptr[u + 1]]:
                if not seen[v]:
                    seen[v] = True
                    cnt += 1
                    stack.append(int(v))
        return cnt == n

    return reach(src, dst) and reach(dst, src)


def random_regular_out(n: int, out_degree: int, seed: int,
                       max_attempts: int = 1000) -> Tuple[Topology, int]:
    """Random asymmetric topology: every NPU has ``out_degree`` links to uniformly
    random distinct destinations; per-link bandwidth uniform in {25,50,100,200} GB/s,
    alpha uniform in [0.2, 2] us (integer ps).  The graph of the first attempt that
    is strongly connected is returned together with that attempt number.

    Draw order per attempt (SplitMix64 seeded with seed*0x100000001B3 + attempt):
    for NPU i = 0..n-1: destinations ``r mod n`` (rejecting i and repeats) until
    out_degree are found; then, for those links in draw order, one draw for beta
    and one for alpha."""
    beta_tab = (40_000, 20_000, 10_000, 5_000)  # 25, 50, 100, 200 GB/s in fs/B
    if out_degree > n - 1:
        raise ValueError("out_degree must be < n")
    for attempt in range(max_attempts):
        rng = SplitMix64((seed * 0x100000001B3 + attempt) & _M64)
        edges: List[Tuple[int, int, int, int]] = []
        for i in range(n):
            dsts: List[int] = []
            while len(dsts) < out_degree:
                d = rng.next() % n
                if d == i or d in dsts:
                    continue
                dsts.append(d)
            for d in dsts:
                beta = beta_tab[rng.next() & 3]
                alpha = 200_000 + rng.next() % 1_800_001
                edges.append((i, d, alpha, beta))
        topo = from_edge_list(n, edges, name=f"random{n}k{out_degree}s{seed}a{attempt}")
        if is_strongly_connected(n, topo.row_ptr, topo.col_idx):
            return topo, attempt
    raise RuntimeError("no strongly connected graph found")


# -------------------------------------------------------------------- named workloads

@dataclass(frozen=True)
class Workload:
    name: str
    topo: Topology
    chunks_per_npu: int
    chunk_bytes: int
    collective: int
    seed: int


def workload(idx: int) -> Workload:
    """The benchmark workloads (1-based), all synthetic and seeded.

    1: All-Gather, 8-NPU unidirectional ring, 0.5 us / 50 GB/s, 1 x 1 MiB, seed 0
    2: All-Gather, 8x8 2D mesh, 0.5 us / 100 GB/s, 4 x 256 KiB per NPU, seed 1
    3: All-Reduce, heterogeneous 4x4x8 3D torus (X 200 GB/s 0.3 us, Y 100 GB/s
       0.5 us, Z 50 GB/s 1 us), 4 x 1 MiB per NPU, seed 2
    4: All-Gather, random asymmetric 1024 NPUs, out-degree 6, 1 x 4 MiB, seed 3
    5: All-Gather, 32x32x40 3D torus, 0.5 us / 100 GB/s, 1 x 1 MiB, seed 4
    6: All-Reduce, 200x200 2D mesh (40,000 NPUs), 0.5 us / 50 GB/s, 1 x 1 MiB, seed 6
    7: All-Reduce, 35x35x35 3D mesh (42,875 NPUs), 0.5 us / 50 GB/s, 1 x 1 MiB, seed 7
    (6 and 7 are the shapes of the paper's scalability experiment.)
    """
    MiB = 1 << 20
    if idx == 1:
        return Workload("ring8_ag", ring(8, 500_000, 20_000), 1, MiB, ALL_GATHER, 0)
    if idx == 2:
        return Workload("mesh8x8_ag", mesh2d(8, 8, 500_000, 10_000), 4, 256 << 10, ALL_GATHER, 1)
    if idx == 3:
        t = grid([4, 4, 8], wrap=True, alpha_ps=[300_000, 500_000, 1_000_000],
                 beta_fs_per_B=[5_000, 10_000, 20_000])
        return Workload("torus4x4x8_hetero_ar", t, 4, MiB, ALL_REDUCE, 2)
    if idx == 4:
        t, _ = random_regular_out(1024, 6, seed=3)
        return Workload("random1024_ag", t, 1, 4 * MiB, ALL_GATHER, 3)
    if idx == 5:
        return Workload("torus32x32x40_ag", torus3d(32, 32, 40, 500_000, 10_000), 1, MiB,
                        ALL_GATHER, 4)
    if idx == 6:
        # the paper's scalability study: All-Reduce on an asymmetric homogeneous 2D mesh
        # of about 40K NPUs, the paper's default link (0.5 us, 50 GB/s)
        return Workload("mesh200x200_ar", mesh2d(200, 200, 500_000, 20_000), 1, MiB, ALL_REDUCE, 6)
    if idx == 7:
        # ... and on a 3D "hypercube" (3D mesh without wrap-around) of about 43K NPUs
        return Workload("mesh35x35x35_ar", grid([35, 35, 35], False, 500_000, 20_000), 1, MiB,
                        ALL_REDUCE, 7)
    raise ValueError("workload index must be 1..7")
