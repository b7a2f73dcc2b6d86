"""One-off randomized parity sweep (not collected by pytest).

    python tests/fuzz_parity.py [--cases 400] [--seed 1]

Draws small random workloads (random out-regular heterogeneous graphs, rings, meshes, tori,
unwound switches; 1..70 chunks per NPU; all five collectives; both matching orders; both
link orders; every launch mode) and compares the GPU schedule with the CPU oracle record
by record.  Prints one line per case and stops at the first difference."""
import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2304_05301_amd import binding, topologies as T  # noqa: E402


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cases", type=int, default=400)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--max-chunks", type=int, default=16000,
                    help="upper limit of N * chunks_per_npu (rows of up to ceil(max/8192) one-KiB pieces)")
    ap.add_argument("--min-chunks", type=int, default=0,
                    help="lower limit of the chunk count (above 65536: the streamed-row kernel)")
    args = ap.parse_args()
    import torch
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(args.seed)
    for case in range(args.cases):
        topo = draw_topology(rng)
        max_cpn = max(1, min(700 if args.min_chunks == 0 else 1 << 30, args.max_chunks // topo.n_npus))
        min_cpn = min(max_cpn, -(-args.min_chunks // topo.n_npus) if args.min_chunks else 1)
        cpn = int(rng.integers(min_cpn, max_cpn + 1))
        cb = int(rng.integers(1, 1 << 22))
        coll = int(rng.integers(0, 5))  # 3, 4: Broadcast / Reduce with a random root
        root = int(rng.integers(0, topo.n_npus))
        if coll >= 3:
            cpn = int(rng.integers(max(1, args.min_chunks), max(2, args.max_chunks)))
        seed = int(rng.integers(0, 1 << 62))
        matching = int(rng.integers(0, 2))
        link_order = int(rng.integers(0, 2))
        mode = int(rng.integers(0, 3))
        n_chunks = cpn if coll >= 3 else cpn * topo.n_npus
        if mode == 2 and n_chunks > 16384:  # the single-workgroup kernel takes rows of up to two pieces
            mode = 0
        if n_chunks > 65536:  # streamed rows: link-centric matching only
            matching = 0
        deg_in = np.bincount(topo.col_idx, minlength=topo.n_npus).max()
        deg_out = np.diff(topo.row_ptr).max()
        if matching == 1 and max(deg_in, deg_out) > 64:
            matching = 0
        # heterogeneous link costs: about one span per transfer, and the oracle walks every
        # destination in every span -- keep its work bounded
        hetero = len(set(zip(topo.alpha_ps.tolist(), topo.beta_fs_per_B.tolist()))) > 1
        if hetero and n_chunks * topo.n_npus > 300_000:
            cpn = max(1, 300_000 // (topo.n_npus * (1 if coll >= 3 else topo.n_npus)))
            n_chunks = cpn if coll >= 3 else cpn * topo.n_npus
        print(f"case {case}: {topo.name} N={topo.n_npus} L={topo.n_links} cpn={cpn} coll={coll} matching={matching} "
              f"link_order={link_order} launch_mode={mode} ...", flush=True)
        kw = dict(matching=matching, link_order=link_order, root=root)
        ref = oracle.synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B,
                                cpn, cb, coll, seed, **kw)
        r = binding.tacos_synthesize(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B,
                                     cpn, cb, coll, seed, stream=stream, launch_mode=mode, **kw)
        got = r.read()
        ok = (r.collective_time_ps == ref.collective_time_ps and r.num_events == ref.n_events and
              r.num_xfers == ref.n_xfers and r.digest == ref.digest and np.array_equal(got, ref.xfers))
        print(f"case {case}: {topo.name} N={topo.n_npus} L={topo.n_links} cpn={cpn} coll={coll} matching={matching} "
              f"link_order={link_order} launch_mode={mode} spans={ref.n_events} xfers={ref.n_xfers} "
              f"{'ok' if ok else 'MISMATCH'}", flush=True)
        r.free()
        if not ok:
            sys.exit(1)
    print("FUZZ PARITY: PASS", flush=True)


if __name__ == "__main__":
    main()
