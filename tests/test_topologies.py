"""Input generators: shapes, ordering and the statistics the workloads state."""
import numpy as np

from paper_2304_05301_amd import topologies as T


def test_workload_shapes():
    w1, w2, w3 = T.workload(1), T.workload(2), T.workload(3)
    assert (w1.topo.n_npus, w1.topo.n_links) == (8, 8)
    assert (w2.topo.n_npus, w2.topo.n_links) == (64, 224)
    assert (w3.topo.n_npus, w3.topo.n_links) == (128, 768)
    for w in (w1, w2, w3):
        t = w.topo
        src = t.link_src
        # CSR rows sorted by (src, dst)
        key = src.astype(np.int64) * t.n_npus + t.col_idx
        assert np.all(np.diff(key) >= 0)
        assert not np.any(src == t.col_idx)
    # mesh corner has in-degree 2
    indeg = np.bincount(w2.topo.col_idx, minlength=64)
    assert indeg.min() == 2 and indeg.max() == 4
    # torus: every NPU has 6 in and 6 out links; per-dimension link parameters
    assert np.all(np.bincount(w3.topo.col_idx, minlength=128) == 6)
    assert sorted(set(w3.topo.beta_fs_per_B.tolist())) == [5_000, 10_000, 20_000]


def test_random_topology_statistics():
    w = T.workload(4)
    t = w.topo
    assert (t.n_npus, t.n_links) == (1024, 6144)
    assert np.all(np.diff(t.row_ptr.astype(np.int64)) == 6)
    assert T.is_strongly_connected(t.n_npus, t.row_ptr, t.col_idx)
    assert set(t.beta_fs_per_B.tolist()) == {40_000, 20_000, 10_000, 5_000}
    assert t.alpha_ps.min() >= 200_000 and t.alpha_ps.max() <= 2_000_000
    for i in range(0, 1024, 97):
        d = t.col_idx[t.row_ptr[i]:t.row_ptr[i + 1]]
        assert len(set(d.tolist())) == 6 and i not in d
    # deterministic
    t2, attempt = T.random_regular_out(1024, 6, seed=3)
    assert np.array_equal(t2.col_idx, t.col_idx) and np.array_equal(t2.alpha_ps, t.alpha_ps)


def test_big_torus_shape():
    t = T.torus3d(32, 32, 40, 500_000, 10_000)
    assert (t.n_npus, t.n_links) == (40_960, 245_760)
    assert np.all(np.bincount(t.col_idx, minlength=t.n_npus) == 6)


def test_switch_unwinding():
    t = T.switch_unwound(4, 3, alpha_ps=700, beta_fs_per_B=10)
    assert t.n_links == 12 and set(t.beta_fs_per_B.tolist()) == {30} and set(t.alpha_ps.tolist()) == {700}
    t = T.switch_unwound(5, 2)
    for i in range(5):
        assert sorted(t.col_idx[t.row_ptr[i]:t.row_ptr[i + 1]].tolist()) == sorted([(i + 1) % 5, (i + 2) % 5])
