"""tacos_link_costs_static (the entry point that allocates no device memory) against
tacos_link_costs, through the C ABI: same costs and same error codes, on calls in a row
that share the library's static device array (a large input, then smaller ones, then an
overflowing one, then a good one again)."""
import numpy as np
import pytest

from paper_2304_05301_amd import binding, topologies as T

pytestmark = pytest.mark.gpu


def _both(topo, chunk_bytes):
    args = (topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps, topo.beta_fs_per_B, chunk_bytes)
    return binding.tacos_link_costs_static(*args), binding.tacos_link_costs(*args)


def test_static_link_costs_equal_allocating_entry_point_on_consecutive_calls():
    big = T.workload(5).topo                       # 245,760 links: most of the static array
    het = T.workload(4).topo                       # 6,144 links, every one its own alpha
    small = T.grid([3, 2, 3], True, [300_000, 500_000, 1_000_000], [5_000, 10_000, 20_000])
    for topo, cb in ((big, 1 << 20), (het, 4 << 20), (small, 12_345), (het, 1), (big, 1 << 40)):
        got, want = _both(topo, cb)
        assert got.dtype == np.uint64 and got.shape == (topo.n_links,)
        assert np.array_equal(got, want), (topo.name, cb)
        # and the alpha-beta model itself, in python integers
        exp = [int(a) + (int(b) * cb + 500) // 1000 for a, b in zip(topo.alpha_ps[:64], topo.beta_fs_per_B[:64])]
        assert got[:64].tolist() == exp


def test_static_link_costs_overflow_flag_is_cleared_between_calls():
    topo = T.mesh2d(4, 4)
    huge = T.from_edge_list(2, [(0, 1, 0, (1 << 64) - 1), (1, 0, 5, 7)])
    for f in (binding.tacos_link_costs_static, binding.tacos_link_costs):
        with pytest.raises(binding.TacosError) as ei:
            f(huge.n_npus, huge.row_ptr, huge.col_idx, huge.alpha_ps, huge.beta_fs_per_B, (1 << 64) - 1)
        assert ei.value.code == binding.TACOS_E_OVERFLOW
    got, want = _both(topo, 1 << 20)               # the flag of the failed call must not stick
    assert np.array_equal(got, want)


def test_static_link_costs_rejects_more_links_than_the_static_array_holds():
    n = 262_144 + 2
    # a one-way ring with one link too many for the array; nothing is launched
    topo = T.ring(n)
    assert topo.n_links == n
    with pytest.raises(binding.TacosError) as ei:
        binding.tacos_link_costs_static(topo.n_npus, topo.row_ptr, topo.col_idx, topo.alpha_ps,
                                        topo.beta_fs_per_B, 1 << 20)
    assert ei.value.code == binding.TACOS_E_INVAL and "TACOS_STATIC_MAX_LINKS" in str(ei.value)
    ok = T.ring(262_144)                           # exactly the maximum is accepted
    got, want = _both(ok, 1 << 20)
    assert np.array_equal(got, want)
