"""Host-side checks of the synthetic input generator."""
import numpy as np
import pytest

from paper_2605_07230_amd import workloads as wl


def test_round_bf16_is_idempotent_and_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -3.14159, 0.0], np.float32)
    r = wl.round_bf16(x)
    np.testing.assert_array_equal(r, wl.round_bf16(r))
    assert r[1] == 1.0                      # tie goes to the even mantissa
    assert r[2] == np.float32(1.0 + 2 ** -7)
    assert r[3] == np.float32(1.0 + 2 ** -6)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)


@pytest.mark.parametrize("n,depth", [(1, 0), (15, 3), (60, 6), (256, 10)])
def test_grown_tree_shape(n, depth):
    p = wl.grow_tree(np.random.default_rng(n), n, depth)
    assert len(p) == n and p[0] == -1
    assert all(0 <= p[i] < i for i in range(1, n))
    assert wl.node_depths(p).max() == depth
    assert max(np.bincount(p[1:], minlength=1)) <= 10 if n > 1 else True


def test_tiny_config_layout():
    a = wl.make_config(0, seed=0)
    b = wl.make_config(0, seed=0)
    c = wl.make_config(0, seed=1)
    assert a.dtype == "f32" and a.n_rows == 1 and a.n_nodes == 15 and a.max_depth == 3
    np.testing.assert_array_equal(a.q, b.q)
    assert not np.array_equal(a.q, c.q)
    assert a.q.shape == (15, 8, 64) and a.k_cache.shape == (1, 8, 256, 64) and a.w.shape == (4096, 512)
    assert a.h_uncond is None and np.all(a.u >= 0) and np.all(a.u < 1)
    for p in range(15):
        kids = np.nonzero(a.parent == p)[0]
        assert len(set(a.token[kids])) == len(kids)


def test_janus_config_layout():
    a = wl.make_config(1, seed=0)
    assert a.dtype == "bf16" and a.n_rows == 2 and a.n_nodes == 60 and a.max_depth == 6
    assert a.row_node_off.tolist() == [0, 60, 120] and a.prefix_len.tolist() == [312, 312]
    np.testing.assert_array_equal(a.row_parent[:60], a.row_parent[60:])
    for arr in (a.q, a.k_cache, a.h_cond, a.h_uncond, a.w):
        assert np.all((arr.view(np.uint32) & 0xFFFF) == 0)      # exactly representable in bf16
    assert a.top_k == 2000 and a.cfg_scale == 5.0
    assert np.all(a.draft_prob > 0) and np.all(a.draft_prob <= 1)
