"""Pins for the checker's projection / guidance / top-k / softmax statistics."""
import numpy as np
import pytest
from scipy.special import log_softmax

from oracle import verify_oracle as vo


def _case(seed, N=5, h=16, V=40):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((N, h)), rng.standard_normal((N, h)), rng.standard_normal((V, h))


def test_basis_hidden_states_pick_columns_of_w():
    rng = np.random.default_rng(0)
    h, V = 6, 11
    w = rng.standard_normal((V, h))
    g, *_ = vo.lmhead_cfg(np.eye(h), None, w)
    np.testing.assert_array_equal(g, w.T)


def test_guidance_scale_one_is_conditional_and_zero_is_unconditional():
    hc, hu, w = _case(1)
    g1, *_ = vo.lmhead_cfg(hc, hu, w, cfg_scale=1.0)
    g0, *_ = vo.lmhead_cfg(hc, hu, w, cfg_scale=0.0)
    gc, *_ = vo.lmhead_cfg(hc, None, w)
    gu, *_ = vo.lmhead_cfg(hu, None, w)
    np.testing.assert_allclose(g1, gc, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(g0, gu, rtol=1e-12, atol=1e-12)


def test_guidance_extrapolates_away_from_unconditional():
    # one hidden unit: l_c = 2 w, l_u = 1 w  =>  g = (1 + s) w for scale s  (u + s (c - u))
    w = np.array([[1.0], [-2.0], [0.5]])
    g, *_ = vo.lmhead_cfg(np.array([[2.0]]), np.array([[1.0]]), w, cfg_scale=5.0)
    np.testing.assert_allclose(g[0], 6.0 * w[:, 0])


def test_temperature_divides_logits():
    hc, hu, w = _case(2)
    g1, *_ = vo.lmhead_cfg(hc, hu, w, cfg_scale=3.0, temperature=1.0)
    g2, *_ = vo.lmhead_cfg(hc, hu, w, cfg_scale=3.0, temperature=2.0)
    np.testing.assert_allclose(g2, g1 / 2.0, rtol=1e-12)


def test_unfiltered_statistics_match_library_log_softmax():
    hc, hu, w = _case(3)
    for k in (0, 40, 99):
        g, m, thr, lse = vo.lmhead_cfg(hc, hu, w, cfg_scale=3.0, top_k=k)
        assert np.all(thr == -np.inf)
        np.testing.assert_allclose(g - lse[:, None], log_softmax(g, axis=1), rtol=1e-12, atol=1e-12)
        np.testing.assert_array_equal(m, g.max(axis=1))
        for i in range(len(g)):
            assert vo.probs_row(g[i], thr[i], lse[i]).sum() == pytest.approx(1.0, abs=1e-12)


@pytest.mark.parametrize("k", [1, 3, 17, 39])
def test_top_k_keeps_exactly_k_and_renormalises(k):
    hc, hu, w = _case(4)
    g, m, thr, lse = vo.lmhead_cfg(hc, hu, w, cfg_scale=3.0, top_k=k)
    for i in range(len(g)):
        Q = vo.probs_row(g[i], thr[i], lse[i])
        assert np.count_nonzero(Q) == k
        assert Q.sum() == pytest.approx(1.0, abs=1e-12)
        # kept entries are the k largest, and their ratios are the softmax ratios
        order = np.argsort(-g[i])
        assert set(np.nonzero(Q)[0]) == set(order[:k])
        full = np.exp(log_softmax(g[i]))
        np.testing.assert_allclose(Q[order[:k]] / Q[order[0]], full[order[:k]] / full[order[0]], rtol=1e-12)
        # brute-force threshold: the value with exactly k-1 strictly larger entries
        assert np.count_nonzero(g[i] > thr[i]) == k - 1


def test_top_k_ties_keep_every_tied_entry():
    g = np.array([[3.0, 1.0, 2.0, 2.0, 0.0]])
    m, thr, lse = vo.row_stats(g, top_k=2)
    assert thr[0] == 2.0
    assert np.count_nonzero(vo.probs_row(g[0], thr[0], lse[0])) == 3
