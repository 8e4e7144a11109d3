"""Logit-space similarity (App. "Preliminary Findings": cosine similarity of target logits as an
alternative to features): the checker's cascade_accept is handed the mixed logits as features."""
import numpy as np

from oracle import verify_oracle as vo
from paper_2605_07230_amd import workloads as wl


def test_orthonormal_projection_gives_identical_sets_and_masses():
    """Logits are a linear projection of features; when the projection has orthonormal columns it
    preserves inner products, so both similarity spaces must yield the same sets and masses."""
    rng = np.random.default_rng(0)
    inp = wl.make_config(0, 3)
    h = inp.h_cond.astype(np.float64)
    Wq, _ = np.linalg.qr(rng.standard_normal((inp.vocab, inp.hidden)))      # [V, h], W^T W = I
    g = h @ Wq.T
    thr = np.full(len(g), -np.inf)
    lse = np.log(np.exp(g).sum(axis=1))
    a = vo.cascade_accept(inp.node_off, inp.parent, inp.token, h, g, thr, lse, 0.9, 0.9)
    b = vo.cascade_accept(inp.node_off, inp.parent, inp.token, g, g, thr, lse, 0.9, 0.9)
    assert a.n_int.sum() > 0
    np.testing.assert_array_equal(a.n_int, b.n_int)
    np.testing.assert_array_equal(a.n_conv, b.n_conv)
    np.testing.assert_allclose(a.cos_parent, b.cos_parent, atol=1e-12)
    np.testing.assert_allclose(a.m_int, b.m_int, rtol=0, atol=0)
    np.testing.assert_allclose(a.m_conv, b.m_conv, rtol=0, atol=0)


def test_a_generic_projection_changes_the_similarities():
    inp = wl.make_config(0, 3)
    out = vo.verify_step(inp)
    g = out["logits"]
    a = out["accept"]
    b = vo.cascade_accept(inp.node_off, inp.parent, inp.token, g, g, out["row_thr"], out["row_lse"], inp.tau_pos, inp.tau_seq)
    assert np.abs(a.cos_parent - b.cos_parent).max() > 1e-3
    np.testing.assert_array_equal(a.q_tok, b.q_tok)       # the token's own probability does not depend on the space
