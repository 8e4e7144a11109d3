"""Pins of the Eq. 4 weight-mask checker."""
import numpy as np
import torch

from oracle import weights_oracle as wo


def test_against_library_cosine_similarity():
    rng = np.random.default_rng(0)
    F = rng.standard_normal((3, 17, 40))
    F[:, 5] = F[:, 4] + 0.05 * rng.standard_normal((3, 40))        # a convergent neighbour pair
    w, cs = wo.convergence_weights(F, 0.9, 2.0)
    ref = torch.nn.functional.cosine_similarity(torch.from_numpy(F[:, :-1]), torch.from_numpy(F[:, 1:]), dim=-1).numpy()
    np.testing.assert_allclose(cs[:, :-1], ref, rtol=1e-12, atol=1e-14)
    np.testing.assert_array_equal(w[:, :-1], np.where(ref >= 0.9, 2.0, 1.0))
    assert (w[:, 4] == 2.0).all() and (w[:, -1] == 1.0).all() and (cs[:, -1] == 0.0).all()


def test_constructed_cosines():
    e = np.eye(4)
    #            same dir      orthogonal   opposite     zero row     3-4-5 triangle
    rows = [e[0], 3 * e[0], e[1], -2 * e[1], 0 * e[0], np.array([3.0, 4, 0, 0]), np.array([4.0, 3, 0, 0])]
    w, cs = wo.convergence_weights(np.array(rows)[None], 0.96, 2.0)
    np.testing.assert_allclose(cs[0], [1.0, 0.0, -1.0, 0.0, 0.0, 0.96, 0.0], atol=1e-15)
    assert w[0].tolist() == [2.0, 1.0, 1.0, 1.0, 1.0, 2.0, 1.0]       # >= : the 0.96 pair is in the set
    w2, _ = wo.convergence_weights(np.array(rows)[None], 0.9600001, 3.0)
    assert w2[0].tolist() == [3.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0]


def test_positive_row_scaling_changes_nothing():
    rng = np.random.default_rng(1)
    F = rng.standard_normal((2, 9, 16))
    s = rng.uniform(0.1, 10.0, size=(2, 9, 1))
    w1, c1 = wo.convergence_weights(F, 0.2, 2.0)
    w2, c2 = wo.convergence_weights(F * s, 0.2, 2.0)
    np.testing.assert_allclose(c1, c2, atol=1e-14)
    np.testing.assert_array_equal(w1, w2)


def test_single_position_sequence():
    w, cs = wo.convergence_weights(np.ones((2, 1, 8)), 0.5, 2.0)
    assert w.tolist() == [[1.0], [1.0]] and cs.tolist() == [[0.0], [0.0]]
