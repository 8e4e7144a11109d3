"""Pins for the checker's tree attention: library routine on the chain special case,
closed forms that expose the attended set, and mask invariants."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as vo


def _rand_case(seed, parent, P=9, Hq=4, Hkv=2, D=8, S=1):
    rng = np.random.default_rng(seed)
    T = len(parent)
    N = S * T
    q = rng.standard_normal((N, Hq, D))
    kt = rng.standard_normal((N, Hkv, D))
    vt = rng.standard_normal((N, Hkv, D))
    kc = rng.standard_normal((S, Hkv, P + 3, D))
    vc = rng.standard_normal((S, Hkv, P + 3, D))
    row_parent = np.concatenate([parent] * S)
    off = np.arange(S + 1) * T
    plen = np.array([P - s for s in range(S)])
    return q, kt, vt, kc, vc, row_parent, off, plen


def test_chain_tree_equals_library_causal_attention():
    T, P, Hq, Hkv, D = 6, 9, 4, 2, 8
    parent = np.arange(-1, T - 1)
    q, kt, vt, kc, vc, rp, off, plen = _rand_case(1, parent, P, Hq, Hkv, D)
    out, _ = vo.tree_attention(q, kt, vt, kc, vc, rp, off, plen)
    # the same thing as ordinary causal attention of T new tokens after a P-token prefix
    k_all = np.concatenate([kc[0, :, :P], kt.transpose(1, 0, 2)], axis=1)      # [Hkv, P+T, D]
    v_all = np.concatenate([vc[0, :, :P], vt.transpose(1, 0, 2)], axis=1)
    k_all = np.repeat(k_all, Hq // Hkv, axis=0)
    v_all = np.repeat(v_all, Hq // Hkv, axis=0)
    q_all = np.concatenate([np.zeros((Hq, P, D)), q.transpose(1, 0, 2)], axis=1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q_all)[None], torch.from_numpy(k_all)[None], torch.from_numpy(v_all)[None], is_causal=True)
    ref = ref[0, :, P:].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("scale", [None, 0.37])
def test_chain_tree_lse_equals_library_logsumexp_of_scaled_causal_scores(scale):
    # non-zero queries and a non-unit scale: a dropped maximum, a dropped scale or a wrong key set all show
    T, P, Hq, Hkv, D = 7, 11, 4, 2, 8
    parent = np.arange(-1, T - 1)
    q, kt, vt, kc, vc, rp, off, plen = _rand_case(7, parent, P, Hq, Hkv, D)
    q *= 3.0                                                                   # scores far from 0: max term matters
    _, lse = vo.tree_attention(q, kt, vt, kc, vc, rp, off, plen, scale=scale)
    sc = (1.0 / np.sqrt(D)) if scale is None else scale
    from scipy.special import logsumexp
    for g in range(Hq):
        kv = g // (Hq // Hkv)
        keys = np.concatenate([kc[0, kv, :P], kt[:, kv]], axis=0)              # [P+T, D]
        scores = sc * (q[:, g] @ keys.T)                                       # [T, P+T]
        for i in range(T):
            want = logsumexp(scores[i, :P + i + 1])                            # causal: prefix + nodes 0..i
            assert lse[i, g] == pytest.approx(want, rel=1e-12, abs=1e-12)


def test_zero_query_reveals_attended_set():
    # q = 0 makes the softmax uniform, one-hot values then read off exactly which positions were attended
    parent = np.array([-1, 0, 0, 1, 1, 2, 5])
    T, P = len(parent), 5
    Hq = Hkv = 1
    D = P + T
    q = np.zeros((T, Hq, D))
    kt = np.random.default_rng(0).standard_normal((T, Hkv, D))
    kc = np.random.default_rng(1).standard_normal((1, Hkv, P, D))
    vc = np.zeros((1, Hkv, P, D))
    vt = np.zeros((T, Hkv, D))
    for j in range(P):
        vc[0, 0, j, j] = 1.0
    for i in range(T):
        vt[i, 0, P + i] = 1.0
    out, lse = vo.tree_attention(q, kt, vt, kc, vc, parent, np.array([0, T]), np.array([P]))
    expected_sets = {0: [0], 1: [0, 1], 2: [0, 2], 3: [0, 1, 3], 4: [0, 1, 4], 5: [0, 2, 5], 6: [0, 2, 5, 6]}
    for i in range(T):
        members = list(range(P)) + [P + a for a in expected_sets[i]]
        want = np.zeros(D)
        want[members] = 1.0 / len(members)
        np.testing.assert_allclose(out[i, 0], want, atol=1e-15)
        assert lse[i, 0] == pytest.approx(np.log(len(members)))


def test_star_tree_children_see_prefix_root_and_self_only():
    parent = np.array([-1, 0, 0, 0, 0])
    q, kt, vt, kc, vc, rp, off, plen = _rand_case(2, parent)
    out, _ = vo.tree_attention(q, kt, vt, kc, vc, rp, off, plen)
    for i in range(1, 5):
        sub_parent = np.array([-1, 0])
        idx = [0, i]
        o2, _ = vo.tree_attention(q[idx], kt[idx], vt[idx], kc, vc, sub_parent, np.array([0, 2]), plen)
        np.testing.assert_allclose(out[i], o2[1], rtol=1e-12)


def test_deleting_a_non_ancestor_subtree_changes_nothing():
    parent = np.array([-1, 0, 0, 1, 1, 2, 2, 3])
    q, kt, vt, kc, vc, rp, off, plen = _rand_case(3, parent)
    out, _ = vo.tree_attention(q, kt, vt, kc, vc, rp, off, plen)
    keep = [0, 1, 3, 4, 7]                     # drop node 2 and its subtree {5, 6}
    new_parent = np.array([-1, 0, 1, 1, 2])
    o2, _ = vo.tree_attention(q[keep], kt[keep], vt[keep], kc, vc, new_parent, np.array([0, 5]), plen)
    np.testing.assert_allclose(out[keep], o2, rtol=1e-12)


def test_sibling_permutation_permutes_outputs_only():
    parent = np.array([-1, 0, 0, 1, 2])
    q, kt, vt, kc, vc, rp, off, plen = _rand_case(4, parent)
    out, _ = vo.tree_attention(q, kt, vt, kc, vc, rp, off, plen)
    perm = [0, 2, 1, 4, 3]                     # swap the two depth-1 siblings (and their children)
    o2, _ = vo.tree_attention(q[perm], kt[perm], vt[perm], kc, vc, parent, off, plen)
    np.testing.assert_allclose(out[perm], o2, rtol=1e-12)


def test_rows_are_independent_and_respect_their_own_prefix_length():
    parent = np.array([-1, 0, 1])
    q, kt, vt, kc, vc, rp, off, plen = _rand_case(5, parent, S=2)
    out, _ = vo.tree_attention(q, kt, vt, kc, vc, rp, off, plen)
    # row 1 alone, with its cache cut to its prefix length, gives the same thing
    P1 = int(plen[1])
    o1, _ = vo.tree_attention(q[3:], kt[3:], vt[3:], kc[1:, :, :P1], vc[1:, :, :P1], parent, np.array([0, 3]), np.array([P1]))
    np.testing.assert_allclose(out[3:], o1, rtol=1e-12)
    # poisoning positions beyond the prefix length has no effect
    kc2 = kc.copy(); kc2[1, :, P1:] = 1e6
    o3, _ = vo.tree_attention(q, kt, vt, kc2, vc, rp, off, plen)
    np.testing.assert_allclose(out, o3, rtol=1e-12)


def test_grouped_heads_share_the_kv_head():
    parent = np.array([-1, 0])
    q, kt, vt, kc, vc, rp, off, plen = _rand_case(6, parent, Hq=4, Hkv=2)
    out, _ = vo.tree_attention(q, kt, vt, kc, vc, rp, off, plen)
    # head 1 uses kv head 0, head 2 uses kv head 1: recompute as single-head problems
    for g, kv in [(0, 0), (1, 0), (2, 1), (3, 1)]:
        o, _ = vo.tree_attention(q[:, [g]], kt[:, [kv]], vt[:, [kv]], kc[:, [kv]], vc[:, [kv]], rp, off, plen)
        np.testing.assert_allclose(out[:, g], o[:, 0], rtol=1e-12)
