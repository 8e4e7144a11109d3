"""Pins for the checker's relaxed acceptance (Eq. 1-3) and walk (Alg. 2 + Alg. 1):
a hand-worked example, brute force from the full cosine matrix, an independently written
strict verifier, monotonicity of the relaxation, budget cases and the correction CDF."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import verify_oracle as vo

GOLD = os.path.join(os.path.dirname(__file__), "golden", "handworked_tree.json")


def _gold():
    with open(GOLD) as f:
        return json.load(f)


def _gold_inputs():
    gd = _gold()
    n = len(gd["parent"])
    Q = np.array([gd["Q"][str(i)] for i in range(n)])
    g = np.log(Q)
    return gd, dict(node_off=np.array([0, n]), parent=np.array(gd["parent"]), token=np.array(gd["token"]),
                    h=np.array(gd["features"], float), g=g, thr=np.full(n, -np.inf), lse=np.zeros(n))


def test_handworked_scalars():
    gd, a = _gold_inputs()
    for k, v in gd["expected_scalars"]["cos_sibling"].items():
        i, j = map(int, k.split("-"))
        assert vo.cosine(a["h"][i], a["h"][j]) == pytest.approx(v, abs=1e-12)
        assert vo.cosine(a["h"][j], a["h"][i]) == pytest.approx(v, abs=1e-12)
    acc = vo.cascade_accept(a["node_off"], a["parent"], a["token"], a["h"], a["g"], a["thr"], a["lse"],
                            gd["tau_pos"], gd["tau_seq"])
    e = gd["expected_scalars"]
    np.testing.assert_allclose(acc.q_tok, e["q_tok"], atol=1e-12)
    np.testing.assert_allclose(acc.m_int, e["m_int"], atol=1e-12)
    np.testing.assert_allclose(acc.m_conv, e["m_conv"], atol=1e-12)
    np.testing.assert_array_equal(acc.n_int, e["n_int"])
    np.testing.assert_array_equal(acc.n_conv, e["n_conv"])
    np.testing.assert_allclose(acc.cos_parent, e["cos_parent"], atol=1e-12)


@pytest.mark.parametrize("case", range(5))
def test_handworked_walks(case):
    gd, a = _gold_inputs()
    w = gd["expected_walks"][case]
    acc = vo.cascade_accept(a["node_off"], a["parent"], a["token"], a["h"], a["g"], a["thr"], a["lse"],
                            gd["tau_pos"], gd["tau_seq"])
    mode = vo.WALK_SEQUENTIAL if w["mode"] == "sequential" else vo.WALK_LONGEST
    r = vo.select_path(a["node_off"], a["parent"], a["token"], acc, np.array(gd["draft_prob"]), np.array(gd["u"]),
                       np.array([gd["u_bonus"]]), w["eps_tvd"], a["g"], a["thr"], a["lse"], 3, mode)
    assert r.accept_len[0] == w["accept_len"]
    assert list(r.path_nodes[0, :w["accept_len"]]) == w["path"]
    assert list(r.emitted[0, :w["accept_len"] + 1]) == w["emitted"]
    assert np.all(r.emitted[0, w["accept_len"] + 1:] == -1)
    assert r.terminal[0] == w["terminal"]
    assert r.tvd_used[0] == pytest.approx(w["tvd_used"], abs=1e-12)


# ------------------------------------------------------------------ random small trees

def _random_tree(rng, n, max_kids=3):
    parent = [-1]
    for i in range(1, n):
        cands = [p for p in range(i) if parent.count(p) < max_kids]
        parent.append(int(rng.choice(cands)))
    # renumber so siblings need not be contiguous but parent < child holds
    return np.array(parent)


def _random_case(seed, n=12, V=24, h=6, dup=0.5, top_k=0, distinct_tokens=True):
    rng = np.random.default_rng(seed)
    parent = _random_tree(rng, n)
    H = rng.standard_normal((n, h))
    for i in range(1, n):
        r = rng.random()
        sibs = [j for j in range(i) if parent[j] == parent[i]]
        if r < dup / 2:
            H[i] = H[parent[i]] * rng.uniform(0.5, 2) + 0.05 * rng.standard_normal(h)
        elif r < dup and sibs:
            H[i] = H[sibs[0]] * rng.uniform(0.5, 2) + 0.05 * rng.standard_normal(h)
    token = rng.integers(0, V, n)
    if distinct_tokens:
        for p in range(n):
            kids = np.nonzero(parent == p)[0]
            token[kids] = rng.choice(V, len(kids), replace=False)
    g = 2.0 * rng.standard_normal((n, V))
    m, thr, lse = vo.row_stats(g, top_k)
    return dict(node_off=np.array([0, n]), parent=parent, token=token, h=H, g=g, thr=thr, lse=lse,
                draft_prob=rng.uniform(0.02, 0.3, n), u=rng.random(n), u_bonus=rng.random(1), V=V)


def _brute_scalars(c, tau_pos, tau_seq):
    """Eq. 1-3 evaluated from the full cosine matrix with set arithmetic."""
    par, tok, H = c["parent"], c["token"], c["h"]
    n = len(par)
    Hn = H / np.linalg.norm(H, axis=1, keepdims=True)
    cosm = Hn @ Hn.T
    soft = np.exp(c["g"] - c["lse"][:, None]) * (c["g"] >= c["thr"][:, None])
    out = []
    for a in range(n):
        if par[a] < 0:
            out.append((0.0, 0.0, 0.0, 0, 0))
            continue
        Q = soft[par[a]]
        I = {b for b in range(n) if b != a and par[b] == par[a] and cosm[a, b] >= tau_pos}
        C = {b for b in range(n) if par[b] == a and cosm[a, b] >= tau_seq}
        ti = {tok[b] for b in I} - {tok[a]}
        tc = {tok[b] for b in C} - {tok[a]} - ti
        out.append((Q[tok[a]], sum(Q[t] for t in ti), sum(Q[t] for t in tc), len(I), len(C)))
    return out


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("distinct", [True, False])
def test_scalars_against_brute_force(seed, distinct):
    c = _random_case(seed, top_k=(0 if seed % 2 else 10), distinct_tokens=distinct)
    acc = vo.cascade_accept(c["node_off"], c["parent"], c["token"], c["h"], c["g"], c["thr"], c["lse"], 0.9, 0.8)
    ref = _brute_scalars(c, 0.9, 0.8)
    for a, (q, mi, mc, ni, nc) in enumerate(ref):
        assert acc.q_tok[a] == pytest.approx(q, rel=1e-12, abs=1e-15)
        assert acc.m_int[a] == pytest.approx(mi, rel=1e-12, abs=1e-15)
        assert acc.m_conv[a] == pytest.approx(mc, rel=1e-12, abs=1e-15)
        assert (acc.n_int[a], acc.n_conv[a]) == (ni, nc)


def _strict_tree_verifier(parent, token, soft, draft_prob, u):
    """Alg. 1's test applied level by level on a tree, written independently (division form, recursion)."""
    def descend(cur, path):
        rejected = []
        for a in [i for i in range(len(parent)) if parent[i] == cur]:
            ratio = soft[cur][token[a]] / draft_prob[a]
            if u[a] < min(1.0, ratio):
                return descend(a, path + [a])
            rejected.append(a)
        return path, cur, rejected
    return descend(0, [])


@pytest.mark.parametrize("seed", range(20))
def test_disabled_thresholds_and_zero_budget_reduce_to_strict_speculative_sampling(seed):
    c = _random_case(100 + seed, top_k=(0 if seed % 2 else 8))
    soft = np.exp(c["g"] - c["lse"][:, None]) * (c["g"] >= c["thr"][:, None])
    path, cur, rejected = _strict_tree_verifier(c["parent"], c["token"], soft, c["draft_prob"], c["u"])
    resid = soft[cur].copy()
    resid[[c["token"][a] for a in rejected]] = 0.0
    cdf = np.cumsum(resid / resid.sum())
    x = int(np.searchsorted(cdf, c["u_bonus"][0], side="right"))
    for tau, eps in [(2.0, 0.5), (0.5, 0.0)]:
        acc = vo.cascade_accept(c["node_off"], c["parent"], c["token"], c["h"], c["g"], c["thr"], c["lse"], tau, tau)
        if tau > 1:
            assert not acc.n_int.any() and not acc.n_conv.any() and not acc.m_int.any() and not acc.m_conv.any()
        for mode in (vo.WALK_SEQUENTIAL,):
            r = vo.select_path(c["node_off"], c["parent"], c["token"], acc, c["draft_prob"], c["u"], c["u_bonus"], eps,
                               c["g"], c["thr"], c["lse"], 12, mode)
            assert list(r.path_nodes[0, :r.accept_len[0]]) == path
            assert r.terminal[0] == cur
            assert r.emitted[0, r.accept_len[0]] == x
            assert r.tvd_used[0] == 0.0


def _isolated_flags(c, acc, eps=np.inf):
    return np.array([a > 0 and c["u"][a] * c["draft_prob"][a] < acc.q_tok[a] + acc.m_int[a] + acc.m_conv[a]
                     for a in range(len(c["parent"]))])


@pytest.mark.parametrize("seed", range(15))
def test_relaxation_only_adds_acceptances(seed):
    c = _random_case(200 + seed, dup=0.8)
    args = (c["node_off"], c["parent"], c["token"], c["h"], c["g"], c["thr"], c["lse"])
    strict = _isolated_flags(c, vo.cascade_accept(*args, 2.0, 2.0))
    only_i = _isolated_flags(c, vo.cascade_accept(*args, 0.8, 2.0))
    only_c = _isolated_flags(c, vo.cascade_accept(*args, 2.0, 0.8))
    both = _isolated_flags(c, vo.cascade_accept(*args, 0.8, 0.8))
    assert np.all(strict <= only_i) and np.all(strict <= only_c)
    assert np.all((only_i | only_c) <= both)
    # lower thresholds never shrink the sets
    lo = vo.cascade_accept(*args, 0.5, 0.5)
    hi = vo.cascade_accept(*args, 0.9, 0.9)
    assert np.all(lo.n_int >= hi.n_int) and np.all(lo.n_conv >= hi.n_conv)
    # unlimited budget: at every level where the strict walk accepts a child, the relaxed walk accepts
    # that child or an earlier sibling; and the best single path never gets shorter
    acc_s = vo.cascade_accept(*args, 2.0, 2.0)
    acc_r = vo.cascade_accept(*args, 0.8, 0.8)
    kw = dict(max_depth=12)
    longest_s = vo.select_path(c["node_off"], c["parent"], c["token"], acc_s, c["draft_prob"], c["u"], c["u_bonus"], 1e9,
                               c["g"], c["thr"], c["lse"], 12, vo.WALK_LONGEST)
    longest_r = vo.select_path(c["node_off"], c["parent"], c["token"], acc_r, c["draft_prob"], c["u"], c["u_bonus"], 1e9,
                               c["g"], c["thr"], c["lse"], 12, vo.WALK_LONGEST)
    assert longest_r.accept_len[0] >= longest_s.accept_len[0]
    seq_s = vo.select_path(c["node_off"], c["parent"], c["token"], acc_s, c["draft_prob"], c["u"], c["u_bonus"], 1e9,
                           c["g"], c["thr"], c["lse"], 12)
    seq_r = vo.select_path(c["node_off"], c["parent"], c["token"], acc_r, c["draft_prob"], c["u"], c["u_bonus"], 1e9,
                           c["g"], c["thr"], c["lse"], 12)
    if seq_s.accept_len[0] >= 1:
        assert seq_r.accept_len[0] >= 1 and seq_r.path_nodes[0, 0] <= seq_s.path_nodes[0, 0]
    assert longest_s.accept_len[0] >= seq_s.accept_len[0]


@pytest.mark.parametrize("seed", range(15))
def test_walks_against_brute_force_path_enumeration(seed):
    c = _random_case(300 + seed, dup=0.8)
    par = c["parent"]
    n = len(par)
    acc = vo.cascade_accept(c["node_off"], par, c["token"], c["h"], c["g"], c["thr"], c["lse"], 0.8, 0.8)
    flags = _isolated_flags(c, acc)
    # unlimited budget: a path is acceptable iff every node on it passes its isolated test
    leaves = [i for i in range(n) if not np.any(par == i)]
    best_len = 0
    for leaf in leaves:
        chain = vo.ancestors_or_self(par, leaf)[1:]
        k = 0
        for a in chain:
            if not flags[a]:
                break
            k += 1
        best_len = max(best_len, k)
    longest = vo.select_path(c["node_off"], par, c["token"], acc, c["draft_prob"], c["u"], c["u_bonus"], 1e9,
                             c["g"], c["thr"], c["lse"], 12, vo.WALK_LONGEST)
    assert longest.accept_len[0] == best_len
    seq = vo.select_path(c["node_off"], par, c["token"], acc, c["draft_prob"], c["u"], c["u_bonus"], 1e9,
                         c["g"], c["thr"], c["lse"], 12)
    # the sequential walk is the lexicographically first acceptable, non-extendable path
    cur, want = 0, []
    while True:
        nxt = [a for a in range(n) if par[a] == cur and flags[a]]
        if not nxt:
            break
        cur = nxt[0]
        want.append(cur)
    assert list(seq.path_nodes[0, :seq.accept_len[0]]) == want
    # with an unlimited budget every tried node (rejected earlier siblings and the accepted one) adds its masses
    tried, cur = [], 0
    for step in want + [None]:
        for a in [a for a in range(n) if par[a] == cur]:
            tried.append(a)
            if a == step:
                break
        if step is None:
            break
        cur = step
    assert seq.tvd_used[0] == pytest.approx(sum(acc.m_int[a] + acc.m_conv[a] for a in tried), rel=1e-12)


def test_budget_is_all_or_nothing_and_inclusive():
    gd, a = _gold_inputs()
    acc = vo.cascade_accept(a["node_off"], a["parent"], a["token"], a["h"], a["g"], a["thr"], a["lse"], 0.9, 0.9)
    def run(eps):
        return vo.select_path(a["node_off"], a["parent"], a["token"], acc, np.array(gd["draft_prob"]),
                              np.array(gd["u"]), np.array([0.75]), eps, a["g"], a["thr"], a["lse"], 3)
    # node 1 adds 0.20, node 2's interchangeable set needs a running total of 0.40
    t = float(acc.m_conv[1] + acc.m_int[2])
    assert run(t).tvd_used[0] == pytest.approx(t)               # budget exactly met: admitted (<=)
    assert run(t + 1e-3).path_nodes[0, 0] == 2
    r = run(t - 1e-3)                                            # just short: set refused, node 2 rejected
    # node 3's interchangeable set (0.15) still fits on top of node 1's 0.20
    assert r.path_nodes[0, 0] == 3 and r.tvd_used[0] == pytest.approx(0.35)
    for eps in (0.0, 0.1, 0.25, 0.4, 0.5, 0.66, 5.0):
        assert run(eps).tvd_used[0] <= eps + 1e-15


def test_correction_token_follows_the_closed_form_cdf():
    # four-token vocabulary, root with two children that are both rejected (u = 0.999..)
    Q = np.array([0.1, 0.2, 0.3, 0.4])
    g = np.log(np.tile(Q, (3, 1)))
    parent = np.array([-1, 0, 0])
    token = np.array([0, 1, 3])
    h = np.eye(3)
    acc = vo.cascade_accept(np.array([0, 3]), parent, token, h, g, np.full(3, -np.inf), np.zeros(3), 2.0, 2.0)
    # residual = [q - delta_tried]_+ renormalised = (0.1, 0, 0.3, 0) / 0.4  ->  cdf 0.25, 0.25, 1, 1
    for ub, want in [(0.0, 0), (0.2, 0), (0.2499, 0), (0.2501, 2), (0.9, 2), (0.999999, 2)]:
        r = vo.select_path(np.array([0, 3]), parent, token, acc, np.array([1.0, 1.0, 1.0]), np.array([0.0, 0.999, 0.999]),
                           np.array([ub]), 0.5, g, np.full(3, -np.inf), np.zeros(3), 2)
        assert r.accept_len[0] == 0 and r.emitted[0, 0] == want
    # literal Alg. 1 residual norm([q - p]_+) with a point-mass drafter on one rejected token
    p = np.zeros(4); p[1] = 1.0
    resid = np.maximum(Q - p, 0); resid /= resid.sum()
    parent1 = np.array([-1, 0]); token1 = np.array([0, 1])
    acc1 = vo.cascade_accept(np.array([0, 2]), parent1, token1, np.eye(2), g[:2], np.full(2, -np.inf), np.zeros(2), 2.0, 2.0)
    cdf = np.cumsum(resid)
    for ub in np.linspace(0.01, 0.99, 23):
        r = vo.select_path(np.array([0, 2]), parent1, token1, acc1, np.array([1.0, 1.0]), np.array([0.0, 0.999]),
                           np.array([ub]), 0.5, g[:2], np.full(2, -np.inf), np.zeros(2), 1)
        assert r.emitted[0, 0] == int(np.searchsorted(cdf, ub, side="right"))


def test_root_only_tree_and_leaf_bonus():
    Q = np.array([0.1, 0.2, 0.3, 0.4])
    g = np.log(Q)[None]
    acc = vo.cascade_accept(np.array([0, 1]), np.array([-1]), np.array([2]), np.ones((1, 2)), g, np.array([-np.inf]), np.zeros(1), 0.5, 0.5)
    r = vo.select_path(np.array([0, 1]), np.array([-1]), np.array([2]), acc, None, np.array([0.3]), np.array([0.35]),
                       0.5, g, np.array([-np.inf]), np.zeros(1), 0)
    assert r.accept_len[0] == 0 and r.terminal[0] == 0 and r.emitted[0, 0] == 2


def test_zero_norm_feature_has_zero_cosine():
    assert vo.cosine(np.zeros(3), np.ones(3)) == 0.0
    assert vo.cosine(np.ones(3), np.zeros(3)) == 0.0


def test_duplicate_tokens_are_counted_once_and_own_token_never():
    # node 1 and 2 are siblings with identical features; node 1's children 3 and 4 repeat tokens
    parent = np.array([-1, 0, 0, 1, 1, 1])
    token = np.array([0, 1, 2, 2, 1, 3])       # child 3 repeats the sibling's token, child 4 repeats node 1's own
    h = np.ones((6, 2))
    Q = np.array([0.1, 0.2, 0.3, 0.4])
    g = np.log(np.tile(Q, (6, 1)))
    acc = vo.cascade_accept(np.array([0, 6]), parent, token, h, g, np.full(6, -np.inf), np.zeros(6), 0.9, 0.9)
    assert acc.q_tok[1] == pytest.approx(0.2)
    assert acc.m_int[1] == pytest.approx(0.3) and acc.n_int[1] == 1
    assert acc.m_conv[1] == pytest.approx(0.4) and acc.n_conv[1] == 3       # only token 3 is new mass
