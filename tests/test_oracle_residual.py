"""Pins of the residual-walk checker (oracle/residual_oracle.py)."""
import json
import os

import numpy as np

from oracle import residual_oracle as ro
from oracle import verify_oracle as vo

GOLD = os.path.join(os.path.dirname(__file__), "golden", "handworked_residual.json")


def _zero_scalars(n):
    z = np.zeros(n)
    zi = np.zeros(n, np.int32)
    return vo.AcceptScalars(z.copy(), z.copy(), z.copy(), zi.copy(), zi.copy(), z.copy(), np.inf)


def _logits(Qrows):
    with np.errstate(divide="ignore"):
        g = np.log(np.asarray(Qrows, np.float64))
    n = len(Qrows)
    return g, np.full(n, -np.inf), np.zeros(n)


def test_handworked_residual_chain():
    gold = json.load(open(GOLD))
    chain = gold["residual_chain"]
    p = gold["draft_rows"]["1"]
    f = np.array(chain["start"])
    for key, z_expect in zip(["after_1_rejection", "after_2_rejections", "after_3_rejections"], chain["normalisers"]):
        f, z = ro.residual(f, p)
        np.testing.assert_allclose(f, chain[key], rtol=0, atol=1e-15)
        assert abs(z - z_expect) < 1e-15


def test_handworked_walks():
    gold = json.load(open(GOLD))
    parent = np.array(gold["parent"], np.int32)
    n, V = len(parent), gold["vocab"]
    g, thr, lse = _logits([gold["Q"][str(i)] for i in range(n)])
    dd = np.zeros((n, V))
    for k, row in gold["draft_rows"].items():
        dd[int(k)] = row
    off = np.array([0, n], np.int32)
    for case in gold["cases"]:
        tok = np.array(case["token"], np.int32)
        res = ro.select_path_residual(off, parent, tok, _zero_scalars(n), dd, np.array(case["u"]), np.array([case["u_bonus"]]),
                                      0.5, g, thr, lse, 3)
        assert res.accept_len[0] == case["accept_len"], case["_why"]
        assert res.path_nodes[0, :case["accept_len"]].tolist() == case["path"], case["_why"]
        assert res.emitted[0, :case["accept_len"] + 1].tolist() == case["emitted"], case["_why"]
        assert res.terminal[0] == case["terminal"], case["_why"]


def test_emitted_token_follows_the_target_distribution():
    """One level, two drafts drawn i.i.d. from the drafter: whatever is emitted first (an accepted
    draft or the correction token) is distributed as the target — the property the residual
    recursion exists to keep.  40000 seeded trials, tolerance 4 standard deviations."""
    rng = np.random.default_rng(123)
    Q = np.array([0.5, 0.3, 0.2])
    p = np.array([0.2, 0.2, 0.6])
    parent = np.array([-1, 0, 0], np.int32)
    off = np.array([0, 3], np.int32)
    g, thr, lse = _logits([Q, Q, Q])
    dd = np.stack([p, p, p])
    acc = _zero_scalars(3)
    n_trials = 40000
    counts = np.zeros(3)
    toks = rng.choice(3, size=(n_trials, 2), p=p)
    us = rng.random((n_trials, 3))
    ub = rng.random(n_trials)
    for t in range(n_trials):
        tok = np.array([0, toks[t, 0], toks[t, 1]], np.int32)
        res = ro.select_path_residual(off, parent, tok, acc, dd, us[t], ub[t:t + 1], 0.5, g, thr, lse, 1)
        counts[res.emitted[0, 0]] += 1
    freq = counts / n_trials
    sd = np.sqrt(Q * (1 - Q) / n_trials)
    assert np.all(np.abs(freq - Q) < 4 * sd), (freq, Q)


def test_one_hot_drafter_rows_reproduce_the_base_correction_token():
    """With a point-mass drafter per node, norm([q - p]_+) zeroes that node's token: after all
    children are rejected the last token must be the one the base walk draws."""
    rng = np.random.default_rng(7)
    V, n_kids = 64, 6
    for trial in range(50):
        Q = rng.dirichlet(np.ones(V))
        parent = np.array([-1] + [0] * n_kids, np.int32)
        order = np.argsort(Q)
        tok = np.array([0] + order[:n_kids].tolist(), np.int32)       # the least likely tokens: all get rejected
        u = np.full(n_kids + 1, 0.999)
        off = np.array([0, n_kids + 1], np.int32)
        g, thr, lse = _logits([Q] * (n_kids + 1))
        acc = _zero_scalars(n_kids + 1)
        acc.q_tok[1:] = Q[tok[1:]]
        dd = np.zeros((n_kids + 1, V))
        dd[np.arange(1, n_kids + 1), tok[1:]] = 1.0
        ub = rng.random(1)
        base = vo.select_path(off, parent, tok, acc, None, u, ub, 0.5, g, thr, lse, 1)
        res = ro.select_path_residual(off, parent, tok, acc, dd, u, ub, 0.5, g, thr, lse, 1)
        assert base.accept_len[0] == 0 and res.accept_len[0] == 0
        assert base.emitted[0, 0] == res.emitted[0, 0]
        assert res.emitted[0, 0] not in tok[1:].tolist()


def test_drafter_equal_to_target_accepts_every_first_child():
    rng = np.random.default_rng(3)
    V = 16
    parent = np.array([-1, 0, 0, 1, 1, 3], np.int32)
    n = len(parent)
    Qs = rng.dirichlet(np.ones(V), size=n)
    tok = rng.integers(0, V, size=n).astype(np.int32)
    dd = np.zeros((n, V))
    for a in range(1, n):
        dd[a] = Qs[parent[a]]
    g, thr, lse = _logits(Qs)
    res = ro.select_path_residual(np.array([0, n], np.int32), parent, tok, _zero_scalars(n), dd, rng.random(n), rng.random(1),
                                  0.5, g, thr, lse, 3)
    assert res.path_nodes[0].tolist() == [1, 3, 5]


def test_relaxation_terms_still_apply_under_the_budget():
    """A mass that fits the budget lifts a node over the bar exactly as in the base walk."""
    parent = np.array([-1, 0, 0], np.int32)
    Q = [0.4, 0.3, 0.2, 0.1]
    g, thr, lse = _logits([Q, Q, Q])
    tok = np.array([0, 3, 2], np.int32)
    acc = _zero_scalars(3)
    acc.n_int[1], acc.m_int[1] = 1, 0.2          # node 1 may borrow token 2's mass
    dd = np.tile(np.array([0.1, 0.1, 0.1, 0.7]), (3, 1))
    u = np.array([0.0, 0.4, 0.9])                # 0.4*0.7 = 0.28: above 0.1, below 0.1 + 0.2
    off = np.array([0, 3], np.int32)
    tight = ro.select_path_residual(off, parent, tok, acc, dd, u, np.array([0.5]), 0.1, g, thr, lse, 1)
    loose = ro.select_path_residual(off, parent, tok, acc, dd, u, np.array([0.5]), 0.5, g, thr, lse, 1)
    assert tight.path_nodes[0, 0] != 1 and loose.path_nodes[0, 0] == 1
    assert abs(loose.tvd_used[0] - 0.2) < 1e-15 and tight.tvd_used[0] == 0.0
