"""CPU checker for the walk with the exact multi-draft residual.  TEST INFRASTRUCTURE ONLY.

Alg. 1's correction step keeps the target's excess mass over the drafter, norm([q - p]_+)
(Preliminaries).  With several drafts per level (tree decoding), that step is applied once per
rejected sibling: the distribution that verifies the next sibling, and finally the one the last
token is drawn from, is the residual left by all siblings rejected so far at that level.  Each node
a carries the full drafter distribution p_a it was drawn from (draft_dist[a], a row of V
probabilities); the drafter probability in the acceptance test is p_a[token[a]].

The relaxation terms of Alg. 2 are unchanged: the aggregated masses stay the ones measured under the
parent's softmax (the algorithm's gtp), gated by the running budget.

Readings taken here: the residual recursion uses each rejected node's own row p_a unchanged (draws
with replacement); if a residual has no mass left (q <= p everywhere) the distribution is kept as
it was; only the SEQUENTIAL walk is defined in this mode.

Pins (tests/test_oracle_residual.py): a hand-worked residual chain (tests/golden); Monte-Carlo
check that the emitted token of a one-level tree follows the target distribution (the theorem the
correction step exists for); one-hot drafter rows reproduce the base walk's correction token; a
drafter equal to the target accepts every first child.
"""
from __future__ import annotations

from typing import List

import numpy as np

from . import verify_oracle as vo

F64 = np.float64


def residual(f, p):
    """norm([f - p]_+), or f itself when nothing is left (Alg. 1, correction step)."""
    r = np.maximum(np.asarray(f, F64) - np.asarray(p, F64), 0.0)
    z = r.sum()
    if not z > 0.0:
        return np.array(f, F64), 0.0
    return r / z, float(z)


def select_path_residual(node_off, parent, token, acc: vo.AcceptScalars, draft_dist, u, u_bonus, eps_tvd,
                         g, row_thr, row_lse, max_depth) -> vo.PathResult:
    """SEQUENTIAL walk of Alg. 2 in which every rejection replaces the verifying distribution by
    its residual against the rejected node's drafter row.  draft_dist [N, V]."""
    B = len(node_off) - 1
    accept_len = np.zeros(B, np.int32)
    path_nodes = np.full((B, max_depth), -1, np.int32)
    emitted = np.full((B, max_depth + 1), -1, np.int32)
    terminal = np.zeros(B, np.int32)
    tvd_used = np.zeros(B)
    margins: List[float] = []
    for b in range(B):
        lo, hi = int(node_off[b]), int(node_off[b + 1])
        par = np.asarray(parent[lo:hi])
        cur, curr, path = 0, 0.0, []
        f = vo.probs_row(g[lo + cur], row_thr[lo + cur], row_lse[lo + cur])
        while True:
            kids = vo.children_of(par, cur)
            if not kids:
                break
            hit = None
            for a in kids:
                ta = int(token[lo + a])
                p_a = np.asarray(draft_dist[lo + a], F64)
                ok, curr = vo._try_node(a, lo, acc, None, u, eps_tvd, curr, margins, q_base=f[ta], p_base=p_a[ta])
                if ok:
                    hit = a
                    break
                f, _ = residual(f, p_a)
            if hit is None:
                break
            path.append(hit)
            cur = hit
            f = vo.probs_row(g[lo + cur], row_thr[lo + cur], row_lse[lo + cur])
        x = vo._sample_last(f, [], float(u_bonus[b]), margins)
        accept_len[b] = len(path)
        path_nodes[b, :len(path)] = path
        emitted[b, :len(path)] = [int(token[lo + a]) for a in path]
        emitted[b, len(path)] = x
        terminal[b] = cur
        tvd_used[b] = curr
    return vo.PathResult(accept_len, path_nodes, emitted, terminal, tvd_used, float(min(margins)) if margins else np.inf)
