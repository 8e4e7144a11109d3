"""CPU checker for one tree-verification step of CASCADE.  TEST INFRASTRUCTURE ONLY.

Plain numpy in float64, written from the paper's definitions so that it can be
read against them.  It shares no code with the GPU library and must never be
imported by it: only the tests, the smoke check and the benchmark's CPU-baseline
leg call into this file.

What is pinned by the CPU tests, and by what:

* ``tree_attention``  — softmax attention over prefix + ancestors + self
  (Preliminaries, "parallel forward pass"; tree decoding with a tree mask).
  Pins: chain tree == a library causal attention; zero queries reveal the
  attended set through one-hot values; subtree deletion / sibling permutation
  invariance.
* ``lmhead_cfg``      — final projection, guidance mix, top-k, softmax
  (Sec. 4.2 cost discussion; App. "Configuration Details").  Pins: library
  log-softmax, basis-vector hidden states, guidance scale 0 and 1, kept count.
* ``cascade_accept``  — cosine similarity, Eq. 1, Eq. 2 and the aggregated masses
  of Eq. 3.  Pins: a hand-worked example stored under tests/golden, brute force
  from the full cosine matrix with python sets.
* ``select_path``     — Alg. 2 control flow with the budget, Alg. 1 acceptance test
  and correction step.  Pins: the hand-worked example, an independently written
  strict tree verifier (thresholds disabled), brute-force path enumeration,
  budget straddling cases, closed-form inverse-CDF on a 4-token vocabulary.
  Parity with the authors' own implementation is UNPINNED: the paper prints no
  numeric example, so the pins are the definitions above.

Readings of the paper taken where it is loose (all listed in the design notes):
features are the node's own final hidden state; the interchangeable set is taken
among siblings, the convergent set among a node's children; added mass is measured
under the distribution that verifies the node (its parent's); thresholds compare
with >=; the budget is consumed all-or-nothing per set, including by siblings that
are then rejected; the walk stops at the first level with no accepted child; the
correction token is drawn from the unrelaxed distribution with the tried siblings'
tokens removed (Alg. 1's residual for a point-mass drafter).
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- tree helpers

def children_of(parent: np.ndarray, p: int) -> List[int]:
    """Children of node p in ascending node index (the order siblings are tried in)."""
    return [int(i) for i in range(len(parent)) if parent[i] == p]


def ancestors_or_self(parent: np.ndarray, i: int) -> List[int]:
    out = []
    while i >= 0:
        out.append(int(i))
        i = int(parent[i])
    return out[::-1]


# --------------------------------------------------------------------------- step A

def tree_attention(q, k_tree, v_tree, k_cache, v_cache, row_parent, row_node_off, prefix_len, scale=None):
    """Tree-masked attention of the drafted tree against the prefix KV cache.

    Every node of a row attends the row's prefix positions, its ancestors in the tree
    and itself: the parallel verification pass conditions each draft token on the
    prefix plus its own draft path (Preliminaries; tree decoding, "tree mask").

    q [N,Hq,D]; k_tree,v_tree [N,Hkv,D]; k_cache,v_cache [S,Hkv,P_cap,D];
    row_parent [N] local indices; row_node_off [S+1]; prefix_len [S].
    Returns (out [N,Hq,D] float64, lse [N,Hq] float64) with lse = log sum exp of the
    scaled scores over the attended set.
    """
    q = np.asarray(q, F64)
    k_tree = np.asarray(k_tree, F64)
    v_tree = np.asarray(v_tree, F64)
    N, Hq, D = q.shape
    Hkv = k_tree.shape[1]
    group = Hq // Hkv
    if scale is None or scale == 0:
        scale = 1.0 / np.sqrt(D)
    out = np.zeros((N, Hq, D), F64)
    lse = np.zeros((N, Hq), F64)
    S = len(prefix_len)
    for s in range(S):
        lo, hi = int(row_node_off[s]), int(row_node_off[s + 1])
        par = np.asarray(row_parent[lo:hi])
        P = int(prefix_len[s])
        for g in range(Hq):
            kv = g // group
            kp = np.asarray(k_cache[s, kv, :P], F64)
            vp = np.asarray(v_cache[s, kv, :P], F64)
            for i in range(hi - lo):
                anc = [lo + a for a in ancestors_or_self(par, i)]
                keys = np.concatenate([kp, k_tree[anc, kv]], axis=0)
                vals = np.concatenate([vp, v_tree[anc, kv]], axis=0)
                z = scale * (keys @ q[lo + i, g])
                m = z.max()
                e = np.exp(z - m)
                den = e.sum()
                out[lo + i, g] = (e / den) @ vals
                lse[lo + i, g] = m + np.log(den)
    return out, lse


# --------------------------------------------------------------------------- step B

def lmhead_cfg(h_cond, h_uncond, w, cfg_scale=1.0, temperature=1.0, top_k=0):
    """Final projection with guidance mixing, temperature, top-k threshold and softmax statistics.

    l = H W^T for the conditional and unconditional rows; g = l_u + s (l_c - l_u)
    (no unconditional rows: g = l_c); g /= temperature; thr = k-th largest g of the row
    (top_k == 0 or >= V: no filtering, thr = -inf); row_max; lse = log sum over kept
    entries of exp(g).  (Sec. 4.2: the O(hV) final projection; App. "Configuration
    Details": guidance scale, temperature 1, top-k 2000, top-p 1.)
    Returns (g [N,V], row_max [N], row_thr [N], row_lse [N]) in float64.
    """
    w = np.asarray(w, F64)
    lc = np.asarray(h_cond, F64) @ w.T
    if h_uncond is not None:
        lu = np.asarray(h_uncond, F64) @ w.T
        g = lu + F64(cfg_scale) * (lc - lu)
    else:
        g = lc
    g = g / F64(temperature)
    return (g,) + row_stats(g, top_k)


def row_stats(g, top_k=0):
    """row_max, k-th-largest threshold and log-sum-exp over kept entries, for each row of g."""
    g = np.asarray(g, F64)
    N, V = g.shape
    row_max = g.max(axis=1)
    if top_k <= 0 or top_k >= V:
        thr = np.full(N, -np.inf)
    else:
        thr = np.sort(g, axis=1)[:, V - top_k]
    keep = g >= thr[:, None]
    lse = row_max + np.log(np.where(keep, np.exp(g - row_max[:, None]), 0.0).sum(axis=1))
    return row_max, thr, lse


def probs_row(g_row, thr, lse):
    """The target distribution of one node: exp(g - lse) on kept entries, 0 elsewhere."""
    g_row = np.asarray(g_row, F64)
    return np.where(g_row >= thr, np.exp(g_row - F64(lse)), 0.0)


# --------------------------------------------------------------------------- step C

def cosine(a, b) -> float:
    """<a,b> / (|a| |b|); 0 when either vector has zero norm (Sec. 4.1, measurement method)."""
    a = np.asarray(a, F64)
    b = np.asarray(b, F64)
    na = np.sqrt(a @ a)
    nb = np.sqrt(b @ b)
    if na == 0.0 or nb == 0.0:
        return 0.0
    return float((a @ b) / (na * nb))


@dataclasses.dataclass
class AcceptScalars:
    q_tok: np.ndarray        # [N] probability of the node's draft token under its parent's distribution
    m_int: np.ndarray        # [N] mass added by the interchangeable siblings (Eq. 3, second term)
    m_conv: np.ndarray       # [N] mass added by the convergent children (Eq. 3, third term)
    n_int: np.ndarray        # [N] |I_a|
    n_conv: np.ndarray       # [N] |C_a|
    cos_parent: np.ndarray   # [N] cos(F_parent, F_node); 0 for roots
    min_cos_margin: float    # smallest |cos - tau| met while forming the sets


def cascade_accept(node_off, parent, token, h_cond, g, row_thr, row_lse, tau_pos, tau_seq) -> AcceptScalars:
    """Per-node quantities of the relaxed acceptance rule (Eq. 1-3), for every non-root node a.

    I_a = siblings b != a with cos(F_a, F_b) >= tau_pos                      (Eq. 1)
    C_a = children b of a with cos(F_a, F_b) >= tau_seq                      (Eq. 2)
    Masses are taken under Q = the distribution of a's parent (the one that verifies a),
    summed over distinct token ids, never counting a's own token, and never counting in
    m_conv a token already counted in m_int.  Root entries are 0.
    """
    N = int(node_off[-1])
    q_tok = np.zeros(N)
    m_int = np.zeros(N)
    m_conv = np.zeros(N)
    n_int = np.zeros(N, np.int32)
    n_conv = np.zeros(N, np.int32)
    cos_parent = np.zeros(N)
    margin = np.inf
    for b in range(len(node_off) - 1):
        lo, hi = int(node_off[b]), int(node_off[b + 1])
        par = np.asarray(parent[lo:hi])
        for a in range(1, hi - lo):
            p = int(par[a])
            Q = probs_row(g[lo + p], row_thr[lo + p], row_lse[lo + p])
            ta = int(token[lo + a])
            q_tok[lo + a] = Q[ta]
            cos_parent[lo + a] = cosine(h_cond[lo + p], h_cond[lo + a])
            set_i = []
            for s in children_of(par, p):
                if s == a:
                    continue
                c = cosine(h_cond[lo + a], h_cond[lo + s])
                margin = min(margin, abs(c - tau_pos))
                if c >= tau_pos:
                    set_i.append(s)
            set_c = []
            for c_ in children_of(par, a):
                c = cosine(h_cond[lo + a], h_cond[lo + c_])
                margin = min(margin, abs(c - tau_seq))
                if c >= tau_seq:
                    set_c.append(c_)
            tok_i = {int(token[lo + s]) for s in set_i} - {ta}
            tok_c = {int(token[lo + c_]) for c_ in set_c} - {ta} - tok_i
            m_int[lo + a] = sum(Q[t] for t in sorted(tok_i))
            m_conv[lo + a] = sum(Q[t] for t in sorted(tok_c))
            n_int[lo + a] = len(set_i)
            n_conv[lo + a] = len(set_c)
    return AcceptScalars(q_tok, m_int, m_conv, n_int, n_conv, cos_parent, float(margin))


# --------------------------------------------------------------------------- step D

WALK_SEQUENTIAL = 0
WALK_LONGEST = 1


@dataclasses.dataclass
class PathResult:
    accept_len: np.ndarray      # [B]
    path_nodes: np.ndarray      # [B, max_depth], -1 padded, local node indices
    emitted: np.ndarray         # [B, max_depth+1], accepted draft tokens then the correction/bonus token, -1 padded
    terminal: np.ndarray        # [B] local index of the node whose distribution gave the last token
    tvd_used: np.ndarray        # [B]
    min_margin: float           # smallest relative margin of any comparison that was taken


def _try_node(a, lo, acc: AcceptScalars, draft_prob, u, eps, curr, margins, q_base=None, p_base=None):
    """Alg. 2 body for one tried node: budget-gated aggregation, then Alg. 1's test.  Returns (accepted, curr).
    q_base / p_base replace the node's stored target / drafter probability (residual walk)."""
    q_x = float(acc.q_tok[lo + a]) if q_base is None else float(q_base)
    if acc.n_int[lo + a] > 0:
        m = float(acc.m_int[lo + a])
        margins.append(abs(curr + m - eps) / max(eps, 1e-30))
        if curr + m <= eps:
            q_x += m
            curr += m
    if acc.n_conv[lo + a] > 0:
        m = float(acc.m_conv[lo + a])
        margins.append(abs(curr + m - eps) / max(eps, 1e-30))
        if curr + m <= eps:
            q_x += m
            curr += m
    p_x = 1.0 if draft_prob is None else float(draft_prob[lo + a])
    if p_base is not None:
        p_x = float(p_base)
    r = float(u[lo + a])
    lhs = r * p_x                       # r < min(1, q_x/p_x)  <=>  r*p_x < q_x   (0 <= r < 1, p_x > 0)
    margins.append(abs(lhs - q_x) / max(abs(lhs), abs(q_x), 1e-30))
    return lhs < q_x, curr


def _sample_last(Q, banned_tokens, u_b, margins):
    """Correction / bonus token: inverse CDF, in vocabulary order, of Q with the tried tokens removed."""
    R = np.array(Q, F64)
    for t in banned_tokens:
        R[t] = 0.0
    tot = R.sum()
    if not tot > 0.0:
        R = np.array(Q, F64)
        tot = R.sum()
    cdf = np.cumsum(R) / tot
    idx = np.nonzero(cdf > u_b)[0]
    if len(idx) == 0:
        x = int(np.nonzero(R > 0)[0][-1])
    else:
        x = int(idx[0])
    prev = cdf[x - 1] if x > 0 else 0.0
    margins.append(min(abs(cdf[x] - u_b), abs(u_b - prev) if x > 0 and prev > 0 else 1.0))
    return x


def select_path(node_off, parent, token, acc: AcceptScalars, draft_prob, u, u_bonus, eps_tvd,
                g, row_thr, row_lse, max_depth, mode=WALK_SEQUENTIAL) -> PathResult:
    """Walk of Alg. 2 over one step's trees, then the correction step of Alg. 1.

    SEQUENTIAL: at each level the children of the current node are tried in ascending
    index; each tried child first aggregates its interchangeable and convergent masses
    when the running total stays within eps_tvd (the running total grows even if the
    child is then rejected), then passes iff u*p < q^R.  First pass moves the walk down;
    no pass ends it.  LONGEST: the same rule is simulated along every root-to-leaf path
    on its own (only that path's node is tried per level); the path with the longest
    accepted prefix wins, ties to the smallest leaf index.
    """
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
        if mode == WALK_SEQUENTIAL:
            cur, curr, path, tried = 0, 0.0, [], []
            while True:
                kids = children_of(par, cur)
                tried = []
                if not kids:
                    break
                hit = None
                for a in kids:
                    ok, curr = _try_node(a, lo, acc, draft_prob, u, eps_tvd, curr, margins)
                    if ok:
                        hit = a
                        break
                    tried.append(a)
                if hit is None:
                    break
                path.append(hit)
                cur = hit
        else:
            best = None
            leaves = [i for i in range(hi - lo) if not children_of(par, i)]
            for leaf in leaves:
                chain = ancestors_or_self(par, leaf)[1:]
                curr, path, tried = 0.0, [], []
                local_margins: List[float] = []
                for a in chain:
                    ok, curr = _try_node(a, lo, acc, draft_prob, u, eps_tvd, curr, local_margins)
                    if not ok:
                        tried = [a]
                        break
                    path.append(a)
                margins.extend(local_margins)
                if best is None or len(path) > len(best[0]):
                    best = (path, tried, curr)
            path, tried, curr = best
            cur = path[-1] if path else 0
        Q = probs_row(g[lo + cur], row_thr[lo + cur], row_lse[lo + cur])
        x = _sample_last(Q, [int(token[lo + t]) for t in tried], float(u_bonus[b]), margins)
        accept_len[b] = len(path)
        path_nodes[b, :len(path)] = path
        emitted[b, :len(path)] = [int(token[lo + a]) for a in path]
        emitted[b, len(path)] = x
        terminal[b] = cur
        tvd_used[b] = curr
    return PathResult(accept_len, path_nodes, emitted, terminal, tvd_used, float(min(margins)) if margins else np.inf)


# --------------------------------------------------------------------------- whole step

def verify_step(inp, mode=WALK_SEQUENTIAL):
    """All four stages on one synthetic step (an object with the fields of the input generator's record)."""
    out, lse = tree_attention(inp.q, inp.k_tree, inp.v_tree, inp.k_cache, inp.v_cache,
                              inp.row_parent, inp.row_node_off, inp.prefix_len)
    g, row_max, row_thr, row_lse = lmhead_cfg(inp.h_cond, inp.h_uncond, inp.w, inp.cfg_scale, inp.temperature, inp.top_k)
    acc = cascade_accept(inp.node_off, inp.parent, inp.token, inp.h_cond, g, row_thr, row_lse, inp.tau_pos, inp.tau_seq)
    res = select_path(inp.node_off, inp.parent, inp.token, acc, inp.draft_prob, inp.u, inp.u_bonus, inp.eps_tvd,
                      g, row_thr, row_lse, inp.max_depth, mode)
    return dict(attn=out, attn_lse=lse, logits=g, row_max=row_max, row_thr=row_thr, row_lse=row_lse, accept=acc, path=res)
