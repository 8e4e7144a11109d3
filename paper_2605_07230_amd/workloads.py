"""Seeded synthetic inputs for one tree-verification step.

This module only draws random numbers and lays arrays out; it holds none of the
verification arithmetic (no attention, no projection, no softmax, no cosine, no
acceptance test).  Both the CPU checker and the GPU library are fed from here so
that they see bit-identical inputs.

Shapes follow the text-to-image workloads the method is evaluated on
(Experiments / "Configuration Details"): a 576-token image with guidance scale 5
for the Janus-Pro-shaped case, a ~2400-token image with guidance scale 3 for the
Lumina-shaped case, top-k 2000, temperature 1.  No dataset item is used: every
array is synthetic.

Conventions
-----------
* A *prompt* owns one token tree.  With classifier-free guidance a prompt has two
  attention rows (conditional, then unconditional) that share the tree.
* Nodes of a tree are numbered so that ``parent[i] < i``; node 0 is the root
  (the last token already emitted), ``parent[0] == -1``.
* bf16 workloads hold float32 arrays whose values are exactly representable in
  bf16, so widening on either side is exact.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np

__all__ = ["VerifyInputs", "round_bf16", "grow_tree", "make_inputs", "make_config", "CONFIG_NAMES"]


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even), returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def grow_tree(rng: np.random.Generator, n_nodes: int, depth: int, max_children: int = 10) -> np.ndarray:
    """Score-driven tree growth, the shape a dynamic drafter produces.

    One chain of ``depth`` levels is forced first so that the depth is exact; then
    the best-scoring candidate (child rank weight ∝ rank^-1.1 × LogNormal(0, 0.5),
    multiplied down the path) is added until ``n_nodes`` exist.  Nodes are finally
    renumbered breadth-first, so ``parent[i] < i`` and siblings are contiguous.
    Returns the parent array (int32, root = -1).
    """
    assert n_nodes >= 1 and depth >= 0
    if n_nodes > 1:
        assert depth >= 1 and n_nodes >= depth + 1
    par = [-1]
    dep = [0]
    score = [1.0]
    nchild = [0]

    def child_weight(rank: int) -> float:
        return float(rank ** -1.1 * rng.lognormal(0.0, 0.5))

    def add(p: int) -> int:
        nchild[p] += 1
        par.append(p)
        dep.append(dep[p] + 1)
        score.append(score[p] * child_weight(nchild[p]))
        nchild.append(0)
        return len(par) - 1

    cur = 0
    for _ in range(min(depth, n_nodes - 1)):
        cur = add(cur)
    while len(par) < n_nodes:
        best, best_s = -1, -1.0
        for p in range(len(par)):
            if nchild[p] >= max_children or dep[p] >= depth:
                continue
            s = score[p] * (nchild[p] + 1) ** -1.1
            if s > best_s:
                best, best_s = p, s
        if best < 0:
            raise ValueError("tree cannot hold that many nodes under the depth/width limits")
        add(best)
    # breadth-first renumbering
    new_of = {0: 0}
    out_order = [0]
    level = [0]
    while level:
        nxt = []
        for p in level:
            kids = [i for i in range(len(par)) if par[i] == p]
            for c in kids:
                new_of[c] = len(out_order)
                out_order.append(c)
                nxt.append(c)
        level = nxt
    parent = np.full(len(par), -1, dtype=np.int32)
    for old, new in new_of.items():
        if old != 0:
            parent[new] = new_of[par[old]]
    assert all(parent[i] < i for i in range(1, len(parent)))
    return parent


def node_depths(parent: np.ndarray) -> np.ndarray:
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


@dataclasses.dataclass
class VerifyInputs:
    """Everything one verification step consumes (host arrays)."""

    name: str
    dtype: str                      # "f32" or "bf16": element type of q/k/v/h/w on the device
    n_prompts: int                  # B
    cfg: bool                       # conditional + unconditional rows per prompt
    n_heads: int
    n_kv_heads: int
    head_dim: int
    hidden: int
    vocab: int
    # per-prompt packing (LM head, acceptance, path selection)
    node_off: np.ndarray            # [B+1] int32
    parent: np.ndarray              # [N_c] int32, local index inside the prompt's tree
    token: np.ndarray               # [N_c] int32, token[root] = last emitted token
    # per-row packing (attention); row = prompt*(2 if cfg else 1) + {0: cond, 1: uncond}
    row_node_off: np.ndarray        # [S+1] int32
    row_parent: np.ndarray          # [N_a] int32
    prefix_len: np.ndarray          # [S] int32
    prefix_cap: int                 # allocated positions per (row, kv head) in the cache
    q: np.ndarray                   # [N_a, Hq, D] float32
    k_tree: np.ndarray              # [N_a, Hkv, D]
    v_tree: np.ndarray              # [N_a, Hkv, D]
    k_cache: np.ndarray             # [S, Hkv, prefix_cap, D]
    v_cache: np.ndarray             # [S, Hkv, prefix_cap, D]
    h_cond: np.ndarray              # [N_c, hidden]
    h_uncond: Optional[np.ndarray]  # [N_c, hidden] or None
    w: np.ndarray                   # [V, hidden]
    cfg_scale: float
    temperature: float
    top_k: int
    draft_prob: np.ndarray          # [N_c] float32 (root entry unused)
    u: np.ndarray                   # [N_c] float32 in [0,1), 24-bit
    u_bonus: np.ndarray             # [B] float32 in [0,1), 24-bit
    tau_pos: float
    tau_seq: float
    eps_tvd: float

    @property
    def n_rows(self) -> int:
        return self.n_prompts * (2 if self.cfg else 1)

    @property
    def n_nodes(self) -> int:
        return int(self.node_off[-1])

    @property
    def max_depth(self) -> int:
        m = 0
        for b in range(self.n_prompts):
            lo, hi = int(self.node_off[b]), int(self.node_off[b + 1])
            m = max(m, int(node_depths(self.parent[lo:hi]).max()))
        return m


def _uniform24(rng: np.random.Generator, n: int) -> np.ndarray:
    return (rng.integers(0, 1 << 24, size=n, dtype=np.int64).astype(np.float32) / np.float32(1 << 24)).astype(np.float32)


def _randn(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_normal(size=shape, dtype=np.float32)


def make_inputs(
    *,
    name: str,
    seed: int,
    dtype: str,
    n_prompts: int,
    cfg: bool,
    n_heads: int,
    n_kv_heads: int,
    head_dim: int,
    hidden: int,
    vocab: int,
    prefix_lens: List[int],
    trees: List[np.ndarray],
    cfg_scale: float,
    temperature: float,
    top_k: int,
    tau_pos: float,
    tau_seq: float,
    eps_tvd: float,
    token_law: str,                 # "uniform" or "zipf"
    dup_sigmas=(0.1, 0.2, 0.25),
    p_dup_parent: float = 0.2,
    p_dup_sibling: float = 0.3,
    align: float = 1.5,
    regular_dups: bool = False,
    w: Optional[np.ndarray] = None,
) -> VerifyInputs:
    """Draw one step's arrays.  See the module docstring for conventions.

    ``align`` scales a drafter/target alignment term: the conditional hidden state of a
    node is nudged towards the LM-head rows of its children's draft tokens, the way a
    trained drafter proposes tokens the target finds likely.  Without it a random LM head
    accepts nothing and the walk would never leave the root.  ``w`` hands in an LM-head matrix
    instead of drawing one.
    """
    rng = np.random.default_rng(seed)
    rows_per_prompt = 2 if cfg else 1
    S = n_prompts * rows_per_prompt
    assert len(prefix_lens) == S and len(trees) == n_prompts
    rnd = round_bf16 if dtype == "bf16" else (lambda a: np.ascontiguousarray(a, dtype=np.float32))

    node_off = np.zeros(n_prompts + 1, dtype=np.int32)
    for b, t in enumerate(trees):
        node_off[b + 1] = node_off[b] + len(t)
    parent = np.concatenate(trees).astype(np.int32)
    N_c = int(node_off[-1])

    row_node_off = np.zeros(S + 1, dtype=np.int32)
    row_parent_parts = []
    for s in range(S):
        t = trees[s // rows_per_prompt]
        row_node_off[s + 1] = row_node_off[s] + len(t)
        row_parent_parts.append(t)
    row_parent = np.concatenate(row_parent_parts).astype(np.int32)
    N_a = int(row_node_off[-1])

    # LM head (a caller sweeping seeds may hand in one matrix to share; the other draws then come
    # from a stream without the matrix's numbers in it)
    if w is None:
        w = rnd(np.float32(0.02) * _randn(rng, (vocab, hidden)))
    else:
        assert w.shape == (vocab, hidden)

    # draft tokens and the drafter's probability of each
    token = np.zeros(N_c, dtype=np.int32)
    draft_prob = np.ones(N_c, dtype=np.float32)
    if token_law == "zipf":
        ranks = np.arange(1, vocab + 1, dtype=np.float64)
        pmf = ranks ** -1.1
        pmf /= pmf.sum()
        cum = np.cumsum(pmf)
        perm = rng.permutation(vocab).astype(np.int32)
    for b in range(n_prompts):
        lo, hi = int(node_off[b]), int(node_off[b + 1])
        t = trees[b]
        token[lo] = rng.integers(0, vocab)
        for p in range(len(t)):
            kids = np.nonzero(t == p)[0]
            if len(kids) == 0:
                continue
            if token_law == "uniform":
                toks = rng.choice(vocab, size=len(kids), replace=False)
                token[lo + kids] = toks
                draft_prob[lo + kids] = np.float32(1.0 / vocab)
            else:
                chosen: list = []
                while len(chosen) < len(kids):
                    r = min(int(np.searchsorted(cum, rng.random(), side="right")), vocab - 1)
                    if r not in chosen:
                        chosen.append(r)
                token[lo + kids] = perm[np.asarray(chosen)]
                draft_prob[lo + kids] = pmf[np.asarray(chosen)].astype(np.float32)

    # hidden states with sibling / parent near-duplicates
    h_cond = np.zeros((N_c, hidden), dtype=np.float32)
    for b in range(n_prompts):
        lo, hi = int(node_off[b]), int(node_off[b + 1])
        t = trees[b]
        group_index = 0
        for i in range(len(t)):
            base = None
            if i > 0:
                sibs = [j for j in range(i) if t[j] == t[i]]
                if regular_dups:
                    # every second sibling group: second sibling = first + 0.1 noise
                    if len(sibs) == 1:
                        if group_index % 2 == 0:
                            base = h_cond[lo + sibs[0]]
                        group_index += 1
                else:
                    r = rng.random()
                    if r < p_dup_parent:
                        base = h_cond[lo + t[i]]
                    elif r < p_dup_parent + p_dup_sibling and sibs:
                        base = h_cond[lo + sibs[int(rng.integers(0, len(sibs)))]]
            if base is None:
                h_cond[lo + i] = _randn(rng, hidden)
            else:
                sigma = 0.1 if regular_dups else float(dup_sigmas[int(rng.integers(0, len(dup_sigmas)))])
                h_cond[lo + i] = base + np.float32(sigma) * _randn(rng, hidden)
    h_uncond = None
    if cfg:
        h_uncond = rnd(h_cond + np.float32(0.5) * _randn(rng, (N_c, hidden)))
    if align != 0.0:
        for b in range(n_prompts):
            lo, hi = int(node_off[b]), int(node_off[b + 1])
            t = trees[b]
            for p in range(len(t)):
                kids = np.nonzero(t == p)[0]
                for c in kids:
                    gain = np.float32(align * rng.uniform(0.4, 1.6))
                    h_cond[lo + p] += gain * w[token[lo + c]] / np.float32(0.02 * 0.02 * hidden)
    h_cond = rnd(h_cond)

    # attention operands
    prefix_cap = int(max(prefix_lens))
    q = rnd(_randn(rng, (N_a, n_heads, head_dim)))
    k_tree = rnd(_randn(rng, (N_a, n_kv_heads, head_dim)))
    v_tree = rnd(_randn(rng, (N_a, n_kv_heads, head_dim)))
    k_cache = rnd(_randn(rng, (S, n_kv_heads, prefix_cap, head_dim)))
    v_cache = rnd(_randn(rng, (S, n_kv_heads, prefix_cap, head_dim)))

    return VerifyInputs(
        name=name, dtype=dtype, n_prompts=n_prompts, cfg=cfg, n_heads=n_heads, n_kv_heads=n_kv_heads,
        head_dim=head_dim, hidden=hidden, vocab=vocab, node_off=node_off, parent=parent, token=token,
        row_node_off=row_node_off, row_parent=row_parent,
        prefix_len=np.asarray(prefix_lens, dtype=np.int32), prefix_cap=prefix_cap,
        q=q, k_tree=k_tree, v_tree=v_tree, k_cache=k_cache, v_cache=v_cache,
        h_cond=h_cond, h_uncond=h_uncond, w=w, cfg_scale=float(cfg_scale), temperature=float(temperature),
        top_k=int(top_k), draft_prob=draft_prob, u=_uniform24(rng, N_c), u_bonus=_uniform24(rng, n_prompts),
        tau_pos=float(tau_pos), tau_seq=float(tau_seq), eps_tvd=float(eps_tvd),
    )


def complete_binary_tree(depth: int) -> np.ndarray:
    n = (1 << (depth + 1)) - 1
    parent = np.full(n, -1, dtype=np.int32)
    for i in range(1, n):
        parent[i] = (i - 1) // 2
    return parent


CONFIG_NAMES = ["tiny_f32", "janus_pro_7b", "lumina_mgpt_7b_768", "janus_batched", "stress_1024px"]


def make_config(index: int, seed: int = 0, **overrides) -> VerifyInputs:
    """The five benchmark configurations, in order.

    0 tiny fp32 (15-node complete binary tree, one sequence, no guidance);
    1 Janus-Pro-7B-shaped (24 text + 288 image prefix tokens, guidance 5, 60-node tree);
    2 Lumina-mGPT-7B-768-shaped (1289-token prefix, vocabulary 65536, guidance 3);
    3 batched Janus-shaped (8 prompts, ragged prefixes and trees);
    4 stress (4 prompts, 4200-token prefix, 256-node trees of depth 10).
    """
    rng = np.random.default_rng([seed, 977, index])
    if index == 0:
        kw = dict(name=CONFIG_NAMES[0], dtype="f32", n_prompts=1, cfg=False, n_heads=8, n_kv_heads=8, head_dim=64,
                  hidden=512, vocab=4096, prefix_lens=[256], trees=[complete_binary_tree(3)], cfg_scale=1.0,
                  temperature=1.0, top_k=0, tau_pos=0.9, tau_seq=0.9, eps_tvd=0.5, token_law="uniform",
                  align=0.0, regular_dups=True)
    elif index == 1:
        kw = dict(name=CONFIG_NAMES[1], dtype="bf16", n_prompts=1, cfg=True, n_heads=32, n_kv_heads=32, head_dim=128,
                  hidden=4096, vocab=16384, prefix_lens=[312, 312], trees=[grow_tree(rng, 60, 6)], cfg_scale=5.0,
                  temperature=1.0, top_k=2000, tau_pos=0.85, tau_seq=0.5, eps_tvd=0.5, token_law="zipf")
    elif index == 2:
        kw = dict(name=CONFIG_NAMES[2], dtype="bf16", n_prompts=1, cfg=True, n_heads=32, n_kv_heads=32, head_dim=128,
                  hidden=4096, vocab=65536, prefix_lens=[1289, 1289], trees=[grow_tree(rng, 60, 6)], cfg_scale=3.0,
                  temperature=1.0, top_k=2000, tau_pos=0.95, tau_seq=0.925, eps_tvd=0.5, token_law="zipf")
    elif index == 3:
        B = 8
        trees = [grow_tree(rng, int(rng.integers(40, 81)), int(rng.integers(4, 8))) for _ in range(B)]
        plens: List[int] = []
        for _ in range(B):
            p = int(rng.integers(100, 601))
            plens += [p, p]
        kw = dict(name=CONFIG_NAMES[3], dtype="bf16", n_prompts=B, cfg=True, n_heads=32, n_kv_heads=32, head_dim=128,
                  hidden=4096, vocab=16384, prefix_lens=plens, trees=trees, cfg_scale=5.0, temperature=1.0,
                  top_k=2000, tau_pos=0.85, tau_seq=0.5, eps_tvd=0.5, token_law="zipf")
    elif index == 4:
        B = 4
        sig = tuple(float(np.sqrt(1.0 / c ** 2 - 1.0)) for c in (0.85, 0.92, 0.97, 0.99))
        kw = dict(name=CONFIG_NAMES[4], dtype="bf16", n_prompts=B, cfg=True, n_heads=32, n_kv_heads=32, head_dim=128,
                  hidden=4096, vocab=65536, prefix_lens=[4200] * (2 * B), trees=[grow_tree(rng, 256, 10) for _ in range(B)],
                  cfg_scale=3.0, temperature=1.0, top_k=2000, tau_pos=0.9, tau_seq=0.9, eps_tvd=0.5,
                  token_law="zipf", dup_sigmas=sig)
    else:
        raise ValueError("config index must be 0..4")
    kw.update(overrides)
    return make_inputs(seed=seed, **kw)


# ------------------------------------------------------------------------------------------------
# inputs of the KV commit that follows a step

@dataclasses.dataclass
class CommitInputs:
    """Multi-layer tree keys / values and a prefix cache with room to append (host arrays)."""

    n_layers: int
    k_tree: np.ndarray        # [L, N_a, Hkv, D]
    v_tree: np.ndarray
    k_cache: np.ndarray       # [L, S, Hkv, cap, D]
    v_cache: np.ndarray
    prefix_cap: int
    row_prompt: np.ndarray    # [S] int32
    accept_len: np.ndarray    # [B] int32     a seeded root-to-node walk per prompt
    path_nodes: np.ndarray    # [B, max_depth] int32, -1 padded


def random_paths(inp: VerifyInputs, seed: int = 0):
    """For every prompt a seeded walk from the root: at each node stop w.p. 0.25, else descend to a
    random child.  Tree structure only; stands in for what the path selection would return."""
    rng = np.random.default_rng(seed + 4242)
    B, md = inp.n_prompts, max(inp.max_depth, 1)
    accept_len = np.zeros(B, dtype=np.int32)
    path_nodes = -np.ones((B, md), dtype=np.int32)
    for b in range(B):
        par = inp.parent[inp.node_off[b]:inp.node_off[b + 1]]
        cur, n = 0, 0
        while True:
            kids = np.nonzero(par == cur)[0]
            if len(kids) == 0 or rng.random() < 0.25:
                break
            cur = int(kids[int(rng.integers(0, len(kids)))])
            path_nodes[b, n] = cur
            n += 1
        accept_len[b] = n
    return accept_len, path_nodes


def make_commit_inputs(inp: VerifyInputs, n_layers: int, seed: int = 0, slack: int = 3) -> CommitInputs:
    """Layer 0 reuses the step's own tree keys / values and cache contents; further layers are fresh
    N(0,1) draws.  The cache gets max_depth + 1 + slack positions beyond the longest prefix."""
    rng = np.random.default_rng(seed + 977)
    rnd = round_bf16 if inp.dtype == "bf16" else (lambda x: x)
    S, Hkv, D = inp.n_rows, inp.n_kv_heads, inp.head_dim
    N_a = inp.q.shape[0]
    cap = inp.prefix_cap + inp.max_depth + 1 + slack
    k_tree = np.empty((n_layers, N_a, Hkv, D), dtype=np.float32)
    v_tree = np.empty_like(k_tree)
    k_cache = np.zeros((n_layers, S, Hkv, cap, D), dtype=np.float32)
    v_cache = np.zeros_like(k_cache)
    for layer in range(n_layers):
        if layer == 0:
            k_tree[0], v_tree[0] = inp.k_tree, inp.v_tree
            k_cache[0, :, :, :inp.prefix_cap], v_cache[0, :, :, :inp.prefix_cap] = inp.k_cache, inp.v_cache
        else:
            k_tree[layer], v_tree[layer] = rnd(_randn(rng, (N_a, Hkv, D))), rnd(_randn(rng, (N_a, Hkv, D)))
            k_cache[layer, :, :, :inp.prefix_cap] = rnd(_randn(rng, (S, Hkv, inp.prefix_cap, D)))
            v_cache[layer, :, :, :inp.prefix_cap] = rnd(_randn(rng, (S, Hkv, inp.prefix_cap, D)))
    rows_per_prompt = 2 if inp.cfg else 1
    row_prompt = (np.arange(S) // rows_per_prompt).astype(np.int32)
    accept_len, path_nodes = random_paths(inp, seed)
    return CommitInputs(n_layers=n_layers, k_tree=k_tree, v_tree=v_tree, k_cache=k_cache, v_cache=v_cache, prefix_cap=cap,
                        row_prompt=row_prompt, accept_len=accept_len, path_nodes=path_nodes)


# ------------------------------------------------------------------------------------------------
# full drafter distributions for the residual walk

def make_draft_dist(inp: VerifyInputs, seed: int = 0, zipf_s: float = 1.1) -> np.ndarray:
    """[N_c, V] float32: the children of one parent share a row, a Zipf(zipf_s) law over a vocabulary
    permutation drawn per parent, with each child's own token moved to a seeded rank among the
    first 32 (so drafted tokens carry visible drafter mass).  Root rows are uniform (never read)."""
    rng = np.random.default_rng(seed + 31337)
    V, N = inp.vocab, inp.n_nodes
    ranks = np.arange(1, V + 1, dtype=np.float64)
    pmf = ranks ** (-zipf_s)
    pmf = (pmf / pmf.sum()).astype(np.float32)
    out = np.empty((N, V), dtype=np.float32)
    for b in range(inp.n_prompts):
        lo, hi = int(inp.node_off[b]), int(inp.node_off[b + 1])
        par = inp.parent[lo:hi]
        out[lo] = np.float32(1.0 / V)
        for p in range(hi - lo):
            kids = np.nonzero(par == p)[0]
            if len(kids) == 0:
                continue
            perm = rng.permutation(V)
            # move the children's tokens to distinct early ranks
            slots = rng.choice(min(32, V), size=min(len(kids), min(32, V)), replace=False)
            for kid, slot in zip(kids, slots):
                t = int(inp.token[lo + kid])
                j = int(np.nonzero(perm == t)[0][0])
                perm[j], perm[slot] = perm[slot], perm[j]
            row = np.empty(V, dtype=np.float32)
            row[perm] = pmf
            out[lo + kids] = row
    return out


# ------------------------------------------------------------------------------------------------
# target feature sequences for the Eq. 4 weight mask

def make_feature_sequence(n_seqs: int, seq_len: int, hidden: int, dtype: str = "bf16", seed: int = 0,
                          p_stay: float = 0.6, sigmas=(0.1, 0.2, 0.3, 0.6)) -> np.ndarray:
    """[n_seqs, seq_len, hidden] float32 (bf16-rounded for dtype "bf16"): a sequence of image
    positions in which, with probability p_stay, a position's feature is its predecessor's plus
    sigma * N(0,1) (a semantically uniform region; cos about 0.995 / 0.98 / 0.96 / 0.86) and
    otherwise a fresh N(0,1) draw (a region boundary)."""
    rng = np.random.default_rng(seed + 555)
    out = np.empty((n_seqs, seq_len, hidden), dtype=np.float32)
    for b in range(n_seqs):
        for k in range(seq_len):
            if k > 0 and rng.random() < p_stay:
                sigma = np.float32(sigmas[int(rng.integers(0, len(sigmas)))])
                out[b, k] = out[b, k - 1] + sigma * _randn(rng, hidden)
            else:
                out[b, k] = _randn(rng, hidden)
    return round_bf16(out) if dtype == "bf16" else out
