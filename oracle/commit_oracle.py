"""CPU checker for the KV commit that follows a verification step.  TEST INFRASTRUCTURE ONLY.

After the walk has chosen a path, the tokens that are now part of the sequence get their keys and
values appended to the prefix cache (Preliminaries: accepted tokens are appended to the prefix;
tree decoding is repeated until the whole image sequence is formed).  The tree's root is the last
token emitted by the previous step; its key/value were computed in this step, so it is appended
first, followed by the accepted nodes in path order.  The correction / bonus token has no key or
value yet: it becomes the root of the next tree.

Plain numpy loops, no arithmetic on the values: the operation is a gather/scatter and the result is
defined bit for bit.  Shares no code with the GPU library.

Pins (tests/test_oracle_commit.py): the hand-worked tree's expected walks; chunked chain decoding
with commits equals one library causal attention over the whole sequence; untouched cache bytes;
the row that would overflow its capacity is left alone and reported.
"""
from __future__ import annotations

import numpy as np


def kv_commit(k_tree, v_tree, k_cache, v_cache, row_node_off, row_prompt, prefix_len, prefix_cap,
              accept_len, path_nodes):
    """Append root + accepted path of every row's tree to that row's cache.

    k_tree, v_tree    [L, N, Hkv, D]      this step's keys / values, rows packed by row_node_off
    k_cache, v_cache  [L, S, Hkv, cap, D] cap >= prefix_cap positions allocated
    row_prompt        [S]                 prompt whose path the row follows (guidance rows share it)
    accept_len        [B], path_nodes [B, max_depth] local node indices (as select_path writes them)

    Returns (k_cache', v_cache', prefix_len', overflow[S] bool).  A row with
    prefix_len + 1 + accept_len > prefix_cap is not modified and has overflow set.
    """
    k_out, v_out = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    S = len(prefix_len)
    new_len = np.array(prefix_len, dtype=np.int32, copy=True)
    overflow = np.zeros(S, dtype=bool)
    L = k_tree.shape[0]
    for s in range(S):
        b = int(row_prompt[s])
        n_acc = int(accept_len[b])
        nodes = [0] + [int(path_nodes[b, j]) for j in range(n_acc)]
        P = int(prefix_len[s])
        if P + len(nodes) > prefix_cap:
            overflow[s] = True
            continue
        base = int(row_node_off[s])
        n_tree = int(row_node_off[s + 1]) - base
        for j, node in enumerate(nodes):
            assert 0 <= node < n_tree
            for layer in range(L):
                k_out[layer, s, :, P + j, :] = k_tree[layer, base + node]
                v_out[layer, s, :, P + j, :] = v_tree[layer, base + node]
        new_len[s] = P + len(nodes)
    return k_out, v_out, new_len, overflow
