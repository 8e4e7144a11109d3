"""Pins of the KV-commit checker (oracle/commit_oracle.py) against things it does not compute itself."""
import ast
import json
import os

import numpy as np
import torch

from oracle import commit_oracle as co
from oracle import verify_oracle as vo

GOLD = os.path.join(os.path.dirname(__file__), "golden", "handworked_tree.json")


def _gold():
    g = json.load(open(GOLD))
    walks = g["expected_walks"]
    if isinstance(walks, str):
        walks = ast.literal_eval(walks)
    return g, walks


def test_handworked_walks_land_in_path_order():
    """Keys carry their node index as value, so the cache shows which node sits at which position."""
    g, walks = _gold()
    parent = np.array(g["parent"], np.int32)
    T = len(parent)
    L, Hkv, D, P, cap = 2, 2, 4, 3, 12
    k_tree = np.zeros((L, T, Hkv, D), np.float32)
    v_tree = np.zeros((L, T, Hkv, D), np.float32)
    for layer in range(L):
        for n in range(T):
            k_tree[layer, n] = 100 * layer + n
            v_tree[layer, n] = -(100 * layer + n)
    k_cache = np.full((L, 1, Hkv, cap, D), 7777.0, np.float32)
    v_cache = np.full((L, 1, Hkv, cap, D), 8888.0, np.float32)
    for w in walks:
        path = list(w["path"])
        path_nodes = -np.ones((1, 6), np.int32)
        path_nodes[0, :len(path)] = path
        k2, v2, new_len, ovf = co.kv_commit(k_tree, v_tree, k_cache, v_cache, np.array([0, T], np.int32), np.array([0], np.int32),
                                            np.array([P], np.int32), cap, np.array([w["accept_len"]], np.int32), path_nodes)
        assert not ovf[0]
        assert new_len[0] == P + 1 + w["accept_len"]
        expect = [0] + path   # root first, then the accepted nodes in walk order
        for layer in range(L):
            got = k2[layer, 0, 0, P:new_len[0], 0].tolist()
            assert got == [100 * layer + n for n in expect]
            gotv = v2[layer, 0, 1, P:new_len[0], 3].tolist()
            assert gotv == [-(100 * layer + n) for n in expect]
        # nothing else moved
        assert np.all(k2[:, :, :, :P] == 7777.0) and np.all(k2[:, :, :, new_len[0]:] == 7777.0)
        assert np.all(v2[:, :, :, :P] == 8888.0) and np.all(v2[:, :, :, new_len[0]:] == 8888.0)


def test_chunked_chain_decoding_equals_library_causal_attention():
    """Decode a sequence in chunks: each chunk is a chain tree whose root is the last committed
    token's successor; after every chunk all of it is committed.  Outputs must equal one causal
    attention over the whole sequence computed by a library routine."""
    rng = np.random.default_rng(5)
    n, Hq, Hkv, D = 23, 4, 2, 8
    q = rng.standard_normal((n, Hq, D))
    k = rng.standard_normal((n, Hkv, D))
    v = rng.standard_normal((n, Hkv, D))
    # library result
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, Hq // Hkv, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, Hq // Hkv, axis=1)).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()

    cap = n + 2
    k_cache = np.zeros((1, 1, Hkv, cap, D))
    v_cache = np.zeros((1, 1, Hkv, cap, D))
    plen = np.array([0], np.int32)
    out = np.zeros_like(q)
    pos, chunks = 0, [5, 1, 7, 4, 6]
    assert sum(chunks) == n
    for c in chunks:
        parent = np.arange(-1, c - 1, dtype=np.int32)        # a chain
        off = np.array([0, c], np.int32)
        o, _ = vo.tree_attention(q[pos:pos + c], k[pos:pos + c], v[pos:pos + c], k_cache[0], v_cache[0], parent, off, plen)
        out[pos:pos + c] = o
        path = -np.ones((1, 8), np.int32)
        path[0, :c - 1] = np.arange(1, c)
        k_cache, v_cache, plen, ovf = co.kv_commit(k[None, pos:pos + c], v[None, pos:pos + c], k_cache, v_cache, off,
                                                   np.array([0], np.int32), plen, cap, np.array([c - 1], np.int32), path)
        assert not ovf[0]
        pos += c
    assert plen[0] == n
    np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)
    # the cache now IS the sequence, in order
    np.testing.assert_array_equal(k_cache[0, 0, :, :n].transpose(1, 0, 2), k)
    np.testing.assert_array_equal(v_cache[0, 0, :, :n].transpose(1, 0, 2), v)


def test_branching_tree_commit_then_attend_matches_in_tree_attention():
    """A node's in-tree attention (prefix + ancestors + itself) equals the attention of a fresh
    one-node tree holding that node, after its ancestors were committed."""
    rng = np.random.default_rng(11)
    parent = np.array([-1, 0, 0, 1, 1, 2, 4, 4, 6], np.int32)
    T, Hq, Hkv, D, P, cap = len(parent), 2, 2, 4, 6, 16
    q = rng.standard_normal((T, Hq, D))
    k = rng.standard_normal((T, Hkv, D))
    v = rng.standard_normal((T, Hkv, D))
    kc = rng.standard_normal((1, Hkv, cap, D))
    vc = rng.standard_normal((1, Hkv, cap, D))
    off = np.array([0, T], np.int32)
    plen = np.array([P], np.int32)
    full, _ = vo.tree_attention(q, k, v, kc, vc, parent, off, plen)
    node = 8
    anc = vo.ancestors_or_self(parent, node)          # [0, 1, 4, 6, 8]
    path = -np.ones((1, 5), np.int32)
    path[0, :len(anc) - 2] = anc[1:-1]                  # commit root .. parent(node)
    k2, v2, plen2, _ = co.kv_commit(k[None], v[None], kc[None], vc[None], off, np.array([0], np.int32), plen, cap,
                                    np.array([len(anc) - 2], np.int32), path)
    one, _ = vo.tree_attention(q[node:node + 1], k[node:node + 1], v[node:node + 1], k2[0], v2[0], np.array([-1], np.int32),
                               np.array([0, 1], np.int32), plen2)
    np.testing.assert_allclose(one[0], full[node], rtol=1e-12, atol=1e-13)
    # committing a sibling branch instead gives a different result (the mask matters)
    path_wrong = -np.ones((1, 5), np.int32)
    path_wrong[0, :3] = [2, 5, 6]
    k3, v3, plen3, _ = co.kv_commit(k[None], v[None], kc[None], vc[None], off, np.array([0], np.int32), plen, cap,
                                    np.array([3], np.int32), path_wrong)
    other, _ = vo.tree_attention(q[node:node + 1], k[node:node + 1], v[node:node + 1], k3[0], v3[0], np.array([-1], np.int32),
                                 np.array([0, 1], np.int32), plen3)
    assert np.abs(other[0] - full[node]).max() > 1e-3


def test_guidance_rows_share_the_path_and_overflow_is_reported():
    rng = np.random.default_rng(2)
    T, Hkv, D, cap = 5, 1, 2, 10
    off = np.array([0, T, 2 * T, 3 * T], np.int32)
    row_prompt = np.array([0, 0, 1], np.int32)
    k = rng.standard_normal((1, 3 * T, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((1, 3 * T, Hkv, D)).astype(np.float32)
    kc = np.zeros((1, 3, Hkv, cap, D), np.float32)
    vc = np.zeros((1, 3, Hkv, cap, D), np.float32)
    plen = np.array([4, 8, 2], np.int32)     # row 1: 8 + 1 + 2 > 10 -> overflow
    accept_len = np.array([2, 0], np.int32)
    path = np.array([[1, 3, -1], [-1, -1, -1]], np.int32)
    k2, v2, new_len, ovf = co.kv_commit(k, v, kc, vc, off, row_prompt, plen, cap, accept_len, path)
    assert ovf.tolist() == [False, True, False]
    assert new_len.tolist() == [7, 8, 3]
    np.testing.assert_array_equal(k2[0, 0, 0, 4:7], k[0, [0, 1, 3], 0])
    np.testing.assert_array_equal(k2[0, 1], kc[0, 1])                     # untouched
    np.testing.assert_array_equal(v2[0, 2, 0, 2:3], v[0, [2 * T], 0])    # root only
    assert np.all(k2[0, 2, :, 3:] == 0)
