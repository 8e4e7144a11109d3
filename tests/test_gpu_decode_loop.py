"""Chained verification steps (attention -> LM head -> acceptance -> walk -> KV commit) on the GPU
against the same chain run with the CPU checkers."""
import numpy as np
import pytest
import torch

from oracle import commit_oracle as co
from oracle import verify_oracle as vo
from paper_2605_07230_amd import workloads as wl
import parity_util as pu

pytestmark = pytest.mark.gpu


def _chain_check(config, seeds, image_tokens):
    from paper_2605_07230_amd import binding, decode
    pool = [wl.make_config(config, s) for s in seeds]
    for p in pool[1:]:
        p.w = pool[0].w                       # one model: every step projects with the same matrix
    print(f"[decode loop] {pool[0].name} seeds={seeds} image_tokens={image_tokens}", flush=True)
    loop = decode.DecodeLoop(pool, image_tokens, packed_w=pool[0].dtype == "bf16")
    res = loop.run(record=True)
    assert res.tokens >= image_tokens and res.steps == len(res.records)

    first = pool[0]
    S, cap = first.n_rows, loop.cap
    k_o = np.zeros((1, S, first.n_kv_heads, cap, first.head_dim), np.float32)
    v_o = np.zeros_like(k_o)
    k_o[0, :, :, :first.prefix_cap], v_o[0, :, :, :first.prefix_cap] = first.k_cache, first.v_cache
    plen = first.prefix_len.copy()
    row_prompt = np.zeros(S, np.int32)
    tol = pu.TOL[first.dtype]
    total = 0
    for n, r in enumerate(res.records):
        inp = pool[r["pool_index"]]
        ref, _ = vo.tree_attention(inp.q, inp.k_tree, inp.v_tree, k_o[0], v_o[0], inp.row_parent, inp.row_node_off, plen)
        assert pu.max_rel_err(r["attn_out"], ref) <= tol, f"step {n}: attention"
        g = r["logits"].astype(np.float64)
        thr, lse = r["row_thr"].astype(np.float64), r["row_lse"].astype(np.float64)
        acc = vo.cascade_accept(inp.node_off, inp.parent, inp.token, inp.h_cond, g, thr, lse, inp.tau_pos, inp.tau_seq)
        walk = vo.select_path(inp.node_off, inp.parent, inp.token, acc, inp.draft_prob, inp.u, inp.u_bonus, inp.eps_tvd,
                              g, thr, lse, inp.max_depth)
        info = f"step {n}: cos margin {acc.min_cos_margin:.2e}, walk margin {walk.min_margin:.2e}"
        assert acc.min_cos_margin > 1e-4 and walk.min_margin > 1e-6, info
        assert r["accept_len"] == walk.accept_len[0], info
        np.testing.assert_array_equal(r["path_nodes"][:, :inp.max_depth], walk.path_nodes, err_msg=info)
        np.testing.assert_array_equal(r["emitted"], walk.emitted, err_msg=info)
        assert res.emitted[n] == walk.emitted[0, :walk.accept_len[0] + 1].tolist()
        k_o, v_o, plen, ovf = co.kv_commit(inp.k_tree[None], inp.v_tree[None], k_o, v_o, inp.row_node_off, row_prompt, plen, cap,
                                           walk.accept_len, walk.path_nodes)
        assert not ovf.any()
        np.testing.assert_array_equal(r["prefix_len"], plen)
        total += int(walk.accept_len[0]) + 1
    assert total == res.tokens
    np.testing.assert_array_equal(loop.k_cache.float().cpu().numpy(), k_o)
    np.testing.assert_array_equal(loop.v_cache.float().cpu().numpy(), v_o)
    assert abs(res.tvd_per_image - sum(res.tvd_used)) < 1e-12 and res.mean_accept_len >= 0
    return res


def test_decode_loop_tiny_f32():
    res = _chain_check(0, [0, 1, 3, 7], 20)
    assert res.steps >= 4


def test_decode_loop_janus_shaped():
    res = _chain_check(1, [0, 2], 8)
    assert res.steps >= 2


@pytest.mark.parametrize("config,seeds,image_tokens", [(0, [0, 1, 3, 7], 40), (1, [0, 2, 5], 24)])
def test_pipelined_loop_equals_the_synchronous_one(config, seeds, image_tokens):
    """Reading the accepted lengths back two steps late changes nothing that is reported: same steps,
    same accepted lengths, same emitted tokens, same budget use; the cache agrees on every position the
    synchronous loop wrote (the pipelined loop may have committed up to two discarded steps beyond)."""
    from paper_2605_07230_amd import decode
    pool = [wl.make_config(config, s) for s in seeds]
    for p in pool[1:]:
        p.w = pool[0].w
    print(f"[pipelined loop] {pool[0].name} seeds={seeds}", flush=True)
    a = decode.DecodeLoop(pool, image_tokens, packed_w=pool[0].dtype == "bf16")
    ra = a.run()
    b = decode.DecodeLoop(pool, image_tokens, packed_w=pool[0].dtype == "bf16")
    rb = b.run_pipelined()
    assert ra.steps == rb.steps and ra.tokens == rb.tokens
    assert ra.accept_lens == rb.accept_lens and ra.emitted == rb.emitted and ra.tvd_used == rb.tvd_used
    n = int(a.prefix_len.max().item())
    assert torch.equal(a.k_cache[..., :n, :], b.k_cache[..., :n, :]) and torch.equal(a.v_cache[..., :n, :], b.v_cache[..., :n, :])
