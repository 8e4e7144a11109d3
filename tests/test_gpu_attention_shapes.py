"""GPU parity of tree_verify_attn over the shapes that select each of its bf16 kernels, and of the
whole step on trees of several hundred to 1024 nodes.  Everything goes through the C ABI; every
(row, head) pair and every node is compared with the CPU checker unless stated otherwise.

Which kernel a shape reaches (units = rows x kv heads x 64-query blocks, M = nodes x heads per kv head):
  M <= 128 and units <= 128                 query-split kernel
  M <= 128, 128 < units < 512               key-split kernel, two (head_dim 128) or four (64) key groups,
                                            split over workgroups + merge kernel when a row has > 16 key tiles
  M <= 128, units >= 512                    key-split kernel, one (128) or two (64) key groups, never split
  M > 128                                   large-tree kernel (split + merge when there are < 256 units)
"""
import numpy as np
import pytest
import torch

from paper_2605_07230_amd import binding
from paper_2605_07230_amd import workloads as wl

import parity_util as pu

pytestmark = pytest.mark.gpu


def _inputs(seed, *, n_prompts, cfg, n_heads, n_kv_heads, head_dim, prefix_lens, tree_sizes, depth=5, width=8,
            hidden=128, vocab=512):
    rng = np.random.default_rng(seed)
    trees = [wl.grow_tree(rng, n, min(depth, max(n - 1, 0)), width) for n in tree_sizes]
    return wl.make_inputs(name="attn_shape", seed=seed, dtype="bf16", n_prompts=n_prompts, cfg=cfg, n_heads=n_heads,
                          n_kv_heads=n_kv_heads, head_dim=head_dim, hidden=hidden, vocab=vocab, prefix_lens=prefix_lens,
                          trees=trees, cfg_scale=3.0, temperature=1.0, top_k=50, tau_pos=0.9, tau_seq=0.9, eps_tvd=0.5,
                          token_law="zipf")


def _run_attention(inp, **kw):
    print(f"[attn shape] rows={inp.n_rows} heads={inp.n_heads}/{inp.n_kv_heads} d={inp.head_dim} "
          f"prefix={inp.prefix_len.tolist()} trees={np.diff(inp.node_off).tolist()}", flush=True)
    ds = binding.DeviceStep(inp, **kw)
    ds.attn_out.fill_(float("nan"))          # an unwritten output must not pass
    ds.attn_lse.fill_(float("nan"))
    ds.attn()
    torch.cuda.synchronize()
    return ds


@pytest.mark.parametrize("head_dim,prefix_lens", [
    (128, [1500, 37, 700, 1100, 260]),     # 24 key tiles: two key groups per workgroup, 2 splits + merge
    (128, [800, 0, 64, 513, 300]),         # at most 14 key tiles: two key groups, no split (an empty prefix among them)
    (64, [1500, 37, 700, 1100, 260]),      # four key groups, 2 splits + merge
    (64, [640, 65, 1, 333, 128]),          # four key groups, no split
])
def test_key_split_kernel_with_scarce_workgroups(head_dim, prefix_lens):
    # 5 rows x 32 kv heads x one 64-query block = 160 units
    inp = _inputs(31, n_prompts=5, cfg=False, n_heads=32, n_kv_heads=32, head_dim=head_dim, prefix_lens=prefix_lens,
                  tree_sizes=[60, 41, 64, 17, 55])
    ds = _run_attention(inp)
    assert ds.ctx.device_status() == binding.OK
    pu.check_attention(inp, ds)


def test_key_split_kernel_grouped_heads_two_query_blocks_split():
    # 4 query heads per kv head x 30 nodes = 120 query rows: two 64-query blocks (the second ragged) per
    # (row, kv head); 10 rows x 8 kv heads x 2 = 160 units; 20 key tiles: 2 splits + merge
    inp = _inputs(32, n_prompts=5, cfg=True, n_heads=32, n_kv_heads=8, head_dim=128,
                  prefix_lens=[1200, 1200, 90, 90, 777, 777, 1000, 1000, 5, 5], tree_sizes=[30, 22, 30, 9, 27])
    ds = _run_attention(inp)
    assert ds.ctx.device_status() == binding.OK
    pu.check_attention(inp, ds)


def test_key_split_kernel_head_dim_64_many_workgroups():
    # 16 rows x 32 kv heads = 512 units: two key groups per workgroup (head_dim 64), no split
    inp = _inputs(33, n_prompts=8, cfg=True, n_heads=32, n_kv_heads=32, head_dim=64,
                  prefix_lens=[p for p in (200, 17, 130, 64, 99, 181, 0, 150) for _ in range(2)],
                  tree_sizes=[40, 64, 13, 33, 60, 25, 48, 1])
    ds = _run_attention(inp)
    assert ds.ctx.device_status() == binding.OK
    pu.check_attention(inp, ds, heads=[0, 9, 22, 31])


def test_large_tree_kernel_split_over_workgroups_with_merge():
    # 2 rows x 2 kv heads x one 256-row block = 4 units: the large-tree kernel splits the keys 16-fold + merge
    inp = _inputs(34, n_prompts=1, cfg=True, n_heads=4, n_kv_heads=2, head_dim=128, prefix_lens=[2100, 2100],
                  tree_sizes=[100], depth=7)
    ds = _run_attention(inp)
    assert ds.ctx.device_status() == binding.OK
    pu.check_attention(inp, ds)


@pytest.mark.parametrize("n_nodes,depth,width,head_dim", [(600, 12, 16, 128), (1024, 20, 40, 64), (1024, 63, 64, 128)])
def test_trees_of_several_hundred_nodes_whole_step(n_nodes, depth, width, head_dim):
    """Attention (several 256-row query blocks, up to 16 tree key tiles), acceptance beyond 256 nodes,
    sibling groups wider than one 64-node chunk boundary, and both walks over up to 16 node chunks."""
    inp = _inputs(35 + n_nodes + depth, n_prompts=1, cfg=True, n_heads=4, n_kv_heads=2, head_dim=head_dim,
                  prefix_lens=[150, 91], tree_sizes=[n_nodes], depth=depth, width=width, hidden=256, vocab=1024)
    assert inp.max_depth == depth
    ds = pu.run_gpu_step(inp)
    pu.check_attention(inp, ds)
    pu.check_lmhead(inp, ds, nodes=np.arange(0, n_nodes, 7))
    pu.check_accept_and_path(inp, ds, require_margin=False)
    ds.select(binding.WALK_LONGEST)
    torch.cuda.synchronize()
    pu.check_accept_and_path(inp, ds, binding.WALK_LONGEST, require_margin=False)
    # a harsher drafter makes the sequential walk try (and reject) many siblings per level
    ds.draft_prob = (ds.draft_prob * 4.0).clamp(max=1.0)
    inp.draft_prob = ds.draft_prob.cpu().numpy()
    for mode in (binding.WALK_SEQUENTIAL, binding.WALK_LONGEST):
        ds.select(mode)
        torch.cuda.synchronize()
        pu.check_accept_and_path(inp, ds, mode, require_margin=False)


def test_tree_larger_than_the_stated_bound_is_flagged_and_not_computed():
    """The host understates max_nodes_per_tree: the oversize tree is flagged (CASCADE_ETREE), its
    attention rows are zeros with lse = -inf, its acceptance scalars beyond the bound are zeros; the
    tree that fits is still verified correctly; nothing faults."""
    for sizes, plens, bound in [([23, 9], [70, 70, 5, 5], 16),          # query-split kernel
                                ([150, 100], [300, 300, 40, 40], 128)]:  # key-split kernel (bound) vs 150 nodes
        inp = _inputs(40, n_prompts=2, cfg=True, n_heads=4, n_kv_heads=2, head_dim=64, prefix_lens=plens,
                      tree_sizes=sizes, depth=4 if sizes[0] < 100 else 8, width=16)
        ds = _run_attention(inp, max_tree=bound)
        ds.lmhead()
        for t in (ds.q_tok, ds.m_int, ds.m_conv, ds.cos_parent):
            t.fill_(float("nan"))
        ds.accept()
        ds.select()
        torch.cuda.synchronize()
        assert ds.ctx.device_status() == binding.ETREE
        assert ds.ctx.device_status() == binding.OK
        big = sizes[0]
        out = ds.attn_out.float().cpu().numpy()
        lse = ds.attn_lse.cpu().numpy()
        for s in (0, 1):                                   # both rows of the oversize prompt
            lo, hi = int(inp.row_node_off[s]), int(inp.row_node_off[s + 1])
            assert np.all(out[lo:hi] == 0.0) and np.all(np.isneginf(lse[lo:hi]))
        pu.check_attention(inp, ds, rows=[2, 3])           # the tree that fits
        q_tok = ds.q_tok.cpu().numpy()
        assert np.all(q_tok[bound:big] == 0.0) and np.all(ds.n_int.cpu().numpy()[bound:big] == 0)
        assert np.all(np.isfinite(q_tok))
        # the second prompt's walk is untouched by the first one's flag
        acc = pu.vo.cascade_accept(inp.node_off, inp.parent, inp.token, inp.h_cond, ds.logits.cpu().numpy().astype(np.float64),
                                   ds.row_thr.cpu().numpy().astype(np.float64), ds.row_lse.cpu().numpy().astype(np.float64),
                                   inp.tau_pos, inp.tau_seq)
        lo2 = int(inp.node_off[1])
        np.testing.assert_array_equal(ds.n_int.cpu().numpy()[lo2:], acc.n_int[lo2:])
        np.testing.assert_allclose(ds.q_tok.cpu().numpy()[lo2:], acc.q_tok[lo2:], rtol=1e-4, atol=1e-9)
