"""GPU parity: the HIP library (through its C ABI) against the CPU checker on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2605_07230_amd import binding
from paper_2605_07230_amd import workloads as wl

import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_f32_whole_step(seed):
    inp = wl.make_config(0, seed)
    ds = pu.run_gpu_step(inp)
    pu.check_attention(inp, ds)
    pu.check_lmhead(inp, ds)
    pu.check_accept_and_path(inp, ds)


@pytest.mark.parametrize("variant", ["topk", "harsh_drafter", "conv_dups", "longest", "strict", "zero_budget"])
def test_tiny_f32_variants(variant):
    kw = {}
    if variant == "topk":
        kw = dict(top_k=256)
    inp = wl.make_config(0, 3, **kw)
    mode = binding.WALK_SEQUENTIAL
    if variant == "harsh_drafter":
        inp.draft_prob = (inp.draft_prob * 3).astype(np.float32)           # q/p around 1/3: many rejections
    if variant == "conv_dups":
        rng = np.random.default_rng(5)
        for a, c in [(1, 3), (2, 6), (5, 11)]:                               # child nearly equal to its parent
            inp.h_cond[c] = inp.h_cond[a] + np.float32(0.1) * rng.standard_normal(inp.hidden).astype(np.float32)
        inp.draft_prob = (inp.draft_prob * 2).astype(np.float32)
    if variant == "longest":
        inp.draft_prob = (inp.draft_prob * 2).astype(np.float32)
        mode = binding.WALK_LONGEST
    if variant == "strict":
        inp.tau_pos = inp.tau_seq = 2.0
    if variant == "zero_budget":
        inp.eps_tvd = 0.0
    ds = pu.run_gpu_step(inp, mode)
    pu.check_lmhead(inp, ds)
    acc, res = pu.check_accept_and_path(inp, ds, mode)
    if variant in ("strict", "zero_budget"):
        assert np.all(ds.tvd_used.cpu().numpy() == 0)
    if variant == "conv_dups":
        assert acc.n_conv.sum() >= 3


@pytest.mark.parametrize("seed,packed", [(0, False), (3, False), (0, True), (5, True)])
def test_janus_shaped_bf16_whole_step(seed, packed):
    inp = wl.make_config(1, seed)
    ds = pu.run_gpu_step(inp, packed_w=packed)
    pu.check_attention(inp, ds, heads=[0, 5, 31])
    pu.check_lmhead(inp, ds)
    pu.check_accept_and_path(inp, ds)
    ds.select(binding.WALK_LONGEST)
    pu.check_accept_and_path(inp, ds, binding.WALK_LONGEST)


def test_janus_shaped_threshold_pairs():
    inp = wl.make_config(1, 4)
    ds = pu.run_gpu_step(inp)
    for tp, ts in [(0.85, 0.5), (0.9, 0.9), (2.0, 2.0), (0.85, 2.0), (2.0, 0.5)]:
        ds.accept(tp, ts)
        ds.select()
        pu.check_accept_and_path(inp, ds, tau_pos=tp, tau_seq=ts)


def test_lumina_shaped_bf16_sampled():
    inp = wl.make_config(2, 0)
    ds = pu.run_gpu_step(inp, packed_w=True)
    pu.check_attention(inp, ds, heads=[3, 17])
    pu.check_lmhead(inp, ds, nodes=[0, 1, 7, 30, 59])
    pu.check_accept_and_path(inp, ds)


def test_batched_ragged_bf16():
    inp = wl.make_config(3, 0)
    ds = pu.run_gpu_step(inp, packed_w=True)
    pu.check_attention(inp, ds, heads=[0, 13, 31])          # all 16 rows: the work-rank dispatch permutes every row
    nodes = np.unique(np.concatenate([inp.node_off[:-1], inp.node_off[1:] - 1, np.arange(0, inp.n_nodes, 37)]))
    pu.check_lmhead(inp, ds, nodes=nodes)
    pu.check_accept_and_path(inp, ds)


def test_stress_bf16_sampled():
    inp = wl.make_config(4, 0)
    ds = pu.run_gpu_step(inp, packed_w=True)
    pu.check_attention(inp, ds, rows=[0, 7], heads=[9])                     # two (row, head) pairs, every node
    worst, n_cmp = pu.check_attention_node_sample(inp, ds, n_picks=4, seed=1)   # every (row, head), ~30 nodes each
    print(f"[stress] attention: {n_cmp} (node, row, head) outputs compared, worst rel err {worst:.2e}", flush=True)
    pu.check_lmhead(inp, ds, nodes=[0, 1, 255, 256, 700, 1023])              # whole rows + statistics
    pu.check_logits_columns(inp, ds, n_cols=512, seed=2)                     # all 1024 nodes, every row tile
    for tau in (0.8, 0.9, 0.95):
        ds.accept(tau, tau)
        ds.select()
        pu.check_accept_and_path(inp, ds, tau_pos=tau, tau_seq=tau)


# ---------------------------------------------------------------------------------- edge cases

def _small_bf16(seed, **kw):
    rng = np.random.default_rng(seed)
    base = dict(name="edge", dtype="bf16", n_prompts=2, cfg=True, n_heads=4, n_kv_heads=2, head_dim=64, hidden=256,
                vocab=512, prefix_lens=[70, 70, 5, 5], trees=[wl.grow_tree(rng, 23, 4, 4), wl.grow_tree(rng, 9, 3, 3)],
                cfg_scale=3.0, temperature=1.0, top_k=50, tau_pos=0.9, tau_seq=0.9, eps_tvd=0.5, token_law="zipf")
    base.update(kw)
    return wl.make_inputs(seed=seed, **base)


def test_grouped_heads_head_dim_64_and_ragged_tail():
    inp = _small_bf16(0)
    ds = pu.run_gpu_step(inp)
    pu.check_attention(inp, ds)
    pu.check_lmhead(inp, ds)
    pu.check_accept_and_path(inp, ds)


def test_empty_prefix_and_root_only_tree():
    rng = np.random.default_rng(1)
    inp = _small_bf16(1, prefix_lens=[0, 0, 33, 33], trees=[np.array([-1], np.int32), wl.grow_tree(rng, 70, 5, 6)])
    ds = pu.run_gpu_step(inp)
    pu.check_attention(inp, ds)
    pu.check_lmhead(inp, ds)
    acc, res = pu.check_accept_and_path(inp, ds)
    assert res.accept_len[0] == 0 and res.terminal[0] == 0


def test_wide_tree_spanning_several_query_blocks_and_key_tiles():
    rng = np.random.default_rng(2)
    inp = _small_bf16(2, n_prompts=1, prefix_lens=[200, 200], trees=[wl.grow_tree(rng, 150, 7, 8)], head_dim=128,
                      n_heads=2, n_kv_heads=2)
    ds = pu.run_gpu_step(inp)
    pu.check_attention(inp, ds)
    pu.check_accept_and_path(inp, ds)


def test_large_query_block_grouped_heads_head_dim_64():
    # 4 query heads per kv head x 90 nodes = 360 query rows per (row, kv head): the large-tree kernel with
    # a ragged last query block, several tree tiles and a prefix that ends inside a tile
    rng = np.random.default_rng(8)
    inp = _small_bf16(8, n_prompts=1, prefix_lens=[150, 91], trees=[wl.grow_tree(rng, 90, 6, 8)], head_dim=64,
                      n_heads=8, n_kv_heads=2)
    ds = pu.run_gpu_step(inp)
    pu.check_attention(inp, ds)


@pytest.mark.parametrize("packed", [False, True])
def test_temperature_and_no_guidance(packed):
    inp = _small_bf16(3, cfg=False, prefix_lens=[17, 40], temperature=0.7, top_k=0)
    ds = pu.run_gpu_step(inp, packed_w=packed)
    pu.check_lmhead(inp, ds)
    pu.check_accept_and_path(inp, ds)


@pytest.mark.parametrize("hidden,cfg", [(128, True), (384, True), (640, False)])
def test_tiled_projection_short_hidden_and_ragged_row_tiles(hidden, cfg):
    """The LDS-tiled projection (>= 512 rows) at hidden sizes of one, three and five ring rounds,
    with a last row tile that is almost empty; every logit is compared."""
    rng = np.random.default_rng(11)
    sizes = [100, 97, 63] if cfg else [200, 200, 130]          # 260 nodes x 2 rows / 530 rows: three row tiles
    trees = [wl.grow_tree(rng, n, 6, 8) for n in sizes]
    print(f"[tiled small] hidden={hidden} cfg={cfg}", flush=True)
    inp = _small_bf16(11, n_prompts=3, cfg=cfg, hidden=hidden, vocab=512, trees=trees,
                      prefix_lens=[33, 33, 20, 20, 7, 7] if cfg else [33, 20, 7], top_k=40)
    ds = pu.run_gpu_step(inp, packed_w=True)
    pu.check_lmhead(inp, ds)
    pu.check_accept_and_path(inp, ds, require_margin=False)


def test_packed_and_row_major_weights_agree_bitwise_on_statistics():
    inp = _small_bf16(6, n_prompts=1, prefix_lens=[9, 9], trees=[wl.grow_tree(np.random.default_rng(6), 70, 5, 6)])
    a = pu.run_gpu_step(inp)
    b = pu.run_gpu_step(inp, packed_w=True)
    # same products, same per-wave k order: the two layouts give identical logits
    assert torch.equal(a.logits, b.logits) and torch.equal(a.row_thr, b.row_thr)
    assert torch.equal(a.emitted, b.emitted)


def test_rows_with_all_equal_logits_take_the_wide_bin_path():
    # zero hidden states give a row of identical logits: every entry ties with the k-th largest and is kept
    inp = _small_bf16(7, n_prompts=1, prefix_lens=[8, 8], trees=[wl.grow_tree(np.random.default_rng(7), 12, 3, 4)],
                      hidden=128, vocab=8192, top_k=100, align=0.0)
    inp.h_cond[3] = 0.0
    inp.h_uncond[3] = 0.0
    ds = pu.run_gpu_step(inp)
    pu.check_lmhead(inp, ds)
    assert float(ds.row_thr[3]) == 0.0 and abs(float(ds.row_lse[3]) - np.log(8192.0)) < 1e-5
    pu.check_accept_and_path(inp, ds, require_margin=False)


def test_rows_with_outliers():
    # 40 vocabulary rows scaled by 60 give every logits row a few huge entries of either sign, far from
    # the bulk: the k-th largest then sits many histogram bins below the row maximum
    inp = _small_bf16(9, n_prompts=1, prefix_lens=[8, 8], trees=[wl.grow_tree(np.random.default_rng(9), 20, 3, 4)],
                      hidden=128, vocab=8192, top_k=300, align=0.0)
    inp.w[:40] = wl.round_bf16(inp.w[:40] * 60.0)
    ds = pu.run_gpu_step(inp)
    pu.check_lmhead(inp, ds)
    g = ds.logits.cpu().numpy()
    kept = (g >= ds.row_thr.cpu().numpy()[:, None]).sum(axis=1)
    assert (kept >= 300).all() and (kept <= 310).all()


@pytest.mark.parametrize("case", ["plain", "ragged_vocab", "all_equal_row", "ties_at_threshold", "huge_k", "outliers", "k_one",
                                  "k_all_but_one", "barely_long"])
def test_row_statistics_of_long_rows(case):
    """Rows of more than 16384 entries (64 values per thread): the linear-bin fast path (plain, ragged_vocab)
    and every way out of it into the radix rounds - a degenerate sample range (all_equal_row), more
    candidates in the k-th largest's bin than the ranking takes (ties_at_threshold), more listed entries per
    thread than the lists hold (huge_k), a range stretched by outliers.  Every variant must select exactly
    the k-th largest of the GPU's own logits."""
    rng = np.random.default_rng(21)
    # barely_long: 18432 entries - the chunk that serves as the sample lies wholly past the end of the row
    vocab = {"ragged_vocab": 65536 - 512, "barely_long": 18432}.get(case, 65536)
    top_k = {"huge_k": 40000, "k_one": 1, "k_all_but_one": vocab - 1}.get(case, 2000)
    print(f"[long rows] {case}", flush=True)
    inp = _small_bf16(21, n_prompts=1, prefix_lens=[8, 8], trees=[wl.grow_tree(rng, 10, 3, 4)], hidden=128, vocab=vocab,
                      top_k=top_k, align=0.0)
    if case == "all_equal_row":
        inp.h_cond[2] = 0.0
        inp.h_uncond[2] = 0.0
    if case == "ties_at_threshold":
        inp.w[1000:9000] = inp.w[1000]          # 8000 identical vocabulary rows: a long run of equal logits in every row
    if case == "outliers":
        inp.w[:40] = wl.round_bf16(inp.w[:40] * 60.0)
    ds = pu.run_gpu_step(inp)
    pu.check_lmhead(inp, ds)
    g = ds.logits.cpu().numpy()
    kept = (g >= ds.row_thr.cpu().numpy()[:, None]).sum(axis=1)
    assert (kept >= top_k).all()
    if case in ("plain", "ragged_vocab", "outliers", "k_one", "k_all_but_one", "barely_long"):
        assert (kept <= top_k + 64).all()
    if case == "all_equal_row":
        assert kept[2] == vocab


def test_f32_ragged_batch():
    rng = np.random.default_rng(4)
    inp = _small_bf16(4, dtype="f32", head_dim=32, hidden=96, vocab=300, top_k=20,
                      trees=[wl.grow_tree(rng, 12, 3, 4), wl.grow_tree(rng, 30, 6, 3)])
    ds = pu.run_gpu_step(inp)
    pu.check_attention(inp, ds)
    pu.check_lmhead(inp, ds)
    pu.check_accept_and_path(inp, ds)


@pytest.mark.parametrize("vocab,top_k", [(5001, 100), (16390, 300), (16390, 1), (16390, 16389), (20000, 0)])
def test_f32_row_lengths_that_are_not_multiples_of_four(vocab, top_k):
    """fp32 logits rows of arbitrary length take the statistics kernels' scalar-load instantiations
    (16 and 64 values per thread), with the top-k bound at both ends and switched off."""
    rng = np.random.default_rng(vocab + top_k)
    inp = _small_bf16(31, dtype="f32", head_dim=32, hidden=64, vocab=vocab, top_k=top_k, n_prompts=1, prefix_lens=[6, 6],
                      trees=[wl.grow_tree(rng, 9, 3, 3)])
    ds = pu.run_gpu_step(inp)
    pu.check_lmhead(inp, ds)
    if 0 < top_k < vocab:
        g = ds.logits.cpu().numpy()
        kept = (g >= ds.row_thr.cpu().numpy()[:, None]).sum(axis=1)
        assert (kept >= top_k).all() and (kept <= top_k + 8).all()


def test_argument_validation_enqueues_nothing():
    inp = wl.make_config(0, 0)
    ds = binding.DeviceStep(inp)
    ds.logits.fill_(7.0)
    with pytest.raises(binding.CascadeError) as e:
        binding.lmhead_softmax_cfg(ds.ctx, h_cond=ds.h_cond, h_uncond=None, w=ds.w, cfg_scale=1.0, temperature=0.0,
                                   top_k=0, logits=ds.logits, row_max=ds.row_max, row_thr=ds.row_thr, row_lse=ds.row_lse)
    assert e.value.status == binding.EINVAL
    big = torch.zeros((5000, inp.hidden), device="cuda")
    with pytest.raises(binding.CascadeError) as e:
        binding.lmhead_softmax_cfg(ds.ctx, h_cond=big, h_uncond=None, w=ds.w, cfg_scale=1.0, temperature=1.0,
                                   top_k=0, logits=ds.logits, row_max=ds.row_max, row_thr=ds.row_thr, row_lse=ds.row_lse)
    assert e.value.status == binding.ESHAPE
    torch.cuda.synchronize()
    assert torch.all(ds.logits == 7.0)


def test_bad_parent_array_is_flagged_not_faulted():
    inp = wl.make_config(0, 0)
    inp.parent = inp.parent.copy()
    inp.parent[5] = 9                      # forward pointer: violates parent[i] < i
    ds = binding.DeviceStep(inp)
    ds.lmhead()
    ds.accept()
    ds.select()
    torch.cuda.synchronize()
    assert ds.ctx.device_status() == binding.ETREE
    assert ds.ctx.device_status() == binding.OK       # flag is cleared by the query
