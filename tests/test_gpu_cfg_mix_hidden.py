"""Guidance mixed into the hidden rows before ONE projection (CASCADE_CFG_MIX_HIDDEN) against the checker's
definition (two products, mix of the logits) at the build's bf16 bar, and - much tighter - against the same
single product written out on the host: the mixed rows u + s (c - u) in float32, rounded once to bf16, times W in
float64.  The second comparison pins that the only thing this path adds is that one rounding."""
import numpy as np
import pytest
import torch

import parity_util as pu
from paper_2605_07230_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def _mixed_rows(inp, nodes):
    c, u, s = inp.h_cond[nodes].astype(np.float32), inp.h_uncond[nodes].astype(np.float32), np.float32(inp.cfg_scale)
    return wl.round_bf16(u + s * (c - u)).astype(np.float64)


def _run(inp, mode=binding.WALK_SEQUENTIAL):
    print(f"[gpu step, hidden-row mix] {inp.name} rows={inp.n_rows} nodes={inp.n_nodes}", flush=True)
    ds = binding.DeviceStep(inp)
    ds.pack_w()
    ds.cfg_mix = binding.CFG_MIX_HIDDEN
    ds.step(mode)
    torch.cuda.synchronize()
    assert ds.ctx.device_status() == binding.OK
    return ds


def _check_single_product(inp, ds, nodes, cols=None, bar=1e-3):
    """GPU logits of `nodes` against (mixed bf16 rows) x W^T / temperature in float64, relative to each row's largest
    |g|.  The GPU may contract u + s (c - u) into one fused multiply-add, which now and then rounds a mixed element
    to the neighbouring bf16 value: the bar leaves room for that, and is 20 times tighter than the build's."""
    nodes = np.asarray(nodes)
    w = inp.w.astype(np.float64) if cols is None else inp.w[cols].astype(np.float64)
    ref = _mixed_rows(inp, nodes) @ w.T / inp.temperature
    got = ds.logits[torch.from_numpy(nodes).to(ds.logits.device)].cpu().numpy().astype(np.float64)
    if cols is not None:
        got = got[:, cols]
    err = (np.abs(got - ref).max(axis=1) / np.abs(ref).max(axis=1)).max()
    assert err <= bar, f"single product: max rel err {err:.3e} > {bar}"
    return float(err)


@pytest.mark.parametrize("index,seed", [(1, 0), (1, 3), (2, 0)])
def test_streaming_projection_with_mixed_rows(index, seed):
    inp = wl.make_config(index, seed)
    ds = _run(inp)
    nodes = np.arange(inp.n_nodes) if index == 1 else np.array([0, 1, 7, 30, 59])
    worst = pu.check_lmhead(inp, ds, nodes=nodes)               # the definition, 2e-2
    tight = _check_single_product(inp, ds, nodes)
    print(f"[hidden-row mix] {inp.name}: {worst:.2e} against the definition, {tight:.2e} against the single product", flush=True)
    pu.check_accept_and_path(inp, ds)                           # decisions follow the GPU's own logits: bit-exact


@pytest.mark.parametrize("hidden,sizes", [(128, [100, 97, 63]), (384, [130, 128, 1]), (640, [200, 200, 130])])
def test_half_tiles_with_mixed_rows_every_logit(hidden, sizes):
    """260 / 259 / 530 mixed rows in 128-row tiles (the last one with 4, 3 and 18 rows) at hidden sizes of one,
    three and five ring rounds; every logit against the definition and against the single product."""
    rng = np.random.default_rng(21)
    trees = [wl.grow_tree(rng, n, 6, 8) if n > 1 else np.array([-1], np.int32) for n in sizes]
    inp = wl.make_inputs(seed=21, name="edge", dtype="bf16", n_prompts=3, cfg=True, n_heads=4, n_kv_heads=2, head_dim=64,
                         hidden=hidden, vocab=512, prefix_lens=[33, 33, 20, 20, 7, 7], trees=trees, cfg_scale=3.0,
                         temperature=0.8, top_k=40, tau_pos=0.9, tau_seq=0.9, eps_tvd=0.5, token_law="zipf")
    ds = _run(inp)
    pu.check_lmhead(inp, ds)
    _check_single_product(inp, ds, np.arange(inp.n_nodes))
    pu.check_accept_and_path(inp, ds, require_margin=False)


@pytest.mark.parametrize("seed", range(6))
def test_tiled_projection_random_shapes_both_mixes(seed):
    """Random row counts (257-700 nodes in 3-6 prompts), hidden sizes and vocabularies through both guidance
    mixes: guidance-pair tiles, plain 256-row tiles and 128-row tiles with ragged last tiles; every logit compared."""
    rng = np.random.default_rng(100 + seed)
    n_prompts = int(rng.integers(3, 7))
    total = int(rng.integers(257, 701))
    cuts = np.sort(rng.choice(np.arange(1, total), size=n_prompts - 1, replace=False))
    sizes = np.diff(np.concatenate([[0], cuts, [total]])).astype(int)
    trees = [wl.grow_tree(rng, int(n), min(6, int(n) - 1), 8) if n > 1 else np.array([-1], np.int32) for n in sizes]
    hidden = int(rng.choice([128, 256, 512, 896]))
    vocab = int(rng.choice([256, 512, 768]))
    scale = float(rng.choice([3.0, 5.0]))
    inp = wl.make_inputs(seed=100 + seed, name="edge", dtype="bf16", n_prompts=n_prompts, cfg=True, n_heads=4, n_kv_heads=2,
                         head_dim=64, hidden=hidden, vocab=vocab, prefix_lens=[int(x) for x in rng.integers(1, 40, size=2 * n_prompts)],
                         trees=trees, cfg_scale=scale, temperature=1.0, top_k=int(rng.choice([0, 30])), tau_pos=0.9, tau_seq=0.9,
                         eps_tvd=0.5, token_law="zipf")
    print(f"[random tiled] nodes={inp.n_nodes} sizes={sizes.tolist()} hidden={hidden} vocab={vocab} scale={scale}", flush=True)
    for mix in (binding.CFG_MIX_LOGITS, binding.CFG_MIX_HIDDEN):
        ds = binding.DeviceStep(inp)
        ds.pack_w()
        ds.cfg_mix = mix
        ds.lmhead()
        torch.cuda.synchronize()
        assert ds.ctx.device_status() == binding.OK
        pu.check_lmhead(inp, ds)
        if mix == binding.CFG_MIX_HIDDEN:
            _check_single_product(inp, ds, np.arange(inp.n_nodes))


def test_tiled_projection_with_mixed_rows_ragged_batch():
    inp = wl.make_config(3, 0)
    ds = _run(inp)
    nodes = np.unique(np.concatenate([inp.node_off[:-1], inp.node_off[1:] - 1, np.arange(0, inp.n_nodes, 37)]))
    pu.check_lmhead(inp, ds, nodes=nodes)
    _check_single_product(inp, ds, nodes)
    pu.check_logits_columns(inp, ds, n_cols=256, seed=5)        # all 924 nodes: every row tile and its ragged tail
    pu.check_accept_and_path(inp, ds)


def test_tiled_projection_with_mixed_rows_stress():
    inp = wl.make_config(4, 0)
    ds = _run(inp)
    pu.check_lmhead(inp, ds, nodes=[0, 1, 255, 256, 700, 1023])
    pu.check_logits_columns(inp, ds, n_cols=512, seed=2)        # all 1024 nodes
    rng = np.random.default_rng(7)
    cols = np.sort(rng.choice(inp.vocab, size=512, replace=False))
    _check_single_product(inp, ds, np.arange(inp.n_nodes), cols=cols)
    pu.check_accept_and_path(inp, ds)


def test_both_mixes_agree_within_the_rounding_of_the_mixed_rows():
    """Same inputs through both paths: logits differ by the one extra rounding only (a few 1e-3 of the row's
    largest |g| at guidance scale 5), the statistics follow their own logits exactly."""
    inp = wl.make_config(1, 1)
    a = binding.DeviceStep(inp)
    a.pack_w()
    a.lmhead()
    b = binding.DeviceStep(inp)
    b.pack_w()
    b.cfg_mix = binding.CFG_MIX_HIDDEN
    b.lmhead()
    torch.cuda.synchronize()
    ga, gb = a.logits.cpu().numpy().astype(np.float64), b.logits.cpu().numpy().astype(np.float64)
    rel = (np.abs(ga - gb).max(axis=1) / np.abs(ga).max(axis=1)).max()
    assert 0.0 < rel <= 6e-3, rel


def test_row_major_weights_and_float32_ignore_the_switch():
    """The switch is honoured for packed bf16 weights only: elsewhere the two products run and the results are
    bit-identical to the default."""
    inp = wl.make_config(1, 2)
    a = binding.DeviceStep(inp)
    a.lmhead()
    b = binding.DeviceStep(inp)
    b.cfg_mix = binding.CFG_MIX_HIDDEN
    b.lmhead()
    torch.cuda.synchronize()
    assert torch.equal(a.logits, b.logits) and torch.equal(a.row_lse, b.row_lse)


def test_invalid_switch_value_is_refused():
    inp = wl.make_config(1, 0)
    ds = binding.DeviceStep(inp)
    ds.cfg_mix = 7
    with pytest.raises(binding.CascadeError):
        ds.lmhead()
