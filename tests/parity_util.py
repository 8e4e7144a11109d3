"""Helpers shared by the GPU parity tests: run the HIP step, run the checker, compare."""
import numpy as np
import torch

from oracle import verify_oracle as vo
from paper_2605_07230_amd import binding

TOL = {"bf16": 2e-2, "f32": 1e-5}      # max relative error, the bar stated for this build


def max_rel_err(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    finite = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), finite), "non-finite pattern differs"
    if not finite.any():
        return 0.0
    return float(np.abs(got[finite] - ref[finite]).max() / max(np.abs(ref[finite]).max(), 1e-30))


def run_gpu_step(inp, mode=binding.WALK_SEQUENTIAL, packed_w=False):
    print(f"[gpu step] {inp.name} dtype={inp.dtype} rows={inp.n_rows} nodes={inp.n_nodes} mode={mode} "
          f"packed_w={packed_w}", flush=True)
    ds = binding.DeviceStep(inp)
    if packed_w:
        ds.pack_w()
    ds.step(mode)
    torch.cuda.synchronize()
    assert ds.ctx.device_status() == binding.OK
    return ds


def check_attention(inp, ds, rows=None, heads=None):
    """Compare attention outputs with the checker, on all (row, head) pairs or a subset."""
    tol = TOL[inp.dtype]
    got = ds.attn_out.float().cpu().numpy()
    got_lse = ds.attn_lse.cpu().numpy()
    rows = range(inp.n_rows) if rows is None else rows
    heads = list(range(inp.n_heads)) if heads is None else list(heads)
    group = inp.n_heads // inp.n_kv_heads
    worst = 0.0
    for s in rows:
        lo, hi = int(inp.row_node_off[s]), int(inp.row_node_off[s + 1])
        for g in heads:
            kv = g // group
            ref, ref_lse = vo.tree_attention(inp.q[lo:hi, [g]], inp.k_tree[lo:hi, [kv]], inp.v_tree[lo:hi, [kv]],
                                             inp.k_cache[[s]][:, [kv]], inp.v_cache[[s]][:, [kv]], inp.row_parent[lo:hi],
                                             np.array([0, hi - lo]), inp.prefix_len[[s]])
            e = max_rel_err(got[lo:hi, g], ref[:, 0])
            el = max_rel_err(got_lse[lo:hi, g], ref_lse[:, 0])
            worst = max(worst, e, el)
            assert e <= tol, f"attention row {s} head {g}: max rel err {e:.3e} > {tol}"
            assert el <= tol, f"attention lse row {s} head {g}: max rel err {el:.3e} > {tol}"
    return worst


def check_attention_node_sample(inp, ds, n_picks=4, seed=0):
    """EVERY (row, head) pair on a seeded sample of nodes.  A node's output depends only on the prefix
    and its ancestors, so the checker is run on the root-to-node chain of each picked node as a chain
    tree (the checker's own pins include that removing non-ancestors changes nothing); this compares
    the picked nodes and all their ancestors."""
    tol = TOL[inp.dtype]
    rng = np.random.default_rng(seed)
    got = ds.attn_out.float().cpu().numpy()
    got_lse = ds.attn_lse.cpu().numpy()
    group = inp.n_heads // inp.n_kv_heads
    worst, n_cmp = 0.0, 0
    for s in range(inp.n_rows):
        lo, hi = int(inp.row_node_off[s]), int(inp.row_node_off[s + 1])
        par = inp.row_parent[lo:hi]
        kc_s, vc_s = inp.k_cache[[s]], inp.v_cache[[s]]
        for g in range(inp.n_heads):
            kv = g // group
            picks = set(int(x) for x in rng.integers(0, hi - lo, size=n_picks)) | {hi - lo - 1}
            for i in picks:
                chain = np.asarray(vo.ancestors_or_self(par, i)) + lo
                ref, ref_lse = vo.tree_attention(inp.q[chain][:, [g]], inp.k_tree[chain][:, [kv]], inp.v_tree[chain][:, [kv]],
                                                 kc_s[:, [kv]], vc_s[:, [kv]], np.arange(-1, len(chain) - 1),
                                                 np.array([0, len(chain)]), inp.prefix_len[[s]])
                e = max_rel_err(got[chain, g], ref[:, 0])
                el = max_rel_err(got_lse[chain, g], ref_lse[:, 0])
                worst = max(worst, e, el)
                n_cmp += len(chain)
                assert e <= tol and el <= tol, f"attention row {s} head {g} chain of node {i}: {e:.3e} / lse {el:.3e} > {tol}"
    return worst, n_cmp


def check_logits_columns(inp, ds, n_cols=512, seed=0):
    """Logits of ALL nodes on a seeded sample of vocabulary columns (the projection restricted to those
    rows of W is the same definition; the row statistics need whole rows and are checked elsewhere)."""
    tol = TOL[inp.dtype]
    rng = np.random.default_rng(seed)
    cols = np.sort(rng.choice(inp.vocab, size=min(n_cols, inp.vocab), replace=False))
    g, _, _, _ = vo.lmhead_cfg(inp.h_cond, inp.h_uncond, inp.w[cols], inp.cfg_scale, inp.temperature, 0)
    got = ds.logits[:, torch.from_numpy(cols).to(ds.logits.device)].cpu().numpy()
    scale = np.abs(g).max(axis=1)                         # per node, as for whole rows
    err = (np.abs(got - g).max(axis=1) / np.maximum(scale, 1e-30)).max()
    assert err <= tol, f"logits column sample: max rel err {err:.3e} > {tol}"
    return float(err)


def check_lmhead(inp, ds, nodes=None):
    """Logits and row statistics against the checker (all nodes or a subset of them)."""
    tol = TOL[inp.dtype]
    nodes = np.arange(inp.n_nodes) if nodes is None else np.asarray(nodes)
    hu = None if inp.h_uncond is None else inp.h_uncond[nodes]
    g, m, thr, lse = vo.lmhead_cfg(inp.h_cond[nodes], hu, inp.w, inp.cfg_scale, inp.temperature, inp.top_k)
    got = ds.logits[torch.from_numpy(nodes).to(ds.logits.device)].cpu().numpy()
    worst = 0.0
    for i in range(len(nodes)):
        e = max_rel_err(got[i], g[i])
        worst = max(worst, e)
        assert e <= tol, f"logits node {nodes[i]}: max rel err {e:.3e} > {tol}"
    gm, gt, gl = (t.cpu().numpy()[nodes] for t in (ds.row_max, ds.row_thr, ds.row_lse))
    assert max_rel_err(gm, m) <= tol and max_rel_err(gl, lse) <= tol
    if inp.top_k > 0 and inp.top_k < inp.vocab:
        assert max_rel_err(gt, thr) <= tol
    # statistics are exact functions of the GPU's own logits: selection is integer work
    gm2, gt2, gl2 = vo.row_stats(got, inp.top_k)
    np.testing.assert_array_equal(gm, gm2.astype(np.float32))
    np.testing.assert_array_equal(gt, gt2.astype(np.float32))
    np.testing.assert_allclose(gl, gl2, rtol=2e-6, atol=2e-6)
    return worst


def check_accept_and_path(inp, ds, mode=binding.WALK_SEQUENTIAL, tau_pos=None, tau_seq=None, eps_tvd=None,
                          require_margin=True):
    """The checker's acceptance stage, fed the GPU's own logits / statistics and the same hidden states
    and uniforms, must give bit-identical discrete outputs; per-node scalars within tolerance."""
    tol = TOL[inp.dtype]
    tau_pos = inp.tau_pos if tau_pos is None else tau_pos
    tau_seq = inp.tau_seq if tau_seq is None else tau_seq
    eps_tvd = inp.eps_tvd if eps_tvd is None else eps_tvd
    g = ds.logits.cpu().numpy().astype(np.float64)
    thr = ds.row_thr.cpu().numpy().astype(np.float64)
    lse = ds.row_lse.cpu().numpy().astype(np.float64)
    acc = vo.cascade_accept(inp.node_off, inp.parent, inp.token, inp.h_cond, g, thr, lse, tau_pos, tau_seq)
    res = vo.select_path(inp.node_off, inp.parent, inp.token, acc, inp.draft_prob, inp.u, inp.u_bonus, eps_tvd,
                         g, thr, lse, inp.max_depth, mode)
    info = f"min cos margin {acc.min_cos_margin:.2e}, min walk margin {res.min_margin:.2e}"
    if require_margin:
        # the seeds used here keep every decision away from its threshold; otherwise the case would not
        # be a valid bit-exactness test (fp32 vs fp64 rounding could legitimately flip it)
        assert acc.min_cos_margin > 1e-4 and res.min_margin > 1e-6, info
    np.testing.assert_array_equal(ds.n_int.cpu().numpy(), acc.n_int, err_msg=info)
    np.testing.assert_array_equal(ds.n_conv.cpu().numpy(), acc.n_conv, err_msg=info)
    for name in ("q_tok", "m_int", "m_conv"):
        got = getattr(ds, name).cpu().numpy()
        ref = getattr(acc, name)
        np.testing.assert_allclose(got, ref, rtol=1e-4, atol=1e-9, err_msg=name)
    assert np.abs(ds.cos_parent.cpu().numpy() - acc.cos_parent).max() <= (1e-5 if inp.dtype == "f32" else 1e-4)
    np.testing.assert_array_equal(ds.accept_len.cpu().numpy(), res.accept_len, err_msg=info)
    if inp.max_depth > 0:
        np.testing.assert_array_equal(ds.path_nodes.cpu().numpy()[:, :inp.max_depth], res.path_nodes, err_msg=info)
    np.testing.assert_array_equal(ds.emitted.cpu().numpy(), res.emitted, err_msg=info)
    np.testing.assert_array_equal(ds.terminal.cpu().numpy(), res.terminal, err_msg=info)
    np.testing.assert_allclose(ds.tvd_used.cpu().numpy(), res.tvd_used, rtol=1e-4, atol=1e-9)
    assert np.all(ds.tvd_used.cpu().numpy() <= eps_tvd * (1 + 1e-6))
    return acc, res
