#!/usr/bin/env python3
"""Benchmark of the MI355X tree-verification step (one GPU).

A step = tree_verify_attn + lmhead_softmax_cfg + cascade_accept + select_path over one batch of
synthetic input that is already resident in HBM.  Prints ONE JSON line.  The headline is the stress
configuration (the largest one: 4 prompts x 2 guidance rows, 4200-key prefix, 256-node trees,
vocabulary 65536), the shape on which the roofline targets mean something: the projection is bound
by the matrix cores, attention and the row statistics by HBM.  The smaller configurations are timed
in the same run and reported as a nested block.

Guidance: by default the mix is taken on the hidden rows (lmhead_args.cfg_mix = CASCADE_CFG_MIX_HIDDEN: the
projection is linear, so one product over the mixed rows gives the mixed logits up to one bf16 rounding of those
rows); `config.cfg_mix` says so, `roofline.algorithmic_flops` counts what that path executes, and the block
`guidance_mix_on_logits` holds the same workload timed with the formula as written (two products).  `--cfg-mix logits`
makes that the headline instead.  `vendor_gemm_yardstick` is torch.matmul on the projection's own shape, for context.

The large read-only inputs (LM-head matrix, KV cache) are rotated over several independent copies
so that consecutive steps cannot be served from the 256 MB Infinity Cache: in a real decode loop a
whole model's weights stream between two verification steps.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM traffic per launch from rocprofv3 --pmc runs of this file: (FETCH_SIZE, WRITE_SIZE) in KiB per
# dispatch, copied from the tracked counter summaries profiles/<workload>_step_counters.md (a CPU test
# compares this table with the "TRAFFIC" lines of those summaries).  Bytes = FETCH x 2.0 + WRITE x 1.0:
# the read counter sees half of the bytes that 16-byte-per-lane loads move, as the same counter shows
# for a streaming read of known size in the same runs; writes count 1.0.  No entry = no counter run =
# traffic null.
FETCH_FACTOR, WRITE_FACTOR = 2.0, 1.0
MEASURED_TRAFFIC_KIB = {
    ("stress_1024px", "accept"): (17650.3, 193.0),
    ("stress_1024px", "attn"): (293568.2, 18432.0),
    ("stress_1024px", "lmhead"): (393828.6, 262144.0),
    ("stress_1024px", "pack_h"): (8196.5, 8192.0),
    ("stress_1024px", "row_stats"): (131197.7, 98.2),
    ("stress_1024px", "select"): (588.3, 0.9),
    ("janus_batched", "accept"): (7529.7, 83.8),
    ("janus_batched", "attn"): (49856.9, 8118.1),
    ("janus_batched", "lmhead"): (82009.7, 28864.0),
    ("janus_batched", "pack_h"): (3612.5, 4096.0),
    ("janus_batched", "row_stats"): (14507.5, 42.3),
    ("janus_batched", "select"): (424.0, 1.4),
    ("janus_pro_7b", "accept"): (989.2, 11.2),
    ("janus_pro_7b", "attn"): (6521.0, 1080.0),
    ("janus_pro_7b", "lmhead"): (67752.2, 3840.0),
    ("janus_pro_7b", "pack_h"): (484.5, 512.0),
    ("janus_pro_7b", "row_stats"): (1995.8, 5.6),
    ("janus_pro_7b", "select"): (52.8, 0.2),
    ("lumina_mgpt_7b_768", "accept"): (997.8, 11.2),
    ("lumina_mgpt_7b_768", "attn"): (22158.7, 1080.0),
    ("lumina_mgpt_7b_768", "lmhead"): (264994.3, 15360.0),
    ("lumina_mgpt_7b_768", "pack_h"): (484.5, 512.0),
    ("lumina_mgpt_7b_768", "row_stats"): (7804.2, 5.6),
    ("lumina_mgpt_7b_768", "select"): (144.2, 0.2),
}


def measured_traffic(workload: str, kernel: str):
    kib = MEASURED_TRAFFIC_KIB.get((workload, kernel))
    return None if kib is None else int((kib[0] * FETCH_FACTOR + kib[1] * WRITE_FACTOR) * 1024)


def algorithmic_bytes_lmhead(inp) -> int:
    """W once + hidden states in + mixed logits out (the projection kernel's own traffic)."""
    rows = inp.n_nodes * (2 if inp.h_uncond is not None else 1)
    e = 2 if inp.dtype == "bf16" else 4
    return inp.vocab * inp.hidden * e + rows * inp.hidden * e + inp.n_nodes * inp.vocab * 4


def algorithmic_flops_lmhead(inp) -> int:
    rows = inp.n_nodes * (2 if inp.h_uncond is not None else 1)
    return 2 * rows * inp.hidden * inp.vocab


def algorithmic_bytes_attn(inp) -> int:
    """K and V of prefix + tree once per (row, kv head); Q in and O out."""
    e = 2 if inp.dtype == "bf16" else 4
    total = 0
    for s in range(inp.n_rows):
        T = int(inp.row_node_off[s + 1] - inp.row_node_off[s])
        total += inp.n_kv_heads * (int(inp.prefix_len[s]) + T) * inp.head_dim * 2 * e
        total += T * inp.n_heads * inp.head_dim * 2 * e
    return total


def algorithmic_bytes_row_stats(inp) -> int:
    """The mixed logits once (row max, k-th largest and log-sum-exp need every entry) + three scalars out."""
    return inp.n_nodes * inp.vocab * 4 + inp.n_nodes * 12


def algorithmic_bytes_accept(inp) -> int:
    """Every node's hidden state once + the six per-node scalars out (token-probability gathers are a few bytes per node)."""
    e = 2 if inp.dtype == "bf16" else 4
    return inp.n_nodes * inp.hidden * e + inp.n_nodes * 24


def cpu_baseline(inp, budget_s: float = 12.0):
    """The CPU checker, as it stands, on the same workload; whole steps until the budget is used
    (at least one: a stress-shaped step takes about 20 s)."""
    from oracle import verify_oracle as vo
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    n, t0 = 0, time.perf_counter()
    while True:
        vo.verify_step(inp)
        n += 1
        el = time.perf_counter() - t0
        if el >= budget_s or n >= 200:
            break
    return {"value": n / el, "unit": "steps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n} whole step(s) of the same workload (numpy float64; BLAS threads = cores), {el:.1f} s"}


def tau_sweep(args) -> int:
    """Stress-shaped trees over many seeds: mean accepted length and acceptance / walk time per
    threshold (both thresholds set to tau).  One LM-head matrix is shared by all seeds and the
    prefix is cut to 64 tokens (attention does not depend on the thresholds)."""
    import numpy as np
    import torch
    from paper_2605_07230_amd import binding, workloads as wl
    binding.load_library()
    taus = (0.8, 0.9, 0.95)
    acc_len = {t: [] for t in taus}
    acc_us = {t: [] for t in taus}
    sel_us = {t: [] for t in taus}
    w0, w_packed = None, None
    for seed in range(args.sweep_seeds):
        inp = wl.make_config(4, seed, prefix_lens=[64] * 8, w=w0)
        if w0 is None:
            w0 = inp.w
        ds = binding.DeviceStep(inp)
        ds.cfg_mix = binding.CFG_MIX_HIDDEN if args.cfg_mix == "hidden" else binding.CFG_MIX_LOGITS
        if w_packed is None:
            w_packed = ds.pack_w()
        ds.lmhead(w_packed, binding.W_PACKED32)
        if args.rank_zipf:
            # draft tokens re-drawn by rank: a child's token is the vocabulary entry at a Zipf(1.1)-distributed
            # rank of its parent's mixed logits (measurement input only; torch sorts the library's logits)
            rng = np.random.default_rng(seed + 99)
            order = torch.argsort(ds.logits, dim=1, descending=True)
            ranks_pmf = np.arange(1, inp.vocab + 1, dtype=np.float64) ** -1.1
            ranks_pmf /= ranks_pmf.sum()
            cdf = np.cumsum(ranks_pmf)
            tok = inp.token.copy()
            dprob = inp.draft_prob.copy()
            for b in range(inp.n_prompts):
                lo, hi = int(inp.node_off[b]), int(inp.node_off[b + 1])
                par = inp.parent[lo:hi]
                for p_ in range(hi - lo):
                    kids = np.nonzero(par == p_)[0]
                    if len(kids) == 0:
                        continue
                    chosen = []
                    while len(chosen) < len(kids):            # distinct ranks among siblings
                        r = int(np.searchsorted(cdf, rng.random()))
                        if r not in chosen:
                            chosen.append(min(r, inp.vocab - 1))
                    ids = order[lo + p_, torch.tensor(chosen, device=order.device)].cpu().numpy()
                    tok[lo + kids] = ids
                    dprob[lo + kids] = ranks_pmf[chosen].astype(np.float32)
            ds.token = torch.from_numpy(tok).to(ds.logits.device)
            ds.draft_prob = torch.from_numpy(dprob).to(ds.logits.device)
        for t in taus:
            for rep in range(3):
                ds.accept(t, t)
                ds.select()
            ds.ctx.set_kernel_timing(True)
            for rep in range(10):
                ds.accept(t, t)
                ds.select()
            ms_a, n_a = ds.ctx.read_kernel_timing(4)
            ms_s, n_s = ds.ctx.read_kernel_timing(5)
            ds.ctx.set_kernel_timing(False)
            acc_len[t] += ds.accept_len.cpu().tolist()
            acc_us[t].append(ms_a * 1e3 / n_a)
            sel_us[t].append(ms_s * 1e3 / n_s)
        assert ds.ctx.device_status() == binding.OK
        ds.w = None
        del ds
    # the cost the accepted tokens are bought with: the WHOLE step (attention, projection, statistics, acceptance,
    # walk) of the full stress configuration (4200-key prefixes), timed per threshold on rotating input copies
    inp = wl.make_config(4, 0, w=w0)
    ds = binding.DeviceStep(inp)
    ds.cfg_mix = binding.CFG_MIX_HIDDEN if args.cfg_mix == "hidden" else binding.CFG_MIX_LOGITS
    kcs = [ds.k_cache] + [ds.k_cache.clone() for _ in range(3)]
    vcs = [ds.v_cache] + [ds.v_cache.clone() for _ in range(3)]
    ws = [w_packed] + [w_packed.clone() for _ in range(3)]
    step_us = {}
    for t in taus:
        def one(i):
            ds.k_cache, ds.v_cache = kcs[i % 4], vcs[i % 4]
            ds.attn()
            ds.lmhead(ws[i % 4], binding.W_PACKED32)
            ds.accept(t, t)
            ds.select()
        for i in range(5):
            one(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(40):
            one(i)
        torch.cuda.synchronize()
        step_us[t] = (time.perf_counter() - t0) * 1e6 / 40
    assert ds.ctx.device_status() == binding.OK
    out = {"metric": "tau_sweep", "cfg_mix": "hidden_rows" if args.cfg_mix == "hidden" else "logits", "tokens": "rank-zipf of the parent's logits" if args.rank_zipf else "generator's tokens",
           "workload": "stress_1024px trees (prefix cut to 64), seeds 0..%d; whole-step time on the full configuration" % (args.sweep_seeds - 1),
           "per_tau": {str(t): {"mean_accept_len": float(np.mean(acc_len[t])), "accept_us": float(np.mean(acc_us[t])),
                                "select_us": float(np.mean(sel_us[t])), "prompts": len(acc_len[t]),
                                "whole_step_us": step_us[t],
                                "accepted_tokens_per_s": float(np.mean(acc_len[t])) * inp.n_prompts / (step_us[t] * 1e-6)}
                       for t in taus}}
    print(json.dumps(out))
    return 0


KERNEL_NAMES = {0: "attn", 1: "attn_merge", 2: "lmhead", 3: "row_stats", 4: "accept", 5: "select", 8: "pack_h"}


def measure_workload(index: int, steps: int, warmup: int, args, hbm_meas: float, mfma_meas: float, cfg_mix: str = None):
    """Times `steps` whole steps of one configuration (wall clock), then the same steps again with the
    library's per-kernel events on; returns (inputs, device step, dict for the JSON line)."""
    import torch
    from paper_2605_07230_amd import binding, workloads as wl
    inp = wl.make_config(index, args.seed)
    ds = binding.DeviceStep(inp)
    cfg_mix = cfg_mix or args.cfg_mix
    copies = max(1, args.copies)
    # weights are repacked once into MFMA operand order, as at model load (outside the timed region)
    packed = inp.dtype == "bf16" and not args.row_major_w
    layout = binding.W_PACKED32 if packed else binding.W_ROWMAJOR
    w0 = ds.pack_w() if packed else ds.w
    # guidance mixed into the hidden rows (one product over n_nodes rows) or into the logits (two products)
    premix = packed and inp.h_uncond is not None and cfg_mix == "hidden"
    ds.cfg_mix = binding.CFG_MIX_HIDDEN if premix else binding.CFG_MIX_LOGITS
    ws = [w0] + [w0.clone() for _ in range(copies - 1)]
    kcs = [ds.k_cache] + [ds.k_cache.clone() for _ in range(copies - 1)]
    vcs = [ds.v_cache] + [ds.v_cache.clone() for _ in range(copies - 1)]

    def step(i: int) -> None:
        j = i % copies
        ds.k_cache, ds.v_cache = kcs[j], vcs[j]
        ds.step(w=ws[j], w_layout=layout)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert ds.ctx.device_status() == binding.OK

    # the same steps on ONE copy of the inputs (W and KV stay in the 256 MB last-level cache where they fit): context only
    ms_cache_warm = None
    if args.cache_warm:
        n_warm = min(steps, 200)
        for i in range(10):
            step(0)
        torch.cuda.synchronize()
        tw = time.perf_counter()
        for i in range(n_warm):
            step(0)
        torch.cuda.synchronize()
        ms_cache_warm = (time.perf_counter() - tw) * 1e3 / n_warm

    # second pass over the same steps with the dispatch's own begin / end timestamps on every launch
    # (HIP events on the library's stream, handed to the launch itself)
    ds.ctx.set_kernel_timing(True)
    n_timed = min(steps, 2000)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(n_timed):
        step(i)
    torch.cuda.synchronize()
    ms_events = (time.perf_counter() - t1) * 1e3 / n_timed
    kernel_us = {}
    for kid, name in KERNEL_NAMES.items():
        ms, n = ds.ctx.read_kernel_timing(kid)
        if n:
            kernel_us[name] = ms * 1e3 / n
    ds.ctx.set_kernel_timing(False)

    rows = inp.n_nodes * (2 if (inp.h_uncond is not None and not premix) else 1)   # rows the projection multiplies
    guidance_pairs = inp.h_uncond is not None and not premix
    tiled = packed and rows >= (512 if guidance_pairs else 257) and inp.vocab % 256 == 0   # the library's own rule
    # projection: bound by the matrix cores when the step has several hundred rows, by the W stream otherwise
    if tiled:
        flops = 2 * rows * inp.hidden * inp.vocab      # executed: with the hidden-row mix half of the two-product count
        ach = flops / (kernel_us["lmhead"] * 1e-6) / 1e12
        roof_lm = {"kernel": "lmhead_bf16_tiled_kernel", "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                   "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": measured_traffic(inp.name, "lmhead"),
                   "algorithmic_flops": flops, "flops_two_products": algorithmic_flops_lmhead(inp),
                   "algorithmic_bytes": algorithmic_bytes_lmhead(inp), "frac_of_measured_peak": ach / mfma_meas}
    else:
        nbytes = algorithmic_bytes_lmhead(inp)
        ach = nbytes / (kernel_us["lmhead"] * 1e-6) / 1e9
        kname = "lmhead_f32_kernel" if inp.dtype == "f32" else ("lmhead_bf16_packed_kernel" if packed else "lmhead_bf16_kernel")
        roof_lm = {"kernel": kname, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                   "frac": ach / HBM_PEAK_GBS, "traffic": measured_traffic(inp.name, "lmhead"), "algorithmic_bytes": nbytes,
                   "frac_of_measured_peak": ach / hbm_meas}
    roof_lm["avg_launch_us"] = kernel_us["lmhead"]

    def hbm_block(kernel, nbytes, us, traffic):
        ach = nbytes / (us * 1e-6) / 1e9
        return {"kernel": kernel, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": traffic, "algorithmic_bytes": nbytes,
                "frac_of_measured_peak": ach / hbm_meas, "avg_launch_us": us}

    max_tree = int((inp.node_off[1:] - inp.node_off[:-1]).max())
    m_rows = max_tree * (inp.n_heads // inp.n_kv_heads)
    units = inp.n_rows * inp.n_kv_heads * ((m_rows + 63) // 64)
    if inp.dtype == "f32":
        attn_kernel = "attn_f32_kernel"
    elif m_rows > 128:
        # 256 query rows per workgroup; the ring kernel unless the keys are split to fill an idle GPU
        attn_kernel = "attn_bf16_kernel" if "attn_merge" in kernel_us else "attn_bf16_ring_kernel"
    else:
        attn_kernel = "attn_bf16_qsplit_kernel" if units <= 128 else "attn_bf16_ksplit_kernel"
    attn_us = kernel_us.get("attn", 0.0) + kernel_us.get("attn_merge", 0.0)
    t_attn, t_merge = measured_traffic(inp.name, "attn"), measured_traffic(inp.name, "attn_merge")
    if t_attn is not None and "attn_merge" in kernel_us:
        t_attn = None if t_merge is None else t_attn + t_merge
    roof_attn = hbm_block(attn_kernel + (" + attn_merge_kernel" if "attn_merge" in kernel_us else ""),
                          algorithmic_bytes_attn(inp), attn_us, t_attn)
    roof_stats = hbm_block("row_stats_kernel", algorithmic_bytes_row_stats(inp), kernel_us["row_stats"],
                           measured_traffic(inp.name, "row_stats"))
    # attention + everything that turns logits into an accepted path (row statistics, acceptance scalars, walk)
    acc_bytes = algorithmic_bytes_attn(inp) + algorithmic_bytes_row_stats(inp) + algorithmic_bytes_accept(inp)
    acc_us = attn_us + kernel_us["row_stats"] + kernel_us["accept"] + kernel_us["select"]
    parts = [measured_traffic(inp.name, k) for k in ("row_stats", "accept", "select")] + [t_attn]
    roof_acc = hbm_block("attention + row statistics + acceptance + walk", acc_bytes, acc_us,
                         None if any(x is None for x in parts) else sum(parts))

    out = {
        "workload": inp.name, "steps": steps, "warmup": warmup, "ms_per_step": elapsed * 1e3 / steps,
        "steps_per_s": steps / elapsed, "tree_nodes_per_s": inp.n_nodes * steps / elapsed,
        "ms_per_step_with_events": ms_events, "ms_per_step_cache_warm": ms_cache_warm,
        "kernel_us": kernel_us, "accept_len": ds.accept_len.cpu().tolist(),
        "roofline": roof_lm, "roofline_attention": roof_attn, "roofline_row_stats": roof_stats,
        "roofline_attn_accept": roof_acc,
        "config": {"workload": inp.name, "rows": inp.n_rows, "prompts": inp.n_prompts, "tree_nodes": inp.n_nodes,
                   "prefix_len": int(inp.prefix_len.max()), "heads": inp.n_heads, "head_dim": inp.head_dim,
                   "hidden": inp.hidden, "vocab": inp.vocab, "cfg_scale": inp.cfg_scale, "top_k": inp.top_k,
                   "input_copies_rotated": copies, "lmhead_w_layout": "packed32" if packed else "row_major",
                   "cfg_mix": "hidden_rows" if premix else ("logits" if inp.h_uncond is not None else "none")},
    }
    del ws, kcs, vcs
    return inp, ds, out, packed


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=4, help="index into the five configurations (default 4: the stress configuration)")
    ap.add_argument("--others", type=str, default="1,2,3", help="configurations also timed and reported in the nested block ('' = none)")
    ap.add_argument("--other-steps", type=int, default=200)
    ap.add_argument("--copies", type=int, default=4, help="independent copies of W / KV rotated between steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cfg-mix", choices=["hidden", "logits"], default="hidden",
                    help="where the guidance mix is taken: on the hidden rows (one product, default) or on the logits (two products)")
    ap.add_argument("--no-two-products", action="store_true", help="skip the second timing of the headline workload with the mix on the logits")
    ap.add_argument("--no-vendor-gemm", action="store_true", help="skip the vendor GEMM timed beside the tiled projection")
    ap.add_argument("--row-major-w", action="store_true", help="keep the LM-head matrix row-major (default: packed once, as at model load)")
    ap.add_argument("--cache-warm", action="store_true", help="also time the steps on one copy of the inputs (served from the last-level cache)")
    ap.add_argument("--commit-layers", type=int, default=30, help="decoder layers in the separately timed KV commit (0: skip)")
    ap.add_argument("--weights-seqs", type=int, default=8, help="sequences in the separately timed Eq. 4 weight mask (0: skip)")
    ap.add_argument("--decode-image", type=int, default=0, help="tokens of the separately timed multi-step decode loop (0: skip; single-prompt workloads)")
    ap.add_argument("--tau-sweep", action="store_true", help="instead of the step benchmark: threshold sweep on stress-shaped trees")
    ap.add_argument("--sweep-seeds", type=int, default=32)
    ap.add_argument("--rank-zipf", action="store_true", help="tau sweep: re-draw draft tokens by Zipf rank of the parent's logits")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1", file=sys.stderr)
        return 2
    if args.tau_sweep:
        return tau_sweep(args)

    import torch
    from paper_2605_07230_amd import binding, workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the verification path has no CPU fallback", file=sys.stderr)
        return 3
    binding.load_library()
    torch.cuda.set_device(0)

    # what this device sustains: a plain streaming read of 1 GiB and a register-only MFMA loop
    cal = binding.Context(max_rows=1, max_nodes_total=1, max_nodes_per_tree=1, max_prefix=1, n_heads=1, head_dim=64, hidden=128, vocab=64)
    big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    big.zero_()
    hbm_meas = cal.measure_hbm_read(big, 5)
    mfma_meas = cal.measure_mfma_bf16(8192)
    del big
    cal.close()

    print(f"[bench] headline workload {args.workload}", file=sys.stderr, flush=True)
    inp, ds, head, packed = measure_workload(args.workload, args.steps, args.warmup, args, hbm_meas, mfma_meas)

    # the KV commit that follows the step (not part of the step metric): all decoder layers' worth of
    # tree keys / values, the path the step just chose, appended to a cache with room
    commit = None
    if args.commit_layers > 0:
        Lc, S, Hkv, D = args.commit_layers, inp.n_rows, inp.n_kv_heads, inp.head_dim
        cap = inp.max_depth + 8          # room for root + path; the prefix itself is not touched by the commit
        dt = ds.k_tree.dtype
        kt = torch.randn((Lc, ds.k_tree.shape[0], Hkv, D), device="cuda").to(dt)
        vt = torch.randn((Lc, ds.k_tree.shape[0], Hkv, D), device="cuda").to(dt)
        kc = torch.zeros((Lc, S, Hkv, cap, D), dtype=dt, device="cuda")
        vc = torch.zeros((Lc, S, Hkv, cap, D), dtype=dt, device="cuda")
        row_prompt = (torch.arange(S, device="cuda", dtype=torch.int32) // (2 if inp.cfg else 1)).to(torch.int32)
        plen0 = torch.zeros_like(ds.prefix_len)
        plen_out = torch.empty_like(ds.prefix_len)
        ds.ctx.set_kernel_timing(True)
        for i in range(60):
            binding.kv_commit(ds.ctx, node_off=ds.row_node_off, row_prompt=row_prompt, accept_len=ds.accept_len,
                              path_nodes=ds.path_nodes, k_tree=kt, v_tree=vt, k_cache=kc, v_cache=vc,
                              prefix_len=plen0, prefix_len_out=plen_out)
            if i == 9:
                ds.ctx.read_kernel_timing(6)      # drop the warm-up launches
        ms, n = ds.ctx.read_kernel_timing(6)
        ds.ctx.set_kernel_timing(False)
        assert ds.ctx.device_status() == binding.OK
        moved = int((plen_out - plen0).sum().item()) * Lc * Hkv * D * kt.element_size() * 2 * 2   # K and V, read + write
        commit = {"layers": Lc, "us": ms * 1e3 / n, "bytes": moved, "GBs": moved / (ms * 1e-3 / n) / 1e9}
        del kt, vt, kc, vc

    # the Eq. 4 weight mask (drafter-training side, not part of the step metric): Lumina-shaped
    # sequences, one pass over [8, 2356, hidden] features; HBM-bound, rotated over 4 copies
    weights = None
    if args.weights_seqs > 0:
        Bw, Kw = args.weights_seqs, 2356
        feats = [torch.randn((Bw, Kw, inp.hidden), device="cuda").to(torch.bfloat16) for _ in range(4)]
        wout = torch.empty((Bw, Kw), dtype=torch.float32, device="cuda")
        ds.ctx.set_kernel_timing(True)
        for i in range(44):
            binding.convergence_weights(ds.ctx, features=feats[i % 4], tau_seq=0.9, c=2.0, weights=wout)
            if i == 3:
                ds.ctx.read_kernel_timing(7)
        ms, n = ds.ctx.read_kernel_timing(7)
        ds.ctx.set_kernel_timing(False)
        nbytes_w = Bw * Kw * inp.hidden * 2 + Bw * Kw * 4
        gbs = nbytes_w / (ms * 1e-3 / n) / 1e9
        weights = {"seqs": Bw, "seq_len": Kw, "hidden": inp.hidden, "us": ms * 1e3 / n, "bytes": nbytes_w, "GBs": gbs,
                   "hbm_frac": gbs / HBM_PEAK_GBS}
        del feats

    # chained steps through the KV commit until a whole image is formed (context only: synthetic
    # step inputs cycled from a pool; timed once with a stream wait per step and once pipelined)
    loop_out = None
    if args.decode_image > 0 and inp.n_prompts == 1:
        from paper_2605_07230_amd import decode
        pool = [inp] + [wl.make_config(args.workload, args.seed + 1 + i) for i in range(3)]
        for p_ in pool[1:]:
            p_.w = inp.w
        loop = decode.DecodeLoop(pool, args.decode_image, packed_w=packed, cfg_mix=binding.CFG_MIX_HIDDEN if args.cfg_mix == "hidden" else binding.CFG_MIX_LOGITS)
        loop.run(max_steps=5)                           # warm-up
        loop = decode.DecodeLoop(pool, args.decode_image, packed_w=packed, cfg_mix=binding.CFG_MIX_HIDDEN if args.cfg_mix == "hidden" else binding.CFG_MIX_LOGITS)
        lr_sync = loop.run()                            # one stream wait per step
        loop = decode.DecodeLoop(pool, args.decode_image, packed_w=packed, cfg_mix=binding.CFG_MIX_HIDDEN if args.cfg_mix == "hidden" else binding.CFG_MIX_LOGITS)
        lr = loop.run_pipelined()                       # accepted lengths read back two steps late
        assert lr.accept_lens == lr_sync.accept_lens and lr.emitted == lr_sync.emitted
        loop_out = {"image_tokens": args.decode_image, "steps": lr.steps, "tokens": lr.tokens,
                    "mean_accept_len": lr.mean_accept_len, "tvd_per_image": lr.tvd_per_image,
                    "ms_per_image": lr.seconds * 1e3, "ms_per_step": lr.seconds * 1e3 / max(lr.steps, 1),
                    "ms_per_image_synchronous": lr_sync.seconds * 1e3,
                    "ms_per_step_synchronous": lr_sync.seconds * 1e3 / max(lr_sync.steps, 1)}
        del loop

    # the same workload with the guidance mix on the logits (two products), for comparison
    two_products = None
    if head["config"]["cfg_mix"] == "hidden_rows" and not args.no_two_products:
        print("[bench] headline workload, guidance mix on the logits", file=sys.stderr, flush=True)
        _, ds2, h2, _ = measure_workload(args.workload, min(args.steps, 100), min(args.warmup, 10), args, hbm_meas, mfma_meas, cfg_mix="logits")
        two_products = {"ms_per_step": h2["ms_per_step"], "steps_per_s": h2["steps_per_s"], "kernel_us": h2["kernel_us"], "roofline": h2["roofline"]}
        ds2.ctx.close()
        del ds2
        torch.cuda.empty_cache()

    # yardstick for the tiled projection: the vendor GEMM (torch.matmul, bf16 result) on the same
    # rows x hidden x vocab product, W rotated over two copies; it has no guidance combine and writes half
    # the bytes.  Context only: no part of the step calls it.
    vendor = None
    if head["roofline"]["bound"] == "mfma" and not args.no_vendor_gemm:
        try:
            two = ds.h_uncond is not None and head["config"]["cfg_mix"] != "hidden_rows"
            rows_v = inp.n_nodes * (2 if two else 1)                       # as many rows as the projection multiplies
            a_v = torch.cat([ds.h_cond, ds.h_uncond]) if two else ds.h_cond   # the step's own rows
            w_v = [ds.w.t(), ds.w.clone().t()]
            for i in range(4):
                c_v = a_v @ w_v[i % 2]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for i in range(20):
                c_v = a_v @ w_v[i % 2]
            e1.record()
            torch.cuda.synchronize()
            us_v = e0.elapsed_time(e1) * 1e3 / 20
            tf_v = 2.0 * rows_v * inp.hidden * inp.vocab / (us_v * 1e-6) / 1e12
            vendor = {"what": "torch.matmul bf16 [rows, hidden] x [hidden, vocab], bf16 result, no guidance combine",
                      "us": us_v, "TFLOPs": tf_v, "frac": tf_v / MFMA_BF16_PEAK_TFLOPS,
                      "tiled_projection_us": head["kernel_us"]["lmhead"]}
            del a_v, w_v, c_v
        except Exception as exc:   # context only: the step's own figures do not depend on it
            vendor = {"error": repr(exc)}

    ds.ctx.close()
    del ds
    torch.cuda.empty_cache()

    # the other configurations, same protocol, fewer steps
    others = {}
    for tok in [t for t in args.others.split(",") if t.strip()]:
        idx = int(tok)
        if idx == args.workload:
            continue
        print(f"[bench] workload {idx}", file=sys.stderr, flush=True)
        inp_o, ds_o, res_o, _ = measure_workload(idx, args.other_steps, max(5, args.other_steps // 10), args, hbm_meas, mfma_meas)
        others[res_o["workload"]] = res_o
        ds_o.ctx.close()
        del ds_o, inp_o
        torch.cuda.empty_cache()

    out = {
        "metric": "tree_verify_steps_per_s", "value": head["steps_per_s"], "unit": "steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": inp.dtype, "data": "synthetic",
        "config": head["config"],
        "tree_nodes_per_s": head["tree_nodes_per_s"],
        "ms_per_step_with_events": head["ms_per_step_with_events"],
        "ms_per_step_cache_warm": head["ms_per_step_cache_warm"],
        "measured_peaks": {"hbm_read_GBs": hbm_meas, "mfma_bf16_TFLOPs": mfma_meas},
        "kernel_us": head["kernel_us"],
        "accept_len": head["accept_len"],
        "kv_commit": commit,
        "convergence_weights": weights,
        "decode_loop": loop_out,
        "guidance_mix_on_logits": two_products,
        "vendor_gemm_yardstick": vendor,
        "roofline": head["roofline"],
        "roofline_attention": head["roofline_attention"],
        "roofline_row_stats": head["roofline_row_stats"],
        "roofline_attn_accept": head["roofline_attn_accept"],
        "other_workloads": others,
    }
    if not args.no_cpu_baseline:
        print("[bench] CPU checker baseline", file=sys.stderr, flush=True)
        out["cpu_baseline"] = cpu_baseline(inp)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
