"""Multi-step synthetic decode loop: verification steps chained through the KV commit.

Iterative tree decoding (Preliminaries): every step verifies one drafted tree against the prefix,
keeps the accepted path plus one corrected / bonus token, appends the kept tokens' keys and values
to the prefix cache, and repeats until the whole image sequence is formed.  There is no model here:
each step's tree, queries, keys, values, hidden states and uniforms come from a pool of seeded
synthetic step inputs (``workloads.make_config``) that is cycled through, which stands in for a
stochastic drafter and the target's forward pass.  What is real is the chain: the prefix grows by
what the walk accepted, so attention reads what earlier steps committed.

Host logic only; every computation runs in the library's kernels.
"""
from __future__ import annotations

import dataclasses
import time
from typing import List, Optional

import torch

from . import binding


@dataclasses.dataclass
class LoopResult:
    steps: int
    tokens: int                      # emitted tokens (accepted + one correction / bonus per step)
    accept_lens: List[int]
    tvd_used: List[float]
    emitted: List[List[int]]
    seconds: float
    records: Optional[list] = None   # per-step device outputs (only when record=True)

    @property
    def mean_accept_len(self) -> float:
        return sum(self.accept_lens) / max(len(self.accept_lens), 1)

    @property
    def tvd_per_image(self) -> float:
        return float(sum(self.tvd_used))


class DecodeLoop:
    """One prompt (with its guidance row, if any) decoded for ``image_tokens`` tokens."""

    LAG = 2          # steps the host's knowledge of the accepted lengths may trail the device
    RING = 4         # pinned read-back slots (> LAG)

    def __init__(self, pool, image_tokens: int, device: str = "cuda:0", packed_w: bool = True,
                 cfg_mix: int = binding.CFG_MIX_LOGITS):
        first = pool[0]
        if any(p.n_prompts != 1 for p in pool):
            raise ValueError("the decode loop drives one prompt")
        for p in pool[1:]:
            same = (p.dtype, p.cfg, p.n_heads, p.n_kv_heads, p.head_dim, p.hidden, p.vocab) == \
                   (first.dtype, first.cfg, first.n_heads, first.n_kv_heads, first.head_dim, first.hidden, first.vocab)
            if not same:
                raise ValueError("pool entries must share the model shape")
        self.pool = pool
        self.image_tokens = image_tokens
        self.dev = torch.device(device)
        self.dt = torch.bfloat16 if first.dtype == "bf16" else torch.float32
        self.max_depth = max(p.max_depth for p in pool)
        self.max_tree = max(p.n_nodes for p in pool)
        S, P0 = first.n_rows, int(first.prefix_len.max())
        # room for the initial prefix, the image, and the last step's overshoot
        # (the pipelined loop runs up to LAG further steps before it learns that the image is complete)
        self.cap = -(-(P0 + image_tokens + (self.LAG + 1) * (self.max_depth + 1) + 1) // 8) * 8
        self.steps = [binding.DeviceStep(p, device) for p in pool]
        for st in self.steps:
            st.cfg_mix = cfg_mix           # where the projection takes the guidance mix (honoured for packed bf16 weights)
        self.ctx = binding.Context(max_rows=S, max_nodes_total=self.max_tree * S, max_nodes_per_tree=self.max_tree,
                                   max_prefix=self.cap, n_heads=first.n_heads, head_dim=first.head_dim,
                                   hidden=first.hidden, vocab=first.vocab)
        for st in self.steps:      # all steps share one context (one stream, one workspace) and one weight matrix
            st.ctx = self.ctx
            st.w = self.steps[0].w
        self.w_layout = binding.W_ROWMAJOR
        self.w = self.steps[0].w
        if packed_w and first.dtype == "bf16":
            self.w = binding.cascade_pack_lmhead_w(self.ctx, self.steps[0].w)
            self.w_layout = binding.W_PACKED32
        self.k_cache = torch.zeros((1, S, first.n_kv_heads, self.cap, first.head_dim), dtype=self.dt, device=self.dev)
        self.v_cache = torch.zeros_like(self.k_cache)
        self.k_cache[0, :, :, :first.prefix_cap] = self.steps[0].k_cache
        self.v_cache[0, :, :, :first.prefix_cap] = self.steps[0].v_cache
        self.prefix_len = self.steps[0].prefix_len.clone()
        self.prefix_len_next = torch.empty_like(self.prefix_len)
        self.row_prompt = torch.zeros(S, dtype=torch.int32, device=self.dev)
        self.prefix_host = int(first.prefix_len.max())
        self.h_len = torch.empty(self.RING, dtype=torch.int32, pin_memory=True)
        self.h_tvd = torch.empty(self.RING, dtype=torch.float32, pin_memory=True)
        self.h_emit = torch.empty((self.RING, self.max_depth + 1), dtype=torch.int32, pin_memory=True)
        self.done = [torch.cuda.Event() for _ in range(self.RING)]

    def _enqueue_step(self, st, mode: int, max_prefix_len: int, slot: int) -> None:
        """One verification step and its KV commit on the library's stream, then the asynchronous
        read-back of what the host needs into pinned slot `slot` and the event that marks it complete."""
        binding.tree_verify_attn(self.ctx, node_off=st.row_node_off, parent=st.row_parent, prefix_len=self.prefix_len,
                                 q=st.q, k_tree=st.k_tree, v_tree=st.v_tree, k_cache=self.k_cache[0], v_cache=self.v_cache[0],
                                 out=st.attn_out, lse=st.attn_lse, max_nodes_per_tree=st.max_tree,
                                 max_prefix_len=max_prefix_len)
        st.lmhead(self.w, self.w_layout)
        st.accept()
        st.select(mode)
        binding.kv_commit(self.ctx, node_off=st.row_node_off, row_prompt=self.row_prompt, accept_len=st.accept_len,
                          path_nodes=st.path_nodes, k_tree=st.k_tree.unsqueeze(0), v_tree=st.v_tree.unsqueeze(0),
                          k_cache=self.k_cache, v_cache=self.v_cache, prefix_len=self.prefix_len,
                          prefix_len_out=self.prefix_len_next)
        self.prefix_len, self.prefix_len_next = self.prefix_len_next, self.prefix_len
        self.h_len[slot:slot + 1].copy_(st.accept_len, non_blocking=True)
        self.h_tvd[slot:slot + 1].copy_(st.tvd_used, non_blocking=True)
        self.h_emit[slot:slot + 1, :st.emitted.shape[1]].copy_(st.emitted, non_blocking=True)
        self.done[slot].record()

    def run_pipelined(self, mode: int = binding.WALK_SEQUENTIAL) -> LoopResult:
        """The decode loop without a stream wait per step.  The prefix lengths live on the device (the
        commit writes them, the next attention reads them), so the host needs the accepted lengths only
        to know when the image is complete and how large a prefix the next launch must allow for: it
        reads them LAG steps late, passes an upper bound of the prefix (confirmed prefix + a full path
        per unconfirmed step), and discards the at most LAG steps enqueued after the image was complete."""
        accept_lens, tvds, emitted = [], [], []
        tokens, launched, confirmed = 0, 0, 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        complete = False
        while not complete:
            st = self.steps[launched % len(self.steps)]
            bound = self.prefix_host + (launched - confirmed) * (self.max_depth + 1)
            self._enqueue_step(st, mode, bound, launched % self.RING)
            launched += 1
            while confirmed < launched and (launched - confirmed > self.LAG or self.done[confirmed % self.RING].query()):
                slot = confirmed % self.RING
                self.done[slot].synchronize()
                a_len = int(self.h_len[slot])
                accept_lens.append(a_len)
                tvds.append(float(self.h_tvd[slot]))
                emitted.append(self.h_emit[slot, :a_len + 1].tolist())
                self.prefix_host += a_len + 1
                tokens += a_len + 1
                confirmed += 1
                if tokens >= self.image_tokens:
                    complete = True
                    break
        torch.cuda.synchronize()   # the discarded steps still run to their end
        seconds = time.perf_counter() - t0
        if self.ctx.device_status() != binding.OK:
            raise binding.CascadeError(binding.ETREE)
        return LoopResult(steps=confirmed, tokens=tokens, accept_lens=accept_lens, tvd_used=tvds, emitted=emitted,
                          seconds=seconds)

    def run(self, mode: int = binding.WALK_SEQUENTIAL, record: bool = False, max_steps: Optional[int] = None) -> LoopResult:
        accept_lens, tvds, emitted, records = [], [], [], [] if record else None
        tokens, n = 0, 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while tokens < self.image_tokens and (max_steps is None or n < max_steps):
            st = self.steps[n % len(self.steps)]
            self._enqueue_step(st, mode, self.prefix_host, 0)
            # the host needs the accepted length to know how far the image has advanced: three small
            # asynchronous copies into pinned memory and one wait for the stream
            torch.cuda.current_stream().synchronize()
            a_len = int(self.h_len[0])
            accept_lens.append(a_len)
            tvds.append(float(self.h_tvd[0]))
            emitted.append(self.h_emit[0, :a_len + 1].tolist())
            if record:
                records.append(dict(pool_index=n % len(self.steps), attn_out=st.attn_out.float().cpu().numpy(),
                                    logits=st.logits.cpu().numpy(), row_thr=st.row_thr.cpu().numpy(),
                                    row_lse=st.row_lse.cpu().numpy(), accept_len=a_len,
                                    path_nodes=st.path_nodes.cpu().numpy().copy(), emitted=st.emitted.cpu().numpy().copy(),
                                    terminal=int(st.terminal.cpu()[0]), prefix_len=self.prefix_len.cpu().numpy().copy()))
            self.prefix_host += a_len + 1
            tokens += a_len + 1
            n += 1
        torch.cuda.synchronize()
        seconds = time.perf_counter() - t0
        if self.ctx.device_status() != binding.OK:
            raise binding.CascadeError(binding.ETREE)
        return LoopResult(steps=n, tokens=tokens, accept_lens=accept_lens, tvd_used=tvds, emitted=emitted, seconds=seconds,
                          records=records)
