"""ctypes binding of libcascade_verify.so: argument marshalling only.

Every step of the verification path runs in the HIP library.  torch supplies device
buffers and the stream; nothing here computes.  The four compute functions carry the
names of the C entry points.  If the library cannot be loaded this module raises —
there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcascade_verify.so")

F32, BF16 = 0, 1
WALK_SEQUENTIAL, WALK_LONGEST = 0, 1
FEATURES_HIDDEN, FEATURES_LOGITS = 0, 1
K_ATTN, K_ATTN_MERGE, K_LMHEAD, K_ROW_STATS, K_ACCEPT, K_SELECT = range(6)
W_ROWMAJOR, W_PACKED32 = 0, 1
CFG_MIX_LOGITS, CFG_MIX_HIDDEN = 0, 1
OK, EINVAL, ESHAPE, EDTYPE, ENOMEM, EHIP, ETREE = 0, -1, -2, -3, -4, -5, -6

EXPORTS = ["cascade_create", "cascade_destroy", "cascade_strerror", "cascade_device_status", "cascade_workspace_bytes",
           "cascade_set_kernel_timing", "cascade_read_kernel_timing", "cascade_measure_hbm_read",
           "cascade_measure_mfma_bf16", "cascade_pack_lmhead_w", "tree_verify_attn", "tree_verify_attn_static", "lmhead_softmax_cfg", "cascade_accept", "select_path", "kv_commit", "convergence_weights"]

_vp, _i32, _i64, _f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float


class cascade_limits(C.Structure):
    _fields_ = [("max_rows", _i32), ("max_nodes_total", _i32), ("max_nodes_per_tree", _i32), ("max_prefix", _i32),
                ("n_heads", _i32), ("head_dim", _i32), ("hidden", _i32), ("vocab", _i32)]


class tree_attn_args(C.Structure):
    _fields_ = [("n_rows", _i32), ("node_off", _vp), ("parent", _vp), ("prefix_len", _vp), ("n_nodes_total", _i32),
                ("max_nodes_per_tree", _i32), ("max_prefix_len", _i32), ("dtype", C.c_int), ("n_heads", _i32),
                ("n_kv_heads", _i32), ("head_dim", _i32), ("scale", _f32), ("q", _vp), ("k_tree", _vp), ("v_tree", _vp),
                ("k_cache", _vp), ("v_cache", _vp), ("cache_stride_row", _i64), ("cache_stride_head", _i64),
                ("cache_stride_pos", _i64), ("out", _vp), ("lse", _vp)]


class lmhead_args(C.Structure):
    _fields_ = [("dtype", C.c_int), ("n_nodes", _i32), ("hidden", _i32), ("vocab", _i32), ("h_cond", _vp),
                ("h_uncond", _vp), ("w", _vp), ("w_layout", C.c_int), ("cfg_scale", _f32), ("temperature", _f32), ("top_k", _i32),
                ("cfg_mix", C.c_int), ("logits", _vp), ("row_max", _vp), ("row_thr", _vp), ("row_lse", _vp)]


class accept_args(C.Structure):
    _fields_ = [("h_dtype", C.c_int), ("n_prompts", _i32), ("n_nodes_total", _i32), ("hidden", _i32), ("vocab", _i32),
                ("node_off", _vp), ("parent", _vp), ("token", _vp), ("h_cond", _vp), ("logits", _vp), ("row_thr", _vp),
                ("row_lse", _vp), ("tau_pos", _f32), ("tau_seq", _f32), ("q_tok", _vp), ("m_int", _vp), ("m_conv", _vp),
                ("cos_parent", _vp), ("n_int", _vp), ("n_conv", _vp), ("feature_space", C.c_int)]


class select_args(C.Structure):
    _fields_ = [("n_prompts", _i32), ("n_nodes_total", _i32), ("vocab", _i32), ("max_depth", _i32), ("mode", C.c_int),
                ("node_off", _vp), ("parent", _vp), ("token", _vp), ("q_tok", _vp), ("m_int", _vp), ("m_conv", _vp),
                ("n_int", _vp), ("n_conv", _vp), ("draft_prob", _vp), ("u", _vp), ("u_bonus", _vp), ("eps_tvd", _f32),
                ("logits", _vp), ("row_thr", _vp), ("row_lse", _vp), ("accept_len", _vp), ("path_nodes", _vp),
                ("emitted", _vp), ("terminal", _vp), ("tvd_used", _vp), ("draft_dist", _vp)]


class kv_commit_args(C.Structure):
    _fields_ = [("n_rows", _i32), ("n_prompts", _i32), ("node_off", _vp), ("row_prompt", _vp), ("accept_len", _vp),
                ("path_nodes", _vp), ("max_depth", _i32), ("n_nodes_total", _i32), ("dtype", C.c_int), ("n_layers", _i32),
                ("n_kv_heads", _i32), ("head_dim", _i32), ("k_tree", _vp), ("v_tree", _vp), ("k_cache", _vp), ("v_cache", _vp),
                ("cache_stride_layer", _i64), ("cache_stride_row", _i64), ("cache_stride_head", _i64),
                ("cache_stride_pos", _i64), ("prefix_cap", _i32), ("prefix_len", _vp), ("prefix_len_out", _vp)]


class conv_weight_args(C.Structure):
    _fields_ = [("dtype", C.c_int), ("n_seqs", _i32), ("seq_len", _i32), ("hidden", _i32), ("features", _vp),
                ("tau_seq", _f32), ("c", _f32), ("weights", _vp), ("cos_next", _vp)]


_lib = None


def load_library() -> C.CDLL:
    """Load the HIP library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_07230_amd.build` "
                           "(the verification path has no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    lib.cascade_create.argtypes = [C.POINTER(_vp), C.POINTER(cascade_limits), _vp]
    lib.cascade_create.restype = C.c_int
    lib.cascade_destroy.argtypes = [_vp]
    lib.cascade_destroy.restype = C.c_int
    lib.cascade_strerror.argtypes = [C.c_int]
    lib.cascade_strerror.restype = C.c_char_p
    lib.cascade_device_status.argtypes = [_vp]
    lib.cascade_device_status.restype = C.c_int
    lib.cascade_workspace_bytes.argtypes = [_vp]
    lib.cascade_workspace_bytes.restype = C.c_int64
    lib.cascade_set_kernel_timing.argtypes = [_vp, C.c_int]
    lib.cascade_set_kernel_timing.restype = C.c_int
    lib.cascade_read_kernel_timing.argtypes = [_vp, C.c_int, C.POINTER(C.c_double), C.POINTER(_i32)]
    lib.cascade_read_kernel_timing.restype = C.c_int
    lib.cascade_measure_hbm_read.argtypes = [_vp, _vp, _i64, _i32, C.POINTER(C.c_double)]
    lib.cascade_measure_hbm_read.restype = C.c_int
    lib.cascade_measure_mfma_bf16.argtypes = [_vp, _i32, C.POINTER(C.c_double)]
    lib.cascade_measure_mfma_bf16.restype = C.c_int
    lib.cascade_pack_lmhead_w.argtypes = [_vp, _vp, _i32, _i32, _vp]
    lib.cascade_pack_lmhead_w.restype = C.c_int
    lib.tree_verify_attn_static.argtypes = [_vp, C.POINTER(tree_attn_args), _vp]
    lib.tree_verify_attn_static.restype = C.c_int
    for name, st in (("tree_verify_attn", tree_attn_args), ("lmhead_softmax_cfg", lmhead_args),
                     ("cascade_accept", accept_args), ("select_path", select_args), ("kv_commit", kv_commit_args),
                     ("convergence_weights", conv_weight_args)):
        fn = getattr(lib, name)
        fn.argtypes = [_vp, C.POINTER(st)]
        fn.restype = C.c_int
    _lib = lib
    return lib


class CascadeError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"cascade status {status}: {load_library().cascade_strerror(status).decode()}")


def _check(status: int) -> None:
    if status != OK:
        raise CascadeError(status)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


class Context:
    """Owns a cascade_ctx bound to a torch stream."""

    def __init__(self, *, max_rows, max_nodes_total, max_nodes_per_tree, max_prefix, n_heads, head_dim, hidden, vocab,
                 stream: Optional[torch.cuda.Stream] = None):
        self.lib = load_library()
        self.limits = cascade_limits(max_rows, max_nodes_total, max_nodes_per_tree, max_prefix, n_heads, head_dim, hidden, vocab)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self.handle = _vp()
        _check(self.lib.cascade_create(C.byref(self.handle), C.byref(self.limits), _vp(self.stream.cuda_stream)))

    def close(self) -> None:
        if self.handle:
            self.lib.cascade_destroy(self.handle)
            self.handle = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def device_status(self) -> int:
        return self.lib.cascade_device_status(self.handle)

    def workspace_bytes(self) -> int:
        return int(self.lib.cascade_workspace_bytes(self.handle))

    def set_kernel_timing(self, enable: bool) -> None:
        _check(self.lib.cascade_set_kernel_timing(self.handle, int(enable)))

    def read_kernel_timing(self, kernel_id: int):
        """(total milliseconds, timed launches) of one kernel since the last read."""
        ms, n = C.c_double(), _i32()
        _check(self.lib.cascade_read_kernel_timing(self.handle, kernel_id, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def measure_hbm_read(self, buf, repeats: int = 10) -> float:
        """GB/s this device sustains for a plain streaming read of the tensor `buf`."""
        out = C.c_double()
        _check(self.lib.cascade_measure_hbm_read(self.handle, _ptr(buf), buf.numel() * buf.element_size(), repeats, C.byref(out)))
        return out.value

    def measure_mfma_bf16(self, iters: int = 4096) -> float:
        """TFLOP/s of a register-only bf16 MFMA loop on this device."""
        out = C.c_double()
        _check(self.lib.cascade_measure_mfma_bf16(self.handle, iters, C.byref(out)))
        return out.value


def _tree_attn_args(*, node_off, parent, prefix_len, q, k_tree, v_tree, k_cache, v_cache, out, lse, scale,
                    max_nodes_per_tree, max_prefix_len) -> tree_attn_args:
    a = tree_attn_args()
    a.n_rows = prefix_len.numel()
    a.node_off, a.parent, a.prefix_len = _ptr(node_off), _ptr(parent), _ptr(prefix_len)
    a.n_nodes_total = q.shape[0]
    a.max_nodes_per_tree, a.max_prefix_len = max_nodes_per_tree, max_prefix_len
    a.dtype = _dtype_code(q)
    a.n_heads, a.n_kv_heads, a.head_dim = q.shape[1], k_tree.shape[1], q.shape[2]
    a.scale = scale
    a.q, a.k_tree, a.v_tree = _ptr(q), _ptr(k_tree), _ptr(v_tree)
    a.k_cache, a.v_cache = _ptr(k_cache), _ptr(v_cache)
    if k_cache is not None:
        assert k_cache.stride() == v_cache.stride() and k_cache.stride(3) == 1
        a.cache_stride_row, a.cache_stride_head, a.cache_stride_pos = k_cache.stride(0), k_cache.stride(1), k_cache.stride(2)
    a.out, a.lse = _ptr(out), _ptr(lse)
    return a


def tree_verify_attn(ctx: Context, *, node_off, parent, prefix_len, q, k_tree, v_tree, k_cache, v_cache, out,
                     lse=None, scale: float = 0.0, max_nodes_per_tree: int, max_prefix_len: int) -> None:
    """q/out [N,Hq,D], k_tree/v_tree [N,Hkv,D], k_cache/v_cache [S,Hkv,P_cap,D] (last dim contiguous)."""
    a = _tree_attn_args(node_off=node_off, parent=parent, prefix_len=prefix_len, q=q, k_tree=k_tree, v_tree=v_tree,
                        k_cache=k_cache, v_cache=v_cache, out=out, lse=lse, scale=scale,
                        max_nodes_per_tree=max_nodes_per_tree, max_prefix_len=max_prefix_len)
    _check(ctx.lib.tree_verify_attn(ctx.handle, C.byref(a)))


def tree_verify_attn_static(stream: Optional[torch.cuda.Stream] = None, *, node_off, parent, prefix_len, q, k_tree, v_tree,
                            k_cache, v_cache, out, lse=None, scale: float = 0.0, max_nodes_per_tree: int,
                            max_prefix_len: int, status_out: Optional[torch.Tensor] = None) -> None:
    """The same call without a context: scratch lives in the library's static device array, nothing is
    allocated.  status_out: int32 device tensor of one element that receives the precondition flag word."""
    a = _tree_attn_args(node_off=node_off, parent=parent, prefix_len=prefix_len, q=q, k_tree=k_tree, v_tree=v_tree,
                        k_cache=k_cache, v_cache=v_cache, out=out, lse=lse, scale=scale,
                        max_nodes_per_tree=max_nodes_per_tree, max_prefix_len=max_prefix_len)
    st = stream if stream is not None else torch.cuda.current_stream()
    _check(load_library().tree_verify_attn_static(_vp(st.cuda_stream), C.byref(a), _ptr(status_out)))


def cascade_pack_lmhead_w(ctx: Context, w: torch.Tensor) -> torch.Tensor:
    """One-time repacking of a bf16 [vocab, hidden] LM-head matrix into MFMA operand order (new tensor)."""
    assert w.dtype == torch.bfloat16 and w.is_contiguous()
    out = torch.empty_like(w)
    _check(ctx.lib.cascade_pack_lmhead_w(ctx.handle, _ptr(w), w.shape[0], w.shape[1], _ptr(out)))
    return out


def lmhead_softmax_cfg(ctx: Context, *, h_cond, h_uncond, w, cfg_scale, temperature, top_k, logits, row_max, row_thr, row_lse,
                       w_layout: int = W_ROWMAJOR, cfg_mix: int = CFG_MIX_LOGITS) -> None:
    a = lmhead_args()
    a.dtype = _dtype_code(w)
    a.w_layout = w_layout
    a.cfg_mix = cfg_mix
    a.n_nodes, a.hidden, a.vocab = h_cond.shape[0], h_cond.shape[1], w.shape[0]
    a.h_cond, a.h_uncond, a.w = _ptr(h_cond), _ptr(h_uncond), _ptr(w)
    a.cfg_scale, a.temperature, a.top_k = cfg_scale, temperature, top_k
    a.logits, a.row_max, a.row_thr, a.row_lse = _ptr(logits), _ptr(row_max), _ptr(row_thr), _ptr(row_lse)
    _check(ctx.lib.lmhead_softmax_cfg(ctx.handle, C.byref(a)))


def cascade_accept(ctx: Context, *, node_off, parent, token, h_cond, logits, row_thr, row_lse, tau_pos, tau_seq,
                   q_tok, m_int, m_conv, cos_parent, n_int, n_conv, feature_space: int = FEATURES_HIDDEN) -> None:
    a = accept_args()
    a.feature_space = feature_space
    a.h_dtype = _dtype_code(h_cond)
    a.n_prompts, a.n_nodes_total, a.hidden, a.vocab = node_off.numel() - 1, h_cond.shape[0], h_cond.shape[1], logits.shape[1]
    a.node_off, a.parent, a.token, a.h_cond = _ptr(node_off), _ptr(parent), _ptr(token), _ptr(h_cond)
    a.logits, a.row_thr, a.row_lse = _ptr(logits), _ptr(row_thr), _ptr(row_lse)
    a.tau_pos, a.tau_seq = tau_pos, tau_seq
    a.q_tok, a.m_int, a.m_conv, a.cos_parent = _ptr(q_tok), _ptr(m_int), _ptr(m_conv), _ptr(cos_parent)
    a.n_int, a.n_conv = _ptr(n_int), _ptr(n_conv)
    _check(ctx.lib.cascade_accept(ctx.handle, C.byref(a)))


def select_path(ctx: Context, *, node_off, parent, token, q_tok, m_int, m_conv, n_int, n_conv, draft_prob, u, u_bonus,
                eps_tvd, logits, row_thr, row_lse, max_depth, mode, accept_len, path_nodes, emitted, terminal, tvd_used,
                draft_dist=None) -> None:
    a = select_args()
    a.draft_dist = _ptr(draft_dist)
    a.n_prompts, a.n_nodes_total, a.vocab, a.max_depth, a.mode = node_off.numel() - 1, token.numel(), logits.shape[1], max_depth, mode
    a.node_off, a.parent, a.token = _ptr(node_off), _ptr(parent), _ptr(token)
    a.q_tok, a.m_int, a.m_conv, a.n_int, a.n_conv = _ptr(q_tok), _ptr(m_int), _ptr(m_conv), _ptr(n_int), _ptr(n_conv)
    a.draft_prob, a.u, a.u_bonus, a.eps_tvd = _ptr(draft_prob), _ptr(u), _ptr(u_bonus), eps_tvd
    a.logits, a.row_thr, a.row_lse = _ptr(logits), _ptr(row_thr), _ptr(row_lse)
    a.accept_len, a.path_nodes, a.emitted = _ptr(accept_len), _ptr(path_nodes), _ptr(emitted)
    a.terminal, a.tvd_used = _ptr(terminal), _ptr(tvd_used)
    _check(ctx.lib.select_path(ctx.handle, C.byref(a)))


def kv_commit(ctx: Context, *, node_off, row_prompt, accept_len, path_nodes, k_tree, v_tree, k_cache, v_cache,
              prefix_len, prefix_len_out, n_prompts: Optional[int] = None) -> None:
    """k_tree/v_tree [L,N,Hkv,D]; k_cache/v_cache [L,S,Hkv,cap,D] (last dim contiguous); path_nodes [B,max_depth]."""
    a = kv_commit_args()
    a.n_rows, a.n_prompts = prefix_len.numel(), accept_len.numel() if n_prompts is None else n_prompts
    a.node_off, a.row_prompt, a.accept_len, a.path_nodes = _ptr(node_off), _ptr(row_prompt), _ptr(accept_len), _ptr(path_nodes)
    a.max_depth = path_nodes.shape[1] if path_nodes is not None else 0
    a.n_nodes_total = k_tree.shape[1]
    a.dtype = _dtype_code(k_tree)
    a.n_layers, a.n_kv_heads, a.head_dim = k_tree.shape[0], k_tree.shape[2], k_tree.shape[3]
    assert k_tree.is_contiguous() and v_tree.is_contiguous()
    assert k_cache.stride() == v_cache.stride() and k_cache.stride(4) == 1
    a.k_tree, a.v_tree, a.k_cache, a.v_cache = _ptr(k_tree), _ptr(v_tree), _ptr(k_cache), _ptr(v_cache)
    a.cache_stride_layer, a.cache_stride_row, a.cache_stride_head, a.cache_stride_pos = k_cache.stride()[:4]
    a.prefix_cap = k_cache.shape[3]
    a.prefix_len, a.prefix_len_out = _ptr(prefix_len), _ptr(prefix_len_out)
    _check(ctx.lib.kv_commit(ctx.handle, C.byref(a)))


def convergence_weights(ctx: Context, *, features, tau_seq: float, c: float, weights, cos_next=None) -> None:
    """features [B, K, h] contiguous; weights / cos_next [B, K] float32."""
    a = conv_weight_args()
    assert features.is_contiguous()
    a.dtype = _dtype_code(features)
    a.n_seqs, a.seq_len, a.hidden = features.shape
    a.features, a.tau_seq, a.c = _ptr(features), tau_seq, c
    a.weights, a.cos_next = _ptr(weights), _ptr(cos_next)
    _check(ctx.lib.convergence_weights(ctx.handle, C.byref(a)))


# ------------------------------------------------------------------------------------------------
# convenience: device buffers for a generated workload and one whole step (marshalling only)

class DeviceStep:
    """Uploads a workloads.VerifyInputs record and owns the output buffers of one step."""

    def __init__(self, inp, device="cuda:0", stream: Optional[torch.cuda.Stream] = None, max_tree: Optional[int] = None):
        """max_tree overrides the bound on nodes per tree handed to the library (default: the largest tree)."""
        self.inp = inp
        self.cfg_mix = CFG_MIX_LOGITS     # where lmhead() takes the guidance mix (CFG_MIX_HIDDEN: one product over mixed rows)
        dev = torch.device(device)
        dt = torch.bfloat16 if inp.dtype == "bf16" else torch.float32

        def up(x, dtype=None):
            t = torch.from_numpy(x).to(dev)
            return t.to(dtype) if dtype is not None else t

        self.node_off, self.parent, self.token = up(inp.node_off), up(inp.parent), up(inp.token)
        self.row_node_off, self.row_parent, self.prefix_len = up(inp.row_node_off), up(inp.row_parent), up(inp.prefix_len)
        self.q, self.k_tree, self.v_tree = up(inp.q, dt), up(inp.k_tree, dt), up(inp.v_tree, dt)
        self.k_cache, self.v_cache = up(inp.k_cache, dt), up(inp.v_cache, dt)
        self.h_cond = up(inp.h_cond, dt)
        self.h_uncond = up(inp.h_uncond, dt) if inp.h_uncond is not None else None
        self.w = up(inp.w, dt)
        self.w_packed = None
        self.draft_prob, self.u, self.u_bonus = up(inp.draft_prob), up(inp.u), up(inp.u_bonus)
        N_a, N_c, B = inp.q.shape[0], inp.n_nodes, inp.n_prompts
        self.max_depth = inp.max_depth
        self.max_tree = int((inp.node_off[1:] - inp.node_off[:-1]).max()) if max_tree is None else int(max_tree)
        f32, i32 = torch.float32, torch.int32
        self.attn_out = torch.empty((N_a, inp.n_heads, inp.head_dim), dtype=dt, device=dev)
        self.attn_lse = torch.empty((N_a, inp.n_heads), dtype=f32, device=dev)
        self.logits = torch.empty((N_c, inp.vocab), dtype=f32, device=dev)
        self.row_max, self.row_thr, self.row_lse = (torch.empty(N_c, dtype=f32, device=dev) for _ in range(3))
        self.q_tok, self.m_int, self.m_conv, self.cos_parent = (torch.empty(N_c, dtype=f32, device=dev) for _ in range(4))
        self.n_int, self.n_conv = (torch.empty(N_c, dtype=i32, device=dev) for _ in range(2))
        self.accept_len = torch.empty(B, dtype=i32, device=dev)
        self.path_nodes = torch.empty((B, max(self.max_depth, 1)), dtype=i32, device=dev)
        self.emitted = torch.empty((B, self.max_depth + 1), dtype=i32, device=dev)
        self.terminal = torch.empty(B, dtype=i32, device=dev)
        self.tvd_used = torch.empty(B, dtype=f32, device=dev)
        self.ctx = Context(max_rows=inp.n_rows, max_nodes_total=max(N_a, N_c), max_nodes_per_tree=self.max_tree,
                           max_prefix=int(inp.prefix_len.max()), n_heads=inp.n_heads, head_dim=inp.head_dim,
                           hidden=inp.hidden, vocab=inp.vocab, stream=stream)

    def attn(self):
        tree_verify_attn(self.ctx, node_off=self.row_node_off, parent=self.row_parent, prefix_len=self.prefix_len,
                         q=self.q, k_tree=self.k_tree, v_tree=self.v_tree, k_cache=self.k_cache, v_cache=self.v_cache,
                         out=self.attn_out, lse=self.attn_lse, max_nodes_per_tree=self.max_tree,
                         max_prefix_len=int(self.inp.prefix_len.max()))

    def pack_w(self):
        """Switch the LM head to the packed weight layout (done once, like at model load)."""
        self.w_packed = cascade_pack_lmhead_w(self.ctx, self.w)
        return self.w_packed

    def lmhead(self, w=None, w_layout=None):
        if w is None:
            w = self.w_packed if self.w_packed is not None else self.w
            w_layout = W_PACKED32 if self.w_packed is not None else W_ROWMAJOR
        lmhead_softmax_cfg(self.ctx, h_cond=self.h_cond, h_uncond=self.h_uncond, w=w, w_layout=w_layout or W_ROWMAJOR,
                           cfg_scale=self.inp.cfg_scale, temperature=self.inp.temperature, top_k=self.inp.top_k,
                           logits=self.logits, row_max=self.row_max, row_thr=self.row_thr, row_lse=self.row_lse,
                           cfg_mix=self.cfg_mix)

    def accept(self, tau_pos=None, tau_seq=None, feature_space=FEATURES_HIDDEN):
        cascade_accept(self.ctx, feature_space=feature_space, node_off=self.node_off, parent=self.parent, token=self.token, h_cond=self.h_cond,
                       logits=self.logits, row_thr=self.row_thr, row_lse=self.row_lse,
                       tau_pos=self.inp.tau_pos if tau_pos is None else tau_pos,
                       tau_seq=self.inp.tau_seq if tau_seq is None else tau_seq,
                       q_tok=self.q_tok, m_int=self.m_int, m_conv=self.m_conv, cos_parent=self.cos_parent,
                       n_int=self.n_int, n_conv=self.n_conv)

    def select(self, mode=WALK_SEQUENTIAL, eps_tvd=None, draft_dist=None):
        select_path(self.ctx, draft_dist=draft_dist, node_off=self.node_off, parent=self.parent, token=self.token, q_tok=self.q_tok,
                    m_int=self.m_int, m_conv=self.m_conv, n_int=self.n_int, n_conv=self.n_conv,
                    draft_prob=self.draft_prob, u=self.u, u_bonus=self.u_bonus,
                    eps_tvd=self.inp.eps_tvd if eps_tvd is None else eps_tvd, logits=self.logits,
                    row_thr=self.row_thr, row_lse=self.row_lse, max_depth=self.max_depth, mode=mode,
                    accept_len=self.accept_len, path_nodes=self.path_nodes, emitted=self.emitted,
                    terminal=self.terminal, tvd_used=self.tvd_used)

    def step(self, mode=WALK_SEQUENTIAL, w=None, w_layout=None):
        """One whole verification step: the four calls in order on the context's stream."""
        self.attn()
        self.lmhead(w, w_layout)
        self.accept()
        self.select(mode)
