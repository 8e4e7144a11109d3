"""convergence_weights (Eq. 4 mask) on the GPU against the CPU checker."""
import numpy as np
import pytest
import torch

from oracle import weights_oracle as wo
from paper_2605_07230_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _run(F, dtype, tau, c, want_cos=True):
    from paper_2605_07230_amd import binding
    dev = torch.device("cuda:0")
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    B, K, h = F.shape
    feats = torch.from_numpy(F).to(dev).to(dt).contiguous()
    w = torch.full((B, K), -5.0, dtype=torch.float32, device=dev)
    cs = torch.full((B, K), -5.0, dtype=torch.float32, device=dev) if want_cos else None
    ctx = binding.Context(max_rows=1, max_nodes_total=1, max_nodes_per_tree=1, max_prefix=0, n_heads=1, head_dim=64, hidden=64, vocab=64)
    binding.convergence_weights(ctx, features=feats, tau_seq=tau, c=c, weights=w, cos_next=cs)
    assert ctx.device_status() == binding.OK
    return w.cpu().numpy(), None if cs is None else cs.cpu().numpy()


@pytest.mark.parametrize("dtype,B,K,h,tau", [
    ("f32", 1, 33, 512, 0.9),         # two vectors per lane, ragged last run
    ("f32", 3, 1, 64, 0.9),           # single-position sequences
    ("f32", 2, 9, 100, 0.9),          # row shorter than one wave of vectors (25 vectors)
    ("bf16", 2, 577, 4096, 0.94),     # Janus-Pro-shaped image sequence (576 + 1), eight vectors per lane
    ("bf16", 1, 130, 1536, 0.97),     # three vectors per lane -> template of four, masked tail
    ("bf16", 1, 40, 8192, 0.9),       # sixteen vectors per lane
])
def test_weights_match_checker(dtype, B, K, h, tau):
    print(f"[weights] dtype={dtype} B={B} K={K} h={h} tau={tau}", flush=True)
    F = wl.make_feature_sequence(B, K, h, dtype, seed=K + h)
    w, cs = _run(F, dtype, tau, 2.0)
    ew, ecs = wo.convergence_weights(F, tau, 2.0)
    margin = np.abs(ecs[:, :-1] - tau).min() if K > 1 else 1.0
    assert margin > 1e-4, margin          # decisions away from the threshold: a valid exactness test
    np.testing.assert_array_equal(w, ew.astype(np.float32))
    assert np.abs(cs - ecs).max() <= (1e-5 if dtype == "f32" else 1e-4)
    if K > 8:
        assert (ew == 2.0).any() and (ew[:, :-1] == 1.0).any()
    assert (w[:, -1] == 1.0).all() and (cs[:, -1] == 0.0).all()


def test_weights_without_cos_output_and_zero_rows():
    F = wl.make_feature_sequence(2, 20, 256, "f32", seed=1)
    F[0, 5] = 0.0
    F[1, 0] = 0.0
    w, _ = _run(F, "f32", 0.9, 3.0, want_cos=False)
    ew, _ = wo.convergence_weights(F, 0.9, 3.0)
    np.testing.assert_array_equal(w, ew.astype(np.float32))
    assert w[0, 4] == 1.0 and w[0, 5] == 1.0 and w[1, 0] == 1.0


def test_weights_lumina_shaped_full_size_properties():
    """2356-position sequences at hidden 4096: compare all decisions with the checker on a sample of
    sequences, and every row's cosine on the GPU against a torch reduction of the same bf16 data."""
    F = wl.make_feature_sequence(4, 2356, 4096, "bf16", seed=3)
    w, cs = _run(F, "bf16", 0.9, 2.0)
    ew, ecs = wo.convergence_weights(F[:1], 0.9, 2.0)
    far = np.abs(ecs[0, :-1] - 0.9) > 1e-4
    np.testing.assert_array_equal(w[0, :-1][far], ew[0, :-1][far].astype(np.float32))
    t = torch.from_numpy(F).double()
    ref = torch.nn.functional.cosine_similarity(t[:, :-1], t[:, 1:], dim=-1).numpy()
    assert np.abs(cs[:, :-1] - ref).max() <= 1e-4


def test_weights_empty_inputs_are_accepted():
    from paper_2605_07230_amd import binding
    dev = torch.device("cuda:0")
    ctx = binding.Context(max_rows=1, max_nodes_total=1, max_nodes_per_tree=1, max_prefix=0, n_heads=1, head_dim=64, hidden=64, vocab=64)
    feats = torch.zeros((0, 5, 64), dtype=torch.float32, device=dev)
    w = torch.zeros((0, 5), dtype=torch.float32, device=dev)
    # no sequences: nothing is launched; pointers of empty tensors may be null, so pass a dummy buffer
    dummy = torch.zeros(16, dtype=torch.float32, device=dev)
    a = binding.conv_weight_args()
    a.dtype, a.n_seqs, a.seq_len, a.hidden = binding.F32, 0, 5, 64
    a.features, a.tau_seq, a.c, a.weights, a.cos_next = dummy.data_ptr(), 0.9, 2.0, dummy.data_ptr(), None
    import ctypes as C
    assert ctx.lib.convergence_weights(ctx.handle, C.byref(a)) == binding.OK
    a.n_seqs, a.hidden = 1, 65          # 260-byte rows: not a multiple of 16 bytes
    assert ctx.lib.convergence_weights(ctx.handle, C.byref(a)) == binding.ESHAPE
    assert ctx.device_status() == binding.OK
