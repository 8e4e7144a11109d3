"""CPU checker for the convergence weight mask of the drafter-training loss.  TEST INFRASTRUCTURE ONLY.

Eq. 4 (Sec. "Enhancing Drafter Performance"): over a full target-generated sequence of K
positions, the soft cross-entropy term of position k is weighted by c when the consecutive target
predictions (k, k+1) satisfy the convergence set, i.e. cos(F_k, F_{k+1}) >= tau_seq (Eq. 2 applied
to neighbours in the sequence), and by 1 otherwise.  The last position has no successor: weight 1.
c = 2 in the paper's runs (App. "Configuration Details").

Plain numpy float64 loops.  Shares no code with the GPU library.

Pins (tests/test_oracle_weights.py): a library cosine similarity on random rows; constructed rows
with cosines 1, 0, -1 and a zero row; invariance to positive row scaling; last position.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def convergence_weights(features, tau_seq: float, c: float):
    """features [B, K, h] -> (weights [B, K], cos_next [B, K]) with cos_next[:, K-1] = 0."""
    F = np.asarray(features, F64)
    B, K, _ = F.shape
    w = np.ones((B, K), F64)
    cosn = np.zeros((B, K), F64)
    for b in range(B):
        for k in range(K - 1):
            x, y = F[b, k], F[b, k + 1]
            nx, ny = np.sqrt(x @ x), np.sqrt(y @ y)
            cs = float((x @ y) / (nx * ny)) if nx > 0 and ny > 0 else 0.0
            cosn[b, k] = cs
            if cs >= tau_seq:
                w[b, k] = c
    return w, cosn
