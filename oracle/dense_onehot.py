"""Second, structurally different oracle for TINY inputs -- TEST INFRASTRUCTURE.

Sec. 5.4 (Eq. 7) states the layer without any gather or scatter: a boolean
dispatch tensor D[token, expert, slot] moves the tokens into fixed-size expert
batches by a tensor contraction, and a float combine tensor (D scaled by the
gate) brings the expert outputs back.  This file builds D straight from the
definitions -- Eq. 1 for the probabilities, the top-1 choice of Sec. 2.1, the
sequence-order rank of Fig. 3 written as an O(T^2) count of earlier tokens with
the same choice, Eq. 3's capacity as the number of slots -- and evaluates the
layer as contractions with D in numpy fp64 (O(T E C) memory: tiny inputs only).
The loss is Eq. 4's sum over experts of f_i P_i (Eqs. 5 and 6).  It is a
cross-check of the index-based C oracle; the two share nothing but numpy.
"""
from __future__ import annotations

import numpy as np


def capacity_real(T: int, E: int, capacity_factor: float) -> float:
    """Eq. 3 as printed: a real number, no rounding."""
    return (T / E) * capacity_factor


def _dispatch_tensor(chosen: np.ndarray, E: int, C: int):
    """D[t, e, c] = 1 iff token t chose expert e and c of its predecessors did too, c < C."""
    T = chosen.shape[0]
    same_choice = chosen[:, None] == chosen[None, :]
    earlier = np.tri(T, T, -1, dtype=bool)                 # [t, s] true iff s < t
    rank = np.count_nonzero(same_choice & earlier, axis=1)
    D = np.zeros((T, E, C), dtype=bool)
    fits = np.flatnonzero(rank < C)
    D[fits, chosen[fits], rank[fits]] = True
    return D, rank


def switch_layer_dense(x, W_r, W_in, W_out, capacity: int, alpha: float, b_r=None):
    x, W_r, W_in, W_out = (np.asarray(a, dtype=np.float64) for a in (x, W_r, W_in, W_out))
    T = x.shape[0]
    E = W_r.shape[1]
    C = int(capacity)

    # Eq. 1
    h = x @ W_r
    if b_r is not None:
        h = h + np.asarray(b_r, dtype=np.float64)
    w = np.exp(h - h.max(axis=1, keepdims=True))
    p = w / w.sum(axis=1, keepdims=True)
    # top-1 (Sec. 2.1): the first expert that attains the row maximum of the logits
    chosen = np.array([int(np.flatnonzero(row == row.max())[0]) for row in h], dtype=np.int64)
    g = p[np.arange(T), chosen]

    # Eqs. 4-6
    f = np.bincount(chosen, minlength=E) / T
    P = p.sum(axis=0) / T
    aux = alpha * E * float(f @ P)

    # Sec. 5.4: dispatch by contraction over the token axis, batched FFN, combine
    D, _ = _dispatch_tensor(chosen, E, C)
    Comb = g[:, None, None] * D
    batches = np.tensordot(D.astype(np.float64), x, axes=([0], [0]))      # [E, C, d]
    outputs = np.maximum(batches @ W_in, 0.0) @ W_out                      # [E, C, d]
    y = np.tensordot(Comb, outputs, axes=([1, 2], [0, 1]))                 # [T, d]
    kept = D.any(axis=(1, 2))
    return dict(y=y, aux_loss=aux, dispatch=D, combine=Comb,
                expert_index=chosen.astype(np.int32), gate=g,
                dropped=(~kept).astype(np.uint8), probs=p)
