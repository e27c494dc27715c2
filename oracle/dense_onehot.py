"""Second, structurally different oracle for TINY inputs -- TEST INFRASTRUCTURE.

The paper's own formulation of the layer (Sec. 5.4, Eq. 7 and Appendix F) never
gathers or scatters: the router emits a boolean dispatch tensor and a float
combine tensor of shape [tokens, experts, capacity] and the layer is three
einsums around a batched FFN.  This file evaluates exactly that in numpy fp64
(O(T*E*C) memory, so tiny inputs only) as a cross-check of the index-based C
oracle; the two share nothing but numpy.

The load-balancing loss is written here the way the appendix computes it --
mean over tokens of the one-hot expert mask, mean over tokens of the router
probabilities, mean over experts of their product, times E squared -- rather
than as Eq. 4's sum, so that the two forms check each other.
"""
from __future__ import annotations

import numpy as np


def capacity_real(T: int, E: int, capacity_factor: float) -> float:
    """Eq. 3 as printed: a real number, no rounding."""
    return (T / E) * capacity_factor


def switch_layer_dense(x, W_r, W_in, W_out, capacity: int, alpha: float, b_r=None):
    x = np.asarray(x, dtype=np.float64)
    W_r = np.asarray(W_r, dtype=np.float64)
    W_in = np.asarray(W_in, dtype=np.float64)
    W_out = np.asarray(W_out, dtype=np.float64)
    T, d = x.shape
    E = W_r.shape[1]
    C = int(capacity)

    router_logits = np.einsum("td,de->te", x, W_r)
    if b_r is not None:
        router_logits = router_logits + np.asarray(b_r, dtype=np.float64)[None, :]
    z = router_logits - router_logits.max(axis=1, keepdims=True)
    router_probs = np.exp(z) / np.exp(z).sum(axis=1, keepdims=True)

    expert_index = router_probs.argmax(axis=1)            # numpy: first maximum
    expert_gate = router_probs.max(axis=1)
    expert_mask = np.eye(E, dtype=np.float64)[expert_index]            # [T, E] one-hot

    # load balancing loss, appendix form
    density = expert_mask.mean(axis=0)
    density_proxy = router_probs.mean(axis=0)
    aux = alpha * np.mean(density_proxy * density) * float(E) ** 2

    # inclusive cumulative count, made exclusive (0-based slot number)
    position = (np.cumsum(expert_mask, axis=0) - 1.0) * expert_mask    # [T, E]
    keep = expert_mask * (position < C)
    keep_flat = keep.sum(axis=1)                                       # [T] 0/1
    slot = position.sum(axis=1).astype(np.int64)                       # rank in chosen expert
    slot_onehot = np.zeros((T, max(C, 1)), dtype=np.float64)
    in_range = slot < C
    slot_onehot[np.arange(T)[in_range], slot[in_range]] = 1.0
    slot_onehot = slot_onehot[:, :C]

    combine = (expert_gate * keep_flat)[:, None, None] * expert_mask[:, :, None] * slot_onehot[:, None, :]
    dispatch = combine != 0.0                                          # [T, E, C] bool

    expert_inputs = np.einsum("td,tec->ecd", x, dispatch.astype(np.float64))
    hidden = np.maximum(np.einsum("ecd,edf->ecf", expert_inputs, W_in), 0.0)
    expert_outputs = np.einsum("ecf,efd->ecd", hidden, W_out)
    y = np.einsum("ecd,tec->td", expert_outputs, combine)
    return dict(y=y, aux_loss=float(aux), dispatch=dispatch, combine=combine,
                expert_index=expert_index.astype(np.int32), gate=expert_gate,
                dropped=(1 - keep_flat).astype(np.uint8), probs=router_probs)
