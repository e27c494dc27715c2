"""Seeded synthetic inputs for the Switch FFN layer.

This module only draws random tensors.  It contains none of the layer's
arithmetic and is the one piece of code that both the CPU oracle's tests and
the HIP path's tests / benchmark use, so that both sides read the same bits.

Workload recipe (layer shapes follow the paper's model table, Sec. 5.6; the
tensors stand in for C4-derived activations, which the layer's cost does not
depend on beyond shapes and the routing histogram):

  x, dy   ~ N(0, 1)
  W_r     ~ N(0, 0.02^2)                              (fp32 always)
  W_in    ~ truncated N(0, 1/d_model), W_out ~ truncated N(0, 1/d_ff):
            sigma = sqrt(s / fan_in) with s = 1, values beyond two standard
            deviations redrawn (Sec. 2.4, initialisation paragraph + footnote)
  b_r     absent, except for the skewed-routing stress case, where
            b_r[e] = 2 * ln(w_e), w_e = (e + 1)^-1.1  (Zipf weights)

Every tensor is rounded once (round-to-nearest-even) to the configuration's
storage dtype.  Tensors are drawn in the fixed order x, W_r, W_in, W_out, dy
from one torch.Generator seeded with BASE_SEED + the configuration's index.
The generator is device specific (CPU and GPU streams differ); a test draws
on one device and copies, it never draws the "same" tensor twice.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, Optional

import torch

BASE_SEED = 210103961


@dataclass(frozen=True)
class SwitchShape:
    name: str
    T: int
    d_model: int
    d_ff: int
    E: int
    capacity_factor: float
    alpha: float = 0.01
    dtype: str = "bf16"          # storage dtype of x, W_in, W_out, dy: "bf16" or "f32"
    zipf_bias: bool = False      # router bias b_r = 2 ln Zipf(1.1) weights
    seed_index: int = 0
    n_groups: int = 1            # routing groups of T / n_groups consecutive tokens
    expert_dropout: float = 0.0  # training-time noise: dropout rate of the experts' hidden units,
    jitter_eps: float = 0.0      # half-width of the multiplicative jitter on the router's input,
    noise_seed: int = 0          # seed of both
    ntlb_rounds: int = 0         # No-Token-Left-Behind re-routing stages
    ffn: str = "relu"            # expert FFN: "relu", or "geglu" (W_in = [W_g | W_l], [E, d, 2 d_ff])
    fused_dispatch: bool = False      # bf16: dispatch / combine inside the GEMMs, not as separate passes

    def with_(self, **kw) -> "SwitchShape":
        return replace(self, **kw)


CONFIGS: Dict[str, SwitchShape] = {
    c.name: c
    for c in [
        SwitchShape("tiny", 256, 64, 256, 4, 1.25, dtype="f32", seed_index=0),
        SwitchShape("base_cf1.0", 65536, 768, 3072, 128, 1.0, seed_index=1),
        SwitchShape("base_cf1.25", 65536, 768, 3072, 128, 1.25, seed_index=2),
        SwitchShape("base_zipf", 65536, 768, 3072, 128, 1.0, zipf_bias=True, seed_index=3),
        SwitchShape("large", 65536, 1024, 2816, 128, 1.25, seed_index=4),
        SwitchShape("xxl", 16384, 4096, 10240, 64, 1.25, seed_index=5),
        SwitchShape("c_share", 32768, 2080, 6144, 64, 1.0, seed_index=6),
        # the model table's own Switch-Base layer: d_ff 2048 with the gated-GELU FFN
        # (three 768 x 2048 matrices per expert, FLOP-matched to base_cf1.0's two 768 x 3072)
        SwitchShape("base_geglu", 65536, 768, 2048, 128, 1.0, seed_index=7, ffn="geglu"),
        # twice the experts of Switch-Base (the paper's scaling runs go to 256): the router
        # beyond one tile of 128 experts
        SwitchShape("base_e256", 65536, 768, 3072, 256, 1.0, seed_index=8),
    ]
}


def torch_dtype(shape: SwitchShape) -> torch.dtype:
    return {"bf16": torch.bfloat16, "f32": torch.float32}[shape.dtype]


def _normal(gen: torch.Generator, size, std: float, device) -> torch.Tensor:
    return torch.randn(size, generator=gen, device=device, dtype=torch.float32) * std


def _trunc_normal(gen: torch.Generator, size, std: float, device) -> torch.Tensor:
    """N(0, std^2) with every value beyond 2 std redrawn until none is left."""
    w = torch.randn(size, generator=gen, device=device, dtype=torch.float32)
    flat = w.view(-1)
    # Redraw in slabs so that the boolean masks stay small next to the tensor.
    slab = 1 << 26
    for lo in range(0, flat.numel(), slab):
        part = flat[lo:lo + slab]
        bad = part.abs() > 2.0
        n_bad = int(bad.sum())
        while n_bad:
            part[bad] = torch.randn(n_bad, generator=gen, device=device, dtype=torch.float32)
            bad = part.abs() > 2.0
            n_bad = int(bad.sum())
    return w.mul_(std)


def zipf_router_bias(E: int, s: float = 1.1) -> torch.Tensor:
    ranks = torch.arange(1, E + 1, dtype=torch.float64)
    return (2.0 * (-s) * torch.log(ranks)).to(torch.float32)


def make_inputs(shape: SwitchShape, device: str = "cpu",
                seed: Optional[int] = None) -> Dict[str, Optional[torch.Tensor]]:
    """Draw x, W_r, b_r, W_in, W_out, dy for `shape` on `device`."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(BASE_SEED + shape.seed_index if seed is None else seed)
    dt = torch_dtype(shape)
    T, d, f, E = shape.T, shape.d_model, shape.d_ff, shape.E
    x = _normal(gen, (T, d), 1.0, dev).to(dt)
    W_r = _normal(gen, (d, E), 0.02, dev)
    f_in = 2 * f if shape.ffn == "geglu" else f
    W_in = _trunc_normal(gen, (E, d, f_in), 1.0 / math.sqrt(d), dev).to(dt)
    W_out = _trunc_normal(gen, (E, f, d), 1.0 / math.sqrt(f), dev).to(dt)
    dy = _normal(gen, (T, d), 1.0, dev).to(dt)
    b_r = zipf_router_bias(E).to(dev) if shape.zipf_bias else None
    return {"x": x, "W_r": W_r, "b_r": b_r, "W_in": W_in, "W_out": W_out, "dy": dy}
