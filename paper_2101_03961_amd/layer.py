"""Buffer-owning convenience wrapper around the C ABI.

`SwitchLayer` allocates the output tensors and the workspace with torch (device
memory and streams are all torch is used for) and forwards every call to
`switch_forward` / `switch_backward`.  It performs no arithmetic.
"""
from __future__ import annotations

from typing import Dict, Optional

import torch

from . import binding as B


class SwitchLayer:
    def __init__(self, T: int, d_model: int, d_ff: int, E: int, capacity_factor: float,
                 alpha: float = 0.01, dtype: str = "bf16", device: str = "cuda:0",
                 want_logits: bool = False, n_groups: int = 1, expert_dropout: float = 0.0,
                 jitter_eps: float = 0.0, seed: int = 0, ffn: str = "relu",
                 ntlb_rounds: int = 0, fused_dispatch: bool = False):
        if not torch.cuda.is_available():
            raise RuntimeError("SwitchLayer needs a GPU: the layer runs only in the HIP library")
        self.cfg = B.SwitchConfig(T, d_model, d_ff, E, float(capacity_factor), float(alpha),
                                  B.SW_BF16 if dtype == "bf16" else B.SW_F32,
                                  {"relu": B.SW_FFN_RELU, "geglu": B.SW_FFN_GEGLU}[ffn],
                                  int(n_groups),
                                  float(expert_dropout), float(jitter_eps), int(seed),
                                  int(ntlb_rounds),
                                  B.SW_FLAG_FUSED_DISPATCH if fused_dispatch else 0)
        self.d_in = d_ff * (2 if ffn == "geglu" else 1)   # columns of W_in
        self.device = torch.device(device)
        self.act = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.capacity = B.switch_capacity(self.cfg)
        self.workspace_bytes = B.switch_workspace_size(self.cfg)
        dev = self.device
        # torch's caching allocator hands out 512-byte aligned blocks
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=dev)
        self.y = torch.empty((T, d_model), dtype=self.act, device=dev)
        self.expert_index = torch.empty(T, dtype=torch.int32, device=dev)
        self.gate = torch.empty(T, dtype=torch.float32, device=dev)
        self.position_in_expert = torch.empty(T, dtype=torch.int32, device=dev)
        self.dropped = torch.empty(T, dtype=torch.uint8, device=dev)
        self.expert_counts = torch.empty(E, dtype=torch.int32, device=dev)
        self.aux_loss = torch.empty(1, dtype=torch.float32, device=dev)
        self.router_logits = (torch.empty((T, E), dtype=torch.float32, device=dev)
                              if want_logits else None)
        self.dx = self.dW_r = self.db_r = self.dW_in = self.dW_out = None

    def set_seed(self, seed: int) -> None:
        """Seed of the training-time noise for the next forward + backward pair."""
        self.cfg.seed = int(seed)

    def _stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def _check_inputs(self, x, W_r, W_in, W_out, b_r, dy=None) -> None:
        """The C ABI takes bare pointers: make sure the tensors are what the kernels will read."""
        c = self.cfg
        want = [("x", x, (c.T, c.d_model), self.act), ("W_r", W_r, (c.d_model, c.E), torch.float32),
                ("W_in", W_in, (c.E, c.d_model, self.d_in), self.act),
                ("W_out", W_out, (c.E, c.d_ff, c.d_model), self.act)]
        if b_r is not None:
            want.append(("b_r", b_r, (c.E,), torch.float32))
        if dy is not None:
            want.append(("dy", dy, (c.T, c.d_model), self.act))
        for name, t, shape, dtype in want:
            if tuple(t.shape) != shape or t.dtype != dtype or not t.is_contiguous() \
                    or t.device != self.device:
                raise ValueError("%s must be a contiguous %s tensor of shape %s on %s, got %s %s on %s"
                                 % (name, dtype, shape, self.device, t.dtype, tuple(t.shape), t.device))

    def forward(self, x, W_r, W_in, W_out, b_r=None) -> Dict[str, torch.Tensor]:
        self._check_inputs(x, W_r, W_in, W_out, b_r)
        B.switch_forward(self.cfg, x, W_r, b_r, W_in, W_out, self.y, self.expert_index, self.gate,
                         self.position_in_expert, self.dropped, self.expert_counts, self.aux_loss,
                         self.router_logits, self.workspace, self.workspace_bytes, self._stream())
        return dict(y=self.y, expert_index=self.expert_index, gate=self.gate,
                    position_in_expert=self.position_in_expert, dropped=self.dropped,
                    expert_counts=self.expert_counts, aux_loss=self.aux_loss,
                    router_logits=self.router_logits)

    def alloc_grads(self, with_bias: bool = True) -> None:
        c, dev = self.cfg, self.device
        self.dx = torch.empty((c.T, c.d_model), dtype=self.act, device=dev)
        self.dW_r = torch.empty((c.d_model, c.E), dtype=torch.float32, device=dev)
        self.db_r = torch.empty(c.E, dtype=torch.float32, device=dev) if with_bias else None
        self.dW_in = torch.empty((c.E, c.d_model, self.d_in), dtype=self.act, device=dev)
        self.dW_out = torch.empty((c.E, c.d_ff, c.d_model), dtype=self.act, device=dev)

    def backward(self, dy, x, W_r, W_in, W_out, b_r=None, d_aux: float = 1.0
                 ) -> Dict[str, Optional[torch.Tensor]]:
        self._check_inputs(x, W_r, W_in, W_out, b_r, dy)
        if self.dx is None:
            self.alloc_grads()
        B.switch_backward(self.cfg, dy, d_aux, x, W_r, b_r, W_in, W_out, self.dx, self.dW_r,
                          self.db_r, self.dW_in, self.dW_out, self.workspace, self.workspace_bytes,
                          self._stream())
        return dict(dx=self.dx, dW_r=self.dW_r, db_r=self.db_r, dW_in=self.dW_in,
                    dW_out=self.dW_out)
