"""switch_forward_static -- the forward pass on the library's own fixed scratch array, for
callers that cannot allocate -- against switch_forward with a caller workspace: same kernels,
so every output must agree bit for bit, on several calls in a row, each with a smaller input
than the one before (the array then still holds the earlier calls' tables)."""
import numpy as np
import pytest
import torch

import paper_2101_03961_amd as sw
from paper_2101_03961_amd.layer import SwitchLayer
from synth_inputs import SwitchShape, make_inputs

pytestmark = pytest.mark.gpu

OUTPUTS = ("y", "expert_index", "gate", "position_in_expert", "dropped", "expert_counts",
           "aux_loss", "router_logits")


def _both_ways(shape, dev):
    inp = make_inputs(shape, dev)
    layer = SwitchLayer(shape.T, shape.d_model, shape.d_ff, shape.E, shape.capacity_factor,
                        shape.alpha, shape.dtype, device=dev, want_logits=True,
                        n_groups=shape.n_groups, ffn=shape.ffn, ntlb_rounds=shape.ntlb_rounds,
                        fused_dispatch=shape.fused_dispatch)
    assert layer.workspace_bytes <= sw.SW_STATIC_SCRATCH_BYTES
    ref = {k: v.clone() for k, v in
           layer.forward(inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], inp["b_r"]).items()}
    torch.cuda.synchronize()
    for k in OUTPUTS:                      # poison the outputs: the second path must write them all
        getattr(layer, k).fill_(3)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream(layer.device).cuda_stream
    sw.switch_forward_static(layer.cfg, inp["x"], inp["W_r"], inp["b_r"], inp["W_in"], inp["W_out"],
                             layer.y, layer.expert_index, layer.gate, layer.position_in_expert,
                             layer.dropped, layer.expert_counts, layer.aux_loss,
                             layer.router_logits, stream)
    torch.cuda.synchronize()
    for k in OUTPUTS:
        assert torch.equal(getattr(layer, k), ref[k]), (shape.name, k)
    assert float(ref["y"].float().abs().sum()) > 0
    return ref


def test_static_scratch_forward_matches_workspace_forward():
    dev = "cuda:0"
    # first call: bf16, matrix-core router, several tiles per expert, dropping, router bias
    first = SwitchShape("static_first", 3500, 256, 520, 12, 1.0, dtype="bf16", seed_index=120,
                        zipf_bias=True)
    a = _both_ways(first, dev)
    assert int(a["dropped"].sum()) > 0
    # second call, smaller, other dtype and options: groups, re-routing stages
    second = SwitchShape("static_second", 700, 64, 96, 6, 1.25, dtype="f32", seed_index=121,
                         n_groups=2, ntlb_rounds=1)
    _both_ways(second, dev)
    # and a third, smaller again, gated-GELU experts, on the array the two calls left behind
    third = SwitchShape("static_third", 300, 64, 72, 4, 0.75, dtype="bf16", seed_index=122,
                        ffn="geglu")
    _both_ways(third, dev)
    # and one with dispatch and combine inside the GEMMs
    fourth = SwitchShape("static_fourth", 280, 72, 136, 5, 1.0, dtype="bf16", seed_index=123,
                         fused_dispatch=True)
    _both_ways(fourth, dev)


def test_static_scratch_forward_against_the_oracle():
    """The path above compares the two entry points; this one pins the new one to the oracle."""
    import oracle
    dev = "cuda:0"
    s = SwitchShape("static_oracle", 1500, 128, 264, 8, 1.0, dtype="bf16", seed_index=123)
    inp = make_inputs(s, dev)
    layer = SwitchLayer(s.T, s.d_model, s.d_ff, s.E, s.capacity_factor, s.alpha, s.dtype,
                        device=dev, want_logits=True)
    stream = torch.cuda.current_stream(layer.device).cuda_stream
    sw.switch_forward_static(layer.cfg, inp["x"], inp["W_r"], None, inp["W_in"], inp["W_out"],
                             layer.y, layer.expert_index, layer.gate, layer.position_in_expert,
                             layer.dropped, layer.expert_counts, layer.aux_loss,
                             layer.router_logits, stream)
    torch.cuda.synchronize()
    f = lambda t: t.float().cpu().numpy()
    ref = oracle.forward(f(inp["x"]), f(inp["W_r"]), f(inp["W_in"]), f(inp["W_out"]),
                         s.capacity_factor, s.alpha, logits_override=f(layer.router_logits))
    assert np.array_equal(layer.expert_index.cpu().numpy(), ref["expert_index"])
    assert np.array_equal(layer.dropped.cpu().numpy(), ref["dropped"])
    assert np.array_equal(layer.position_in_expert.cpu().numpy(), ref["position_in_expert"])
    y = f(layer.y).astype(np.float64)
    kept = ref["dropped"] == 0
    err = np.linalg.norm(y[kept] - ref["y"][kept], axis=1) / np.linalg.norm(ref["y"][kept], axis=1)
    assert err.max() <= 2e-2, err.max()
    assert np.all(y[~kept] == 0)


def test_static_scratch_refuses_a_configuration_beyond_its_limit():
    big = sw.SwitchConfig(65536, 768, 3072, 128, 1.0, 0.01, sw.SW_BF16)
    with pytest.raises(sw.SwitchError) as ei:
        sw.switch_forward_static(big, *([None] * 13))
    assert ei.value.status == -9
