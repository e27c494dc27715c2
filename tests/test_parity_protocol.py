"""The comparison protocol of tests/parity.py checked on the CPU: its error scales must be
neither vacuous nor tighter than correctly rounded arithmetic, and its helpers must do what
their docstrings say.  (The "GPU" here is the oracle with one operand rounded to bf16.)"""
import numpy as np
import torch

import oracle
from parity import a14, boundary_experts, router_grad_scales, row_errors
from synth_inputs import SwitchShape, make_inputs


def _np_inputs(shape):
    t = make_inputs(shape, "cpu")
    return {k: (None if v is None else v.float().numpy()) for k, v in t.items()}


def _bf16(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).bfloat16().float().numpy()


def _run(npi, s, W_out=None):
    W_out = npi["W_out"] if W_out is None else W_out
    fwd = oracle.forward(npi["x"], npi["W_r"], npi["W_in"], W_out, s.capacity_factor, s.alpha)
    bwd = oracle.backward(npi["x"], npi["W_r"], npi["W_in"], W_out, npi["dy"], fwd, s.alpha, 0.5)
    return fwd, bwd


def test_router_gradient_scale_tracks_a_rounding_sized_perturbation():
    """Rounding the expert outputs' last factor to 8 mantissa bits moves every gate gradient by
    about 2^-9 of its terms' scale.  Measured against router_grad_scales the move is that size
    for a handful of tokens as for thousands (which is the point of the scale), far inside the
    2e-2 bound -- while measured against the gradient itself it is several times larger for the
    handful; and a genuinely wrong term (one token's gate gradient doubled) is far outside."""
    rel_scaled, rel_plain = {}, {}
    for T in (6, 2000):
        s = SwitchShape("t", T, 64, 72, 4, 4.0, dtype="f32", seed_index=210)
        npi = _np_inputs(s)
        fwd, bwd = _run(npi, s)
        _, bwd_r = _run(npi, s, W_out=_bf16(npi["W_out"] * 1.003) / 1.003)
        wr, br = router_grad_scales(npi, fwd, fwd["y"], bwd["dlogits"])
        assert wr.shape == bwd["dW_r"].shape and br.shape == bwd["db_r"].shape
        rel_scaled[T] = row_errors(bwd_r["dW_r"], bwd["dW_r"], 2, wr)[0]
        rel_plain[T] = row_errors(bwd_r["dW_r"], bwd["dW_r"], 2)[0]
        assert 1e-4 < rel_scaled[T] < 6e-3, rel_scaled
        assert row_errors(bwd_r["db_r"], bwd["db_r"], 1, br)[0] < 6e-3
        # a wrong term: token 0's dy doubled (its gate gradient and dO double)
        dy2 = npi["dy"].copy()
        dy2[0] *= 2.0
        bad = oracle.backward(npi["x"], npi["W_r"], npi["W_in"], npi["W_out"], dy2, fwd, s.alpha, 0.5)
        if T == 6:
            assert row_errors(bad["dW_r"], bwd["dW_r"], 2, wr)[0] > 5e-2
    assert rel_scaled[6] < 4 * rel_scaled[2000]


def test_scale_is_the_magnitude_of_the_sum_for_a_large_batch():
    s = SwitchShape("t", 3000, 32, 40, 8, 2.0, dtype="f32", seed_index=211)
    npi = _np_inputs(s)
    fwd, bwd = _run(npi, s)
    wr, br = router_grad_scales(npi, fwd, fwd["y"], bwd["dlogits"])
    ratio = np.sqrt(np.mean(wr ** 2) / np.mean(bwd["dW_r"] ** 2))
    assert 1.0 <= ratio < 3.0, ratio       # not a loophole: the same order as the gradient


def test_a14_and_boundary_experts():
    ref = np.array([[3.0, -4.0], [0.0, 0.0]])
    assert a14(ref, ref) == 0.0
    got = ref.copy()
    got[0, 0] += 0.5
    assert abs(a14(got, ref) - 0.5 / np.sqrt(25.0 / 4.0)) < 1e-15
    nan_ref = np.array([[1.0, np.nan]])
    assert a14(np.array([[1.5, 7.0]]), nan_ref) == 0.5          # rows not evaluated are skipped
    assert boundary_experts(128) == [0, 15, 16, 31, 32, 47, 48, 63, 64, 79, 80, 95, 96, 111, 112, 127]
    assert boundary_experts(4) == [0, 1, 2, 3] and boundary_experts(1) == [0]


def test_router_gradients_compose_over_expert_ranges():
    """compare_full_by_experts adds up the router's gradients range by range: each range's run
    minus the run with no token selected (the auxiliary loss's share), plus that share once,
    is the one-call result (the gradients are linear in the gate gradients)."""
    s = SwitchShape("t", 600, 32, 48, 8, 1.0, dtype="f32", seed_index=212)
    npi = _np_inputs(s)
    args = (npi["x"], npi["W_r"], npi["W_in"], npi["W_out"])
    fwd = oracle.forward(*args, s.capacity_factor, s.alpha)
    full = oracle.backward(*args, npi["dy"], fwd, s.alpha, 0.7)
    aux = oracle.backward(*args, npi["dy"], fwd, s.alpha, 0.7, expert_sel=[], token_sel=[])
    dW_r, db_r, dlog = aux["dW_r"].copy(), aux["db_r"].copy(), aux["dlogits"].copy()
    assert np.abs(aux["dW_r"]).max() > 0          # the loss alone reaches the router
    for c in range(4):
        sel = [2 * c, 2 * c + 1]
        part = oracle.backward(*args, npi["dy"], fwd, s.alpha, 0.7, expert_sel=sel)
        dW_r += part["dW_r"] - aux["dW_r"]
        db_r += part["db_r"] - aux["db_r"]
        mask = np.isin(fwd["expert_index"], sel)
        dlog[mask] = part["dlogits"][mask]
        np.testing.assert_allclose(part["dx"][mask], full["dx"][mask], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(dW_r, full["dW_r"], rtol=0, atol=1e-13 * np.abs(full["dW_r"]).max())
    np.testing.assert_allclose(db_r, full["db_r"], rtol=0, atol=1e-13 * np.abs(full["db_r"]).max())
    np.testing.assert_allclose(dlog, full["dlogits"], rtol=1e-12, atol=1e-18)
