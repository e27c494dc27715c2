"""Helpers for the GPU parity tests (not collected by pytest).

Comparison protocol
  routing stage   The oracle is fed the GPU's own fp32 logits: expert_index,
                  position_in_expert, dropped and expert_counts must then be
                  bit-identical (the arg max is decided on fp32 logits on both
                  sides), gate and aux loss agree to fp32 accuracy.
  end to end      The oracle computes its own fp64 logits.  Logits must agree to
                  fp32 accumulation accuracy, and every token whose arg max
                  differs must have an fp64 top-2 logit gap below 1e-5.
  dense tensors   y and all gradients are compared with the oracle run on its own
                  fp64 logits but with the routing decision pinned to the GPU's
                  expert_index, so that one legitimately flipped near-tie does not
                  shift every later position.
Error metric for dense tensors.  Every tensor is cut into blocks whose elements
share one error scale: a token's output vector (rows of y and dx), one expert's
weight-gradient matrix (dW_in[e], dW_out[e]: a sum over that expert's tokens),
the whole of dW_r and db_r (sums over all tokens):
    block error = ||gpu_blk - ref_blk||_2 / ||ref_blk||_2         (acceptance)
    elem error  = |gpu - ref| / max(|ref|, RMS of its row, RMS of its column in the block)
                                                                  (sanity bound)
Acceptance: max block error <= 1e-5 on the all-fp32 path, <= 2e-2 on the bf16 path
(bf16 storage of A, O and of every output, fp32 accumulation).  This is the
"error normalised by the output RMS" read per output block.  It has to be read
that way: one bf16 rounding alone is up to 2^-8 = 0.4 % of an element, so an
element of 5 RMS is off by 2e-2 RMS even when correctly rounded, and three
roundings in sequence (A, O, y) put the largest of millions of elements at about
2 % of its row's RMS by statistics alone; the block-wise L2 error of correct
arithmetic stays near 0.4 %, while any wrong or missing term (one bad element in
a 768-wide row is 3.6 %) exceeds the bound.  The element-wise sanity bound is
1e-5 (fp32) / 5e-2 (bf16) and is what catches a single bad element in a large
block.  A reference block that is exactly zero must be matched exactly.
ReLU decisions.  1[h > 0] is a decision that floating point takes, like the arg max: where a
pre-activation is zero to fp32 rounding (|h| <= RELU_TIE * RMS of the token's h in the fp64
oracle; about one hidden value in 10^7) the GPU's fp32 sum can come out on the other side, and
that unit's gradient is then legitimately all or nothing.  For those few (token, unit) pairs the
oracle takes whichever decision reproduces the GPU's dx row of that token (resolve_relu_ties);
everything else is compared as usual, against the oracle run with those decisions.  Their
number is bounded by what the normal density of h predicts (a few per ten million units).
Router gradients.  dW_r = x^T dl and db_r = sum_t dl_t are sums over tokens of terms that
cancel (the rows of dl sum to zero, dy has zero mean), and each term hangs on the gate gradient
dg_t = <dy_t, o_t>, a d_model-term dot product of mixed signs whose rounding error scales with
|dy_t| |o_t| / sqrt(d_model), not with dg_t.  Their errors are therefore normalised by the
scale of the terms, from the oracle's own quantities (router_grad_scales):
    dl_scale[t][j]^2 = dl[t][j]^2 + (p[t][j] |1[j = e_t] - p[t][e_t]| |dy_t| |o_t| / sqrt(d))^2
    scale(dW_r[k][j]) = sqrt(sum_t x[t][k]^2 dl_scale[t][j]^2),  scale(db_r[j]) = sqrt(sum_t dl_scale[t][j]^2)
(the second factor is |d dl[t][j] / d dg_t|); for a well-conditioned batch this is the
magnitude of the sum itself, for a handful of tokens it is what one badly conditioned dot
product can move.  The same bounds (1e-5 / 2e-2 block-wise, 1e-5 / 5e-2 per element) apply.
Every report also carries max |gpu - ref| / RMS(ref) per tensor (`a14`), the plain reading
of "error normalised by the output RMS", for information.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2101_03961_amd.layer import SwitchLayer

TOL = {"f32": 1e-5, "bf16": 2e-2}          # max block-wise relative L2 error
ELEM_TOL = {"f32": 1e-5, "bf16": 5e-2}     # max element error, floor = row / column RMS
LOGIT_ATOL = 2e-5      # fp32 accumulation of d_model products against fp64
GAP_RULE = 1e-5        # arg max may differ only below this fp64 top-2 logit gap
RELU_TIE = 1e-6        # |h| / RMS(h_t) below which the ReLU decision may differ


def to_np(t: torch.Tensor) -> np.ndarray:
    if t.dtype in (torch.bfloat16, torch.float16):
        t = t.float()
    return t.detach().cpu().numpy()


def np_inputs(inp):
    return {k: (None if v is None else to_np(v)) for k, v in inp.items()}


# trailing dimensions that form one error block, per tensor
BLOCK_DIMS = {"y": 1, "dx": 1, "dW_in": 2, "dW_out": 2, "dW_r": 2, "db_r": 1}


def row_errors(a: np.ndarray, ref: np.ndarray, block_dims: int = 1, scale=None):
    """(max block-wise relative L2 error, max element error) -- see module docstring.
    scale: optional magnitudes (same shape as ref) to normalise by instead of ref itself."""
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert a.shape == ref.shape, (a.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0
    if scale is not None:
        scale = np.maximum(np.abs(np.asarray(scale, dtype=np.float64)), np.abs(ref))
        diff = a - ref
        nrm = np.sqrt(np.mean(scale * scale))
        if nrm == 0.0:
            return (0.0, 0.0) if not diff.any() else (float("inf"), float("inf"))
        return float(np.sqrt(np.mean(diff * diff)) / nrm), float(np.max(np.abs(diff) / np.where(scale == 0, nrm, scale)))
    cols = ref.shape[-1] if ref.ndim else 1
    rows = ref.shape[-2] if (block_dims == 2 and ref.ndim >= 2) else 1
    a3, r3 = a.reshape(-1, rows, cols), ref.reshape(-1, rows, cols)
    diff = a3 - r3
    blk_rms = np.sqrt(np.mean(r3 * r3, axis=(1, 2)))
    # a reference block that is zero, or fp64 rounding noise of an exact zero (1e-14 of the
    # tensor's scale; e.g. the loss gradient of a token when all experts got the same count),
    # has to be matched by (the same kind of) zero
    all_rms = np.sqrt(np.mean(r3 * r3))
    zero = blk_rms <= 1e-14 * all_rms
    if zero.any():
        if np.any(np.abs(diff[zero]) > 1e-12 * all_rms):
            return float("inf"), float("inf")
        if zero.all():
            return 0.0, 0.0
        diff, r3, blk_rms = diff[~zero], r3[~zero], blk_rms[~zero]
    blk = np.sqrt(np.mean(diff * diff, axis=(1, 2))) / blk_rms
    # element floor: the element itself, or the RMS of its row / its column inside
    # the block (a weight-gradient element's error scales with the norms of the
    # activation column and the gradient column that meet in it)
    floor = np.maximum(np.abs(r3), np.sqrt(np.mean(r3 * r3, axis=2, keepdims=True)))
    if rows > 1:
        floor = np.maximum(floor, np.sqrt(np.mean(r3 * r3, axis=1, keepdims=True)))
    floor = np.where(floor == 0.0, blk_rms[:, None, None], floor)
    elem = np.abs(diff) / floor
    return float(blk.max()), float(elem.max())


def assert_close(name, a, ref, dtype, scale=None):
    """Block-wise and element-wise bounds of the module docstring.  `scale`: see row_errors."""
    assert np.all(np.isfinite(a)), name + " has non-finite values"
    row, elem = row_errors(a, ref, BLOCK_DIMS[name.split("[")[0]], scale)
    tol, etol = TOL[dtype], ELEM_TOL[dtype]
    assert row <= tol, "%s: max block error %.3e > %.1e" % (name, row, tol)
    assert elem <= etol, "%s: max element error %.3e > %.1e" % (name, elem, etol)
    return row


def a14(a, ref) -> float:
    """max |a - ref| / RMS(ref) over the whole tensor (reported, not bounded: see docstring)."""
    ref = np.asarray(ref, dtype=np.float64)
    ok = np.isfinite(ref)
    if not ok.any():
        return 0.0
    rms = np.sqrt(np.mean(ref[ok] ** 2))
    if rms == 0.0:
        return 0.0
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64)[ok] - ref[ok])) / rms)


def router_grad_scales(npi, fwd, y_ref, dlogits, dy=None):
    """(scale of dW_r [d, E], scale of db_r [E]): the magnitudes that the rounding errors of the
    router's weight gradients scale with, from the oracle's quantities (module docstring).
    y_ref: the oracle's output (rows it did not evaluate are NaN: their dy must be zero)."""
    x = np.asarray(npi["x"], dtype=np.float64)
    dy = np.asarray(npi["dy"] if dy is None else dy, dtype=np.float64)
    T, d = x.shape
    e = np.asarray(fwd["expert_index"])
    p = np.asarray(fwd["probs"], dtype=np.float64)
    g = np.asarray(fwd["gate"], dtype=np.float64)
    live = (np.asarray(fwd["dropped"]) == 0) & np.isfinite(y_ref).all(axis=1)
    o_norm = np.zeros(T)
    o_norm[live] = np.linalg.norm(y_ref[live], axis=1) / g[live]          # y = g o
    dg_scale = np.linalg.norm(dy, axis=1) * o_norm / np.sqrt(d)
    pe = p[np.arange(T), e]
    sens = p * pe[:, None]                                                 # j != e_t: p_j p_e
    sens[np.arange(T), e] = pe * (1.0 - pe)                                # j  = e_t
    dls2 = np.asarray(dlogits, dtype=np.float64) ** 2 + (sens * dg_scale[:, None]) ** 2
    return np.sqrt((x * x).T @ dls2), np.sqrt(dls2.sum(axis=0))


def noise_of(shape):
    """The shape's training-time noise as the oracle takes it (None when off)."""
    if shape.expert_dropout == 0 and shape.jitter_eps == 0:
        return None
    return (shape.expert_dropout, shape.jitter_eps, shape.noise_seed)


def run_gpu(shape, inp, d_aux=1.0, backward=True, dy=None):
    """One forward (+ backward) through the C ABI; returns (layer, numpy dict)."""
    layer = SwitchLayer(shape.T, shape.d_model, shape.d_ff, shape.E, shape.capacity_factor,
                        shape.alpha, shape.dtype, device=str(inp["x"].device), want_logits=True,
                        n_groups=shape.n_groups, expert_dropout=shape.expert_dropout,
                        jitter_eps=shape.jitter_eps, seed=shape.noise_seed, ffn=shape.ffn,
                        ntlb_rounds=shape.ntlb_rounds, fused_dispatch=shape.fused_dispatch)
    out = layer.forward(inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], inp["b_r"])
    res = {k: to_np(v) for k, v in out.items() if v is not None}
    if backward:
        g = layer.backward(inp["dy"] if dy is None else dy, inp["x"], inp["W_r"], inp["W_in"],
                           inp["W_out"], inp["b_r"], d_aux)
        res.update({k: to_np(v) for k, v in g.items() if v is not None})
    torch.cuda.synchronize()
    return layer, res


def check_routing(shape, npi, gpu):
    """Routing-stage and end-to-end checks; returns the oracle forward (no FFN)
    on fp64 logits with routing pinned to the GPU's expert_index."""
    T, E = shape.T, shape.E
    # (i) routing stage on identical logits: bit exact
    same = oracle.forward(npi["x"], npi["W_r"], npi["W_in"], npi["W_out"], shape.capacity_factor,
                          shape.alpha, b_r=npi["b_r"], logits_override=gpu["router_logits"],
                          skip_ffn=True, n_groups=shape.n_groups, noise=noise_of(shape), ffn=shape.ffn,
                          ntlb_rounds=shape.ntlb_rounds)
    assert np.array_equal(gpu["expert_index"], same["expert_index"]), "expert_index"
    assert np.array_equal(gpu["position_in_expert"], same["position_in_expert"]), "position"
    assert np.array_equal(gpu["dropped"], same["dropped"]), "dropped"
    assert np.array_equal(gpu["expert_counts"].astype(np.int64), same["expert_counts"]), "counts"
    assert int(gpu["expert_counts"].sum()) == T
    np.testing.assert_allclose(gpu["gate"], same["gate"], rtol=1e-5, atol=0)
    assert abs(float(gpu["aux_loss"][0]) - same["aux_loss"]) <= 1e-5 * abs(same["aux_loss"])
    # (ii) end to end against fp64 logits
    h64 = oracle.logits(npi["x"], npi["W_r"], npi["b_r"], noise_of(shape))
    assert np.max(np.abs(gpu["router_logits"] - h64)) <= LOGIT_ATOL * max(1.0, np.abs(h64).max())
    e64 = h64.argmax(axis=1)
    # (with re-routing stages expert_index is the processing expert: the arg max decisions,
    # and what each token asked for in the later stages, are those of the run on the GPU's
    # logits, which (i) has just shown to be the GPU's)
    flipped = np.nonzero(e64 != same["first_choice"])[0]
    if flipped.size:
        srt = np.sort(h64[flipped], axis=1)
        gap = srt[:, -1] - srt[:, -2]
        assert np.all(gap < GAP_RULE), "arg max differs at a gap of %.3e" % gap.max()
    pinned = oracle.forward(npi["x"], npi["W_r"], npi["W_in"], npi["W_out"],
                            shape.capacity_factor, shape.alpha, b_r=npi["b_r"],
                            logits_override=h64, expert_index_override=same["first_choice"],
                            skip_ffn=True, n_groups=shape.n_groups, noise=noise_of(shape), ffn=shape.ffn,
                            ntlb_rounds=shape.ntlb_rounds,
                            ntlb_choices_override=same["ntlb_choices"])
    assert np.array_equal(gpu["expert_index"], pinned["expert_index"])
    assert np.array_equal(gpu["dropped"], pinned["dropped"])
    np.testing.assert_allclose(gpu["gate"], pinned["gate"], rtol=3e-5, atol=0)
    assert abs(float(gpu["aux_loss"][0]) - pinned["aux_loss"]) <= 1e-5 * abs(pinned["aux_loss"])
    return pinned, int(flipped.size)


def check_dropped_rows_are_zero(gpu, dtype):
    drop = gpu["dropped"].astype(bool)
    rows = gpu["y"][drop]
    assert np.all(rows == 0.0) and not np.any(np.signbit(rows)), "dropped rows must be +0"


# P(|h| <= RELU_TIE * RMS) for a normal h: 2 * RELU_TIE * phi(0)
TIE_RATE = 2.0 * RELU_TIE * 0.3989422804014327


def resolve_relu_ties(shape, npi, fwd, gpu_dx, d_aux, expert_sel=None, token_sel=None):
    """(token, unit) pairs, among the evaluated tokens' pre-activations that are zero to fp32
    rounding, whose ReLU gate the GPU took the other way: decided per token by which choice
    reproduces the GPU's dx row.  Almost always empty.  (The gated-GELU FFN is smooth: none.)
    All tokens with such a unit are evaluated together, one oracle run per combination of
    "q-th undecidable unit of the token flipped" (two runs when no token has two)."""
    if shape.ffn != "relu":
        return []
    near = oracle.hidden_near_zero(npi["x"], npi["W_in"], fwd["expert_index"], fwd["dropped"],
                                   RELU_TIE, expert_sel=expert_sel, token_sel=token_sel)
    # no more of them than the density of h predicts: the rule must stay an exception
    e = np.asarray(fwd["expert_index"])
    evaluated = np.asarray(fwd["dropped"]) == 0
    if expert_sel is not None or token_sel is not None:
        sel = np.isin(e, list(expert_sel or []))
        sel[np.asarray(list(token_sel if token_sel is not None else []), dtype=np.int64)] = True
        evaluated &= sel
    units = float(evaluated.sum()) * shape.d_ff
    assert len(near) <= 8 + 4.0 * TIE_RATE * units, \
        "%d hidden units within %.0e of zero among %.3g: more than rounding explains" % (
            len(near), RELU_TIE, units)
    by_token = {}
    for t, j, _ in near:
        by_token.setdefault(t, []).append(j)
    if not by_token:
        return []
    toks = sorted(by_token)
    most = max(len(u) for u in by_token.values())
    assert most <= 4, "too many undecidable units in one token"
    best = {t: (np.inf, []) for t in toks}
    for mask in range(1 << most):
        cand = [(t, j) for t in toks for q, j in enumerate(by_token[t]) if (mask >> q) & 1]
        ref = oracle.backward(npi["x"], npi["W_r"], npi["W_in"], npi["W_out"], npi["dy"], fwd,
                              shape.alpha, d_aux, token_sel=toks, relu_flips=cand)["dx"]
        for t in toks:
            err = np.linalg.norm(gpu_dx[t] - ref[t])
            if err < best[t][0]:
                best[t] = (err, [c for c in cand if c[0] == t])
    return [c for t in toks for c in best[t][1]]


DENSE = ("y", "dx", "dW_r", "db_r", "dW_in", "dW_out")


def compare_full(shape, inp, d_aux=1.0):
    """Whole-tensor parity of forward and backward; returns a dict of errors."""
    tol = shape.dtype
    npi = np_inputs(inp)
    _, gpu = run_gpu(shape, inp, d_aux)
    fwd, flips = check_routing(shape, npi, gpu)
    fwd["y"] = oracle.expert_ffn(npi["x"], npi["W_in"], npi["W_out"], fwd["expert_index"],
                                 fwd["dropped"], fwd["gate"], noise=noise_of(shape), ffn=shape.ffn)
    errs = {"flips": flips}
    errs["y"] = assert_close("y", gpu["y"], fwd["y"], tol)
    check_dropped_rows_are_zero(gpu, shape.dtype)
    ties = resolve_relu_ties(shape, npi, fwd, gpu["dx"], d_aux)
    errs["relu_ties"] = len(ties)
    bwd = oracle.backward(npi["x"], npi["W_r"], npi["W_in"], npi["W_out"], npi["dy"], fwd,
                          shape.alpha, d_aux, relu_flips=ties)
    for k in ("dx", "dW_in", "dW_out"):
        errs[k] = assert_close(k, gpu[k], bwd[k], tol)
    wr_scale, br_scale = router_grad_scales(npi, fwd, fwd["y"], bwd["dlogits"])
    errs["dW_r"] = assert_close("dW_r", gpu["dW_r"], bwd["dW_r"], tol, scale=wr_scale)
    errs["db_r"] = assert_close("db_r", gpu["db_r"], bwd["db_r"], tol, scale=br_scale)
    ref = dict(bwd, y=fwd["y"])
    errs["a14"] = {k: float("%.2e" % a14(gpu[k], ref[k])) for k in DENSE}
    return errs, gpu, fwd, bwd


class FullByExperts:
    """compare_full for layers where one oracle call would run for minutes: the same complete
    comparison -- every token's rows of y and dx, every expert's weight gradients, the router's --
    with the oracle evaluated for one range of experts at a time (its partial evaluation is
    pinned against the full run by the CPU tests), so that a caller can report after each range.
    The router's gradients are linear in the gate gradients: each range contributes its tokens'
    share on top of the auxiliary loss's, which a run with no token selected gives alone.
    Use: the constructor (GPU run, routing on all tokens), ranges 0 .. n_chunks - 1 in any order,
    then router()."""

    def __init__(self, shape, inp, n_chunks=8, d_aux=1.0):
        self.shape, self.n_chunks, self.d_aux = shape, n_chunks, d_aux
        self.npi = np_inputs(inp)
        _, self.gpu = run_gpu(shape, inp, d_aux)
        for k in DENSE:
            assert np.all(np.isfinite(self.gpu[k])), k + " has non-finite values"
        self.fwd, flips = check_routing(shape, self.npi, self.gpu)
        check_dropped_rows_are_zero(self.gpu, shape.dtype)
        npi = self.npi
        self.args = (npi["x"], npi["W_r"], npi["W_in"], npi["W_out"])
        self.aux = oracle.backward(*self.args, npi["dy"], self.fwd, shape.alpha, d_aux,
                                   expert_sel=[], token_sel=[])
        self.dW_r, self.db_r = self.aux["dW_r"].copy(), self.aux["db_r"].copy()
        self.dlog = self.aux["dlogits"].copy()
        self.y_ref = np.full(self.gpu["y"].shape, np.nan)
        self.errs = {"flips": flips, "relu_ties": 0, "y": 0.0, "dx": 0.0, "dW_in": 0.0, "dW_out": 0.0}
        self.worst = {k: 0.0 for k in ("y", "dx", "dW_in", "dW_out")}
        self.done = set()

    def experts_of(self, c):
        E = self.shape.E
        return list(range(c * E // self.n_chunks, (c + 1) * E // self.n_chunks))

    def chunk(self, c):
        """Range c against the oracle; returns a progress line."""
        shape, npi, gpu, fwd, errs, worst = self.shape, self.npi, self.gpu, self.fwd, self.errs, self.worst
        tol = shape.dtype
        sel = self.experts_of(c)
        assert c not in self.done
        self.done.add(c)
        if not sel:
            return "[by experts] range %d is empty" % c
        tmask = np.isin(fwd["expert_index"], sel)
        y_c = oracle.expert_ffn(npi["x"], npi["W_in"], npi["W_out"], fwd["expert_index"],
                                fwd["dropped"], fwd["gate"], expert_sel=sel, noise=noise_of(shape),
                                ffn=shape.ffn)
        errs["y"] = max(errs["y"], assert_close("y[experts %d..]" % sel[0], gpu["y"][tmask], y_c[tmask], tol))
        ties = resolve_relu_ties(shape, npi, fwd, gpu["dx"], self.d_aux, expert_sel=sel)
        errs["relu_ties"] += len(ties)
        bwd = oracle.backward(*self.args, npi["dy"], fwd, shape.alpha, self.d_aux, expert_sel=sel,
                              relu_flips=ties)
        errs["dx"] = max(errs["dx"], assert_close("dx[experts %d..]" % sel[0], gpu["dx"][tmask],
                                                  bwd["dx"][tmask], tol))
        errs["dW_in"] = max(errs["dW_in"], assert_close("dW_in[%d..]" % sel[0], gpu["dW_in"][sel],
                                                        bwd["dW_in"], tol))
        errs["dW_out"] = max(errs["dW_out"], assert_close("dW_out[%d..]" % sel[0],
                                                          gpu["dW_out"][sel], bwd["dW_out"], tol))
        worst["y"] = max(worst["y"], a14(gpu["y"][tmask], y_c[tmask]))
        worst["dx"] = max(worst["dx"], a14(gpu["dx"][tmask], bwd["dx"][tmask]))
        worst["dW_in"] = max(worst["dW_in"], a14(gpu["dW_in"][sel], bwd["dW_in"]))
        worst["dW_out"] = max(worst["dW_out"], a14(gpu["dW_out"][sel], bwd["dW_out"]))
        self.dW_r += bwd["dW_r"] - self.aux["dW_r"]
        self.db_r += bwd["db_r"] - self.aux["db_r"]
        self.dlog[tmask] = bwd["dlogits"][tmask]
        self.y_ref[tmask] = y_c[tmask]
        return ("[by experts] experts %d..%d: %d tokens, block errors y %.2e dx %.2e dW_in %.2e dW_out %.2e"
                % (sel[0], sel[-1], int(tmask.sum()), errs["y"], errs["dx"], errs["dW_in"], errs["dW_out"]))

    def router(self):
        """The router's gradients, once every range has added its share; returns all errors."""
        assert self.done == set(range(self.n_chunks)), "ranges not compared: %s" % (
            sorted(set(range(self.n_chunks)) - self.done),)
        assert not np.isnan(self.y_ref).any()          # every token belonged to a range
        gpu, errs, worst, tol = self.gpu, self.errs, self.worst, self.shape.dtype
        wr_scale, br_scale = router_grad_scales(self.npi, self.fwd, self.y_ref, self.dlog)
        errs["dW_r"] = assert_close("dW_r", gpu["dW_r"], self.dW_r, tol, scale=wr_scale)
        errs["db_r"] = assert_close("db_r", gpu["db_r"], self.db_r, tol, scale=br_scale)
        worst["dW_r"], worst["db_r"] = a14(gpu["dW_r"], self.dW_r), a14(gpu["db_r"], self.db_r)
        errs["a14"] = {k: float("%.2e" % v) for k, v in worst.items()}
        return errs


def compare_full_by_experts(shape, inp, n_chunks=8, d_aux=1.0, progress=print):
    """FullByExperts in one call, a progress line after each range."""
    run = FullByExperts(shape, inp, n_chunks, d_aux)
    progress("[by experts] routing checked on all %d tokens" % shape.T)
    for c in range(n_chunks):
        progress(run.chunk(c))
    return run.router(), run.gpu, run.fwd


def boundary_experts(E: int, ranges: int = 8):
    """First and last expert of each of `ranges` equal cuts of the expert axis: the bf16 grouped
    GEMMs cut their tile list (expert-major) into that many ranges, one per XCD, and some of
    them walk it backwards, so these are the experts where a range starts, ends or turns."""
    out = set()
    for r in range(ranges):
        lo, hi = (r * E) // ranges, ((r + 1) * E + ranges - 1) // ranges - 1
        if lo <= hi:
            out.update((lo, min(hi, E - 1)))
    return sorted(out)


def compare_sampled(shape, inp, n_experts=3, n_tokens=32, d_aux=1.0, seed=0):
    """Parity at sizes where the full fp64 oracle is too slow: routing on all tokens; every
    output finite everywhere; the expert FFN forward/backward on up to n_experts whole experts
    -- always the fullest and the emptiest non-empty one, then the experts at the edges of the
    GEMMs' tile ranges (boundary_experts; evenly thinned if there are more than fit), then random
    ones -- plus a few single tokens; router weight gradients with dy zeroed outside those
    tokens."""
    tol = shape.dtype
    npi = np_inputs(inp)
    layer, gpu = run_gpu(shape, inp, d_aux)
    for k in DENSE:
        assert np.all(np.isfinite(gpu[k])), k + " has non-finite values"
    fwd, flips = check_routing(shape, npi, gpu)
    counts = fwd["expert_counts"]
    rng = np.random.default_rng(seed)
    nonempty = np.nonzero(counts > 0)[0]
    order = nonempty[np.argsort(counts[nonempty], kind="stable")]
    sel = [int(order[-1]), int(order[0])]
    edges = [e for e in boundary_experts(shape.E) if counts[e] > 0 and e not in sel]
    room = max(0, min(n_experts, len(nonempty)) - len(set(sel)))
    if len(edges) > room:       # thin evenly, keeping the first and the last
        edges = [edges[i] for i in sorted(set(np.linspace(0, len(edges) - 1, room).astype(int)))] if room else []
    sel = set(sel + edges)
    while len(sel) < min(n_experts, len(nonempty)):
        sel.add(int(rng.choice(nonempty)))
    sel = sorted(sel)
    toks = rng.choice(shape.T, size=min(n_tokens, shape.T), replace=False)
    drop_idx = np.nonzero(fwd["dropped"])[0]
    if drop_idx.size:
        toks = np.concatenate([toks, drop_idx[:4]])
    tmask = np.isin(fwd["expert_index"], sel)
    tmask[toks] = True

    y_ref = oracle.expert_ffn(npi["x"], npi["W_in"], npi["W_out"], fwd["expert_index"],
                              fwd["dropped"], fwd["gate"], expert_sel=sel, token_sel=toks,
                              noise=noise_of(shape), ffn=shape.ffn)
    errs = {"flips": flips, "experts": sel, "tokens_checked": int(tmask.sum())}
    errs["y"] = assert_close("y[sampled]", gpu["y"][tmask], y_ref[tmask], tol)
    check_dropped_rows_are_zero(gpu, shape.dtype)

    ties = resolve_relu_ties(shape, npi, fwd, gpu["dx"], d_aux, expert_sel=sel, token_sel=toks)
    errs["relu_ties"] = len(ties)
    bwd = oracle.backward(npi["x"], npi["W_r"], npi["W_in"], npi["W_out"], npi["dy"], fwd,
                          shape.alpha, d_aux, expert_sel=sel, token_sel=toks, relu_flips=ties)
    errs["dx"] = assert_close("dx[sampled]", gpu["dx"][tmask], bwd["dx"][tmask], tol)
    errs["dW_in"] = assert_close("dW_in[sel]", gpu["dW_in"][sel], bwd["dW_in"], tol)
    errs["dW_out"] = assert_close("dW_out[sel]", gpu["dW_out"][sel], bwd["dW_out"], tol)
    processed = np.bincount(fwd["expert_index"][fwd["dropped"] == 0], minlength=shape.E)
    empty = np.nonzero(processed == 0)[0]
    if empty.size:
        assert np.all(gpu["dW_in"][empty] == 0) and np.all(gpu["dW_out"][empty] == 0)

    # router weight gradients: zero dy outside the evaluated tokens, so that the
    # oracle's partial evaluation is exact, and run the GPU backward again
    dy_masked = inp["dy"] * torch.from_numpy(tmask).to(inp["dy"].device)[:, None].to(inp["dy"].dtype)
    g2 = layer.backward(dy_masked, inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], inp["b_r"], d_aux)
    torch.cuda.synchronize()
    dy_np = to_np(dy_masked)
    bwd2 = oracle.backward(npi["x"], npi["W_r"], npi["W_in"], npi["W_out"], dy_np, fwd,
                           shape.alpha, d_aux, expert_sel=sel, token_sel=toks, relu_flips=ties)
    wr_scale, br_scale = router_grad_scales(npi, fwd, y_ref, bwd2["dlogits"], dy=dy_np)
    errs["dW_r"] = assert_close("dW_r", to_np(g2["dW_r"]), bwd2["dW_r"], tol, scale=wr_scale)
    errs["db_r"] = assert_close("db_r", to_np(g2["db_r"]), bwd2["db_r"], tol, scale=br_scale)
    errs["a14"] = {"y": float("%.2e" % a14(gpu["y"][tmask], y_ref[tmask])),
                   "dx": float("%.2e" % a14(gpu["dx"][tmask], bwd["dx"][tmask])),
                   "dW_in": float("%.2e" % a14(gpu["dW_in"][sel], bwd["dW_in"])),
                   "dW_out": float("%.2e" % a14(gpu["dW_out"][sel], bwd["dW_out"])),
                   "dW_r": float("%.2e" % a14(to_np(g2["dW_r"]), bwd2["dW_r"]))}
    # tokens outside the mask now get only the router/aux part of dx, which the
    # oracle does evaluate for every token once their expert part is zero
    return errs
