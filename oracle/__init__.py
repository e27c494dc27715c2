"""CPU oracle for the Switch FFN layer -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front end over ``switch_oracle.c`` (plain fp64 C, written from the
paper) plus ``dense_onehot.py`` (the paper's dense dispatch/combine-tensor
formulation in numpy, for tiny inputs).  Only the tests, the smoke check and
the benchmark's ``cpu_baseline`` leg may import this package; the GPU library
never does, and nothing here imports the GPU library.

Tensors go in as numpy float32 arrays holding the exact values given to the
GPU (bf16 widens to float32 without rounding); all arithmetic is fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "switch_oracle.c")
_LIB = os.path.join(_HERE, "libswitch_oracle.so")
_LIB_F64IN = os.path.join(_HERE, "libswitch_oracle_f64in.so")

# Storage dtype of the tensors handed to C.  float32 holds every bf16 / fp32
# value exactly and is what parity tests use.  The finite-difference tests switch
# to float64 storage (second build of the same C file) so that inputs can be
# perturbed by 1e-6; see use_f64_inputs().
_in_dtype = np.float32

_c_f32p = ctypes.c_void_p


class Noise(ctypes.Structure):
    """Training-time noise (mirror of swo_noise): expert dropout rate, jitter eps, seed."""
    _fields_ = [("expert_dropout", ctypes.c_float), ("jitter_eps", ctypes.c_float),
                ("seed", ctypes.c_uint64)]


def _noise(noise):
    """None, or a (expert_dropout, jitter_eps, seed) triple -> pointer argument."""
    if noise is None:
        return None
    rate, eps, seed = noise
    if rate == 0 and eps == 0:
        return None
    return ctypes.byref(Noise(float(rate), float(eps), int(seed)))

_c_f64p = ctypes.POINTER(ctypes.c_double)
_c_i32p = ctypes.POINTER(ctypes.c_int32)
_c_i64p = ctypes.POINTER(ctypes.c_int64)
_c_u8p = ctypes.POINTER(ctypes.c_uint8)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math: fp64 semantics stay IEEE)."""
    for lib, extra in ((_LIB, []), (_LIB_F64IN, ["-DSWO_IN_T=double"])):
        stale = (not os.path.exists(lib)) or os.path.getmtime(lib) < os.path.getmtime(_SRC)
        if force or stale:
            cmd = ["gcc", "-O3", "-fopenmp", "-fno-fast-math", "-std=c11", "-shared", "-fPIC",
                   *extra, "-o", lib, _SRC, "-lm"]
            subprocess.run(cmd, check=True)
    return _LIB


_libs = {}


def use_f64_inputs(on: bool) -> None:
    """Switch the storage dtype of tensors handed to C (float32 <-> float64)."""
    global _in_dtype
    _in_dtype = np.float64 if on else np.float32


def _load():
    key = np.dtype(_in_dtype).name
    if key in _libs:
        return _libs[key]
    build()
    lib = ctypes.CDLL(_LIB if _in_dtype is np.float32 else _LIB_F64IN)
    i64, f64 = ctypes.c_int64, ctypes.c_double
    lib.swo_capacity.restype = i64
    lib.swo_capacity.argtypes = [i64, i64, f64]
    lib.swo_logits.restype = None
    noise_p = ctypes.POINTER(Noise)
    lib.swo_logits.argtypes = [i64, i64, i64, _c_f32p, _c_f32p, _c_f32p, noise_p, _c_f64p]
    lib.swo_mix.restype = ctypes.c_uint32
    lib.swo_mix.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint64]
    lib.swo_jitter_mult.restype = f64
    lib.swo_jitter_mult.argtypes = [noise_p, i64, i64, i64]
    lib.swo_dropout_factor.restype = f64
    lib.swo_dropout_factor.argtypes = [noise_p, i64, i64, i64]
    lib.swo_softmax.restype = None
    lib.swo_softmax.argtypes = [i64, i64, _c_f64p, _c_f64p]
    lib.swo_top1.restype = None
    lib.swo_top1.argtypes = [i64, i64, _c_f64p, _c_f64p, _c_i32p, _c_f64p]
    lib.swo_aux_loss.restype = f64
    lib.swo_aux_loss.argtypes = [i64, i64, i64, _c_i32p, _c_f64p, f64, _c_i64p, _c_i64p, _c_f64p,
                                 _c_f64p]
    lib.swo_positions.restype = None
    lib.swo_positions.argtypes = [i64, i64, i64, i64, _c_i32p, _c_i32p, _c_u8p, _c_i64p]
    lib.swo_ntlb.restype = None
    lib.swo_ntlb.argtypes = [i64, i64, i64, i64, i64, _c_f64p, _c_i32p, _c_i32p, _c_i32p, _c_u8p,
                             _c_i64p, _c_i32p]
    lib.swo_expert_ffn.restype = None
    lib.swo_expert_ffn.argtypes = [i64, i64, i64, i64, _c_f32p, _c_f32p, _c_f32p, _c_i32p,
                                   _c_u8p, _c_f64p, _c_u8p, noise_p, i64, _c_f64p]
    lib.swo_backward.restype = None
    lib.swo_backward.argtypes = [i64, i64, i64, i64, _c_f32p, _c_f32p, _c_f32p, _c_f32p,
                                 _c_f32p, f64, f64, _c_i32p, _c_u8p, _c_f64p, _c_f64p, i64, _c_i64p,
                                 _c_i32p, _c_u8p, i64, _c_i64p, _c_i64p, noise_p, i64, _c_f64p,
                                 _c_f64p, _c_f64p, _c_f64p, _c_f64p, _c_f64p, _c_f64p]
    lib.swo_hidden_near_zero.restype = i64
    lib.swo_hidden_near_zero.argtypes = [i64, i64, i64, _c_f32p, _c_f32p, _c_i32p, _c_u8p, _c_u8p,
                                         f64, i64, _c_i64p, _c_i64p, _c_f64p]
    _libs[key] = lib
    return lib


def _f32(a) -> np.ndarray:
    """Contiguous array in the current input storage dtype (float32 by default)."""
    return np.ascontiguousarray(a, dtype=_in_dtype)


def _ptr(a: Optional[np.ndarray], ctype):
    if a is None:
        return None
    if ctype is ctypes.c_void_p:
        return ctypes.c_void_p(a.ctypes.data)
    return a.ctypes.data_as(ctype)


def set_threads(n: int) -> None:
    """Cap the OpenMP thread count used by the C oracle."""
    os.environ["OMP_NUM_THREADS"] = str(n)
    try:
        omp = ctypes.CDLL("libgomp.so.1")
        omp.omp_set_num_threads(int(n))
    except OSError:
        pass


def max_threads() -> int:
    try:
        omp = ctypes.CDLL("libgomp.so.1")
        return int(omp.omp_get_max_threads())
    except OSError:
        return 1


# --------------------------------------------------------------------------
# step-level wrappers (one per oracle step)
# --------------------------------------------------------------------------
def capacity(T: int, E: int, capacity_factor: float, n_groups: int = 1) -> int:
    """Eq. 3 with floor rounding, for the tokens of one routing group."""
    assert n_groups >= 1 and T % n_groups == 0
    return int(_load().swo_capacity(T // n_groups, E, float(capacity_factor)))


def logits(x, W_r, b_r=None, noise=None) -> np.ndarray:
    """h = x W_r (+ b_r), fp64 (Sec. 2.1); with noise = (dropout, eps, seed) the router sees the
    jittered x (App. C)."""
    x, W_r = _f32(x), _f32(W_r)
    T, d = x.shape
    E = W_r.shape[1]
    assert W_r.shape[0] == d
    b = None if b_r is None else _f32(b_r)
    h = np.empty((T, E), dtype=np.float64)
    _load().swo_logits(T, d, E, _ptr(x, _c_f32p), _ptr(W_r, _c_f32p), _ptr(b, _c_f32p), _noise(noise),
                       _ptr(h, _c_f64p))
    return h


def softmax(h) -> np.ndarray:
    """Eq. 1."""
    h = np.ascontiguousarray(h, dtype=np.float64)
    p = np.empty_like(h)
    _load().swo_softmax(h.shape[0], h.shape[1], _ptr(h, _c_f64p), _ptr(p, _c_f64p))
    return p


def top1(h, p):
    """Expert index (arg max, lowest index on ties) and its gate value."""
    h = np.ascontiguousarray(h, dtype=np.float64)
    p = np.ascontiguousarray(p, dtype=np.float64)
    T, E = h.shape
    e = np.empty(T, dtype=np.int32)
    g = np.empty(T, dtype=np.float64)
    _load().swo_top1(T, E, _ptr(h, _c_f64p), _ptr(p, _c_f64p), _ptr(e, _c_i32p), _ptr(g, _c_f64p))
    return e, g


def aux_loss(expert_index, p, alpha: float, n_groups: int = 1, with_group_counts: bool = False):
    """Eqs. 4-6, averaged over the routing groups.  Returns (loss, counts[E], f, P) with f and
    P of shape [E] for one group and [n_groups][E] otherwise (+ counts per group if asked)."""
    e = np.ascontiguousarray(expert_index, dtype=np.int32)
    p = np.ascontiguousarray(p, dtype=np.float64)
    T, E = p.shape
    assert n_groups >= 1 and T % n_groups == 0
    counts = np.empty(E, dtype=np.int64)
    counts_g = np.empty((n_groups, E), dtype=np.int64)
    f = np.empty((n_groups, E), dtype=np.float64)
    P = np.empty((n_groups, E), dtype=np.float64)
    loss = _load().swo_aux_loss(T, E, n_groups, _ptr(e, _c_i32p), _ptr(p, _c_f64p), float(alpha),
                                _ptr(counts, _c_i64p), _ptr(counts_g, _c_i64p),
                                _ptr(f, _c_f64p), _ptr(P, _c_f64p))
    if n_groups == 1:
        f, P = f[0], P[0]
    if with_group_counts:
        return float(loss), counts, f, P, counts_g
    return float(loss), counts, f, P


def positions(expert_index, E: int, C: int, n_groups: int = 1):
    """Sequence-order rank within the chosen expert (inside the token's group), dropped mask,
    kept counts ([E], or [n_groups][E] for several groups).  C: per-group capacity."""
    e = np.ascontiguousarray(expert_index, dtype=np.int32)
    T = e.shape[0]
    assert n_groups >= 1 and T % n_groups == 0
    pos = np.empty(T, dtype=np.int32)
    dropped = np.empty(T, dtype=np.uint8)
    kept = np.empty((n_groups, E), dtype=np.int64)
    _load().swo_positions(T, E, C, n_groups, _ptr(e, _c_i32p), _ptr(pos, _c_i32p),
                          _ptr(dropped, _c_u8p), _ptr(kept, _c_i64p))
    return pos, dropped, (kept[0] if n_groups == 1 else kept)


def ntlb(h, expert_index, pos, dropped, kept, C: int, n_groups: int, rounds: int,
         choices_override=None):
    """No-Token-Left-Behind stages after the Switch routing (App. B): returns updated copies
    (expert_index, position_in_expert, dropped, kept) and the experts asked for, [T][rounds]."""
    h = np.ascontiguousarray(h, dtype=np.float64)
    T, E = h.shape
    e = np.array(expert_index, dtype=np.int32)
    pos = np.array(pos, dtype=np.int32)
    dropped = np.array(dropped, dtype=np.uint8)
    kept = np.array(kept, dtype=np.int64).reshape(n_groups, E)
    choices = np.empty((T, rounds), dtype=np.int32)
    ov = None
    if choices_override is not None:
        ov = np.ascontiguousarray(choices_override, dtype=np.int32)
        assert ov.shape == (T, rounds)
    _load().swo_ntlb(T, E, C, n_groups, rounds, _ptr(h, _c_f64p), _ptr(ov, _c_i32p),
                     _ptr(e, _c_i32p), _ptr(pos, _c_i32p), _ptr(dropped, _c_u8p),
                     _ptr(kept, _c_i64p), _ptr(choices, _c_i32p))
    return e, pos, dropped, (kept[0] if n_groups == 1 else kept), choices


def _token_mask(expert_index, E, expert_sel, token_sel):
    """uint8[T] mask of the tokens to evaluate, or None for all of them."""
    if expert_sel is None and token_sel is None:
        return None
    e = np.asarray(expert_index)
    mask = np.zeros(e.shape[0], dtype=np.uint8)
    if expert_sel is not None:
        mask[np.isin(e, np.asarray(list(expert_sel), dtype=e.dtype))] = 1
    if token_sel is not None:
        mask[np.asarray(list(token_sel), dtype=np.int64)] = 1
    return mask


FFN_KINDS = {"relu": 0, "geglu": 1}


def _ffn_dims(W_in, W_out, ffn: str):
    """(E, d, f) from the weight shapes: W_in is [E, d, f] (relu) or [E, d, 2 f] (geglu: gate
    columns, then linear columns), W_out is [E, f, d]."""
    E, d, f1 = W_in.shape
    f = f1 // 2 if ffn == "geglu" else f1
    assert ffn in FFN_KINDS and W_out.shape == (E, f, d) and f1 == (2 * f if ffn == "geglu" else f)
    return E, d, f


def expert_ffn(x, W_in, W_out, expert_index, dropped, gate, expert_sel=None,
               token_sel=None, noise=None, ffn: str = "relu") -> np.ndarray:
    """y_t = gate_t * FFN_{e_t}(x_t) for kept tokens, 0 for dropped; FFN = ReLU(x W_in) W_out,
    or with ffn = "geglu" (GELU(x W_g) * (x W_l)) W_out, W_in = [W_g | W_l].

    With expert_sel / token_sel only tokens of those experts / those tokens are
    evaluated; all other rows are NaN."""
    x, W_in, W_out = _f32(x), _f32(W_in), _f32(W_out)
    T, d = x.shape
    E, d2, f = _ffn_dims(W_in, W_out, ffn)
    assert d2 == d
    e = np.ascontiguousarray(expert_index, dtype=np.int32)
    dr = np.ascontiguousarray(dropped, dtype=np.uint8)
    g = np.ascontiguousarray(gate, dtype=np.float64)
    sel = _token_mask(e, E, expert_sel, token_sel)
    y = np.empty((T, d), dtype=np.float64)
    _load().swo_expert_ffn(T, d, f, E, _ptr(x, _c_f32p), _ptr(W_in, _c_f32p), _ptr(W_out, _c_f32p),
                           _ptr(e, _c_i32p), _ptr(dr, _c_u8p), _ptr(g, _c_f64p),
                           _ptr(sel, _c_u8p), _noise(noise), FFN_KINDS[ffn], _ptr(y, _c_f64p))
    return y


# --------------------------------------------------------------------------
# whole layer
# --------------------------------------------------------------------------
def forward(x, W_r, W_in, W_out, capacity_factor: float, alpha: float, b_r=None,
            logits_override=None, expert_index_override=None,
            expert_sel: Optional[Sequence[int]] = None,
            token_sel: Optional[Sequence[int]] = None, skip_ffn: bool = False,
            n_groups: int = 1, noise=None, ffn: str = "relu", ntlb_rounds: int = 0,
            ntlb_choices_override=None) -> Dict:
    """Whole forward pass.

    n_groups: routing groups of T / n_groups consecutive tokens (capacity, positions and the
        auxiliary loss per group; 1 = the whole batch is one group).
    noise: None or (expert_dropout, jitter_eps, seed): training-time noise.
    ffn: "relu" or "geglu" (see expert_ffn).
    ntlb_rounds: No-Token-Left-Behind re-routing stages after the Switch routing (App. B).
        Then expert_index / gate / position_in_expert describe the expert that processes the
        token (for tokens without a slot: the arg max, its probability and raw rank),
        first_choice is the arg max, and expert_counts / the loss keep counting arg max
        decisions.  ntlb_choices_override ([T][rounds]) forces what each token asks for.
    logits_override: use these logits (e.g. another implementation's fp32
        logits, widened) instead of computing them -- for the routing-stage
        comparison, which is defined on identical logits.
    expert_index_override: keep this module's probabilities but force the
        routing decision (used when a near-tie arg max legitimately differs,
        so that one flipped token does not shift every later position).
    expert_sel / token_sel: evaluate the expert FFN only for the tokens of
        these experts plus these tokens (other rows of y are NaN).
    """
    x32 = _f32(x)
    T, d = x32.shape
    E = np.asarray(W_r).shape[1]
    C = capacity(T, E, capacity_factor, n_groups)
    if logits_override is None:
        h = logits(x32, W_r, b_r, noise)
    else:
        h = np.ascontiguousarray(logits_override, dtype=np.float64)
    p = softmax(h)
    e, g = top1(h, p)
    if expert_index_override is not None:
        e = np.ascontiguousarray(expert_index_override, dtype=np.int32)
        g = p[np.arange(T), e].copy()
    loss, counts, f_vec, P_vec, counts_g = aux_loss(e, p, alpha, n_groups, with_group_counts=True)
    pos, dropped, kept = positions(e, E, C, n_groups)
    first_choice, choices = e, None
    if ntlb_rounds > 0:
        e, pos, dropped, kept, choices = ntlb(h, e, pos, dropped, kept, C, n_groups, ntlb_rounds,
                                              ntlb_choices_override)
        g = p[np.arange(T), e].copy()
    out = dict(capacity=C, logits=h, probs=p, expert_index=e, gate=g, aux_loss=loss,
               expert_counts=counts, f=f_vec, P=P_vec, position_in_expert=pos,
               dropped=dropped, kept_counts=kept, n_groups=n_groups, group_counts=counts_g,
               noise=noise, ffn=ffn, first_choice=first_choice, ntlb_choices=choices)
    if not skip_ffn:
        out["y"] = expert_ffn(x32, W_in, W_out, e, dropped, g, expert_sel, token_sel, noise, ffn)
    return out


def mix(idx: int, stream: int, seed: int) -> int:
    """The oracle's counter-based generator: 32 random bits for element idx of a stream."""
    return int(_load().swo_mix(idx & 0xFFFFFFFF, stream, seed & 0xFFFFFFFFFFFFFFFF))


def jitter_mult(noise, t: int, d: int, k: int) -> float:
    return float(_load().swo_jitter_mult(_noise(noise), t, d, k))


def dropout_factor(noise, t: int, f: int, j: int) -> float:
    return float(_load().swo_dropout_factor(_noise(noise), t, f, j))


def hidden_near_zero(x, W_in, expert_index, dropped, rel_eps: float, expert_sel=None,
                     token_sel=None, max_out: int = 4096):
    """(t, j, h) for the evaluated kept tokens' hidden units with |h| <= rel_eps * RMS(h_t):
    pre-activations that are zero to fp32 rounding, where the ReLU decision is not unique."""
    x32, W_in32 = _f32(x), _f32(W_in)
    T, d = x32.shape
    E, _, f = W_in32.shape
    e = np.ascontiguousarray(expert_index, dtype=np.int32)
    dr = np.ascontiguousarray(dropped, dtype=np.uint8)
    sel = _token_mask(e, E, expert_sel, token_sel)
    ot = np.empty(max_out, dtype=np.int64)
    oj = np.empty(max_out, dtype=np.int64)
    oh = np.empty(max_out, dtype=np.float64)
    n = _load().swo_hidden_near_zero(T, d, f, _ptr(x32, _c_f32p), _ptr(W_in32, _c_f32p),
                                     _ptr(e, _c_i32p), _ptr(dr, _c_u8p), _ptr(sel, _c_u8p),
                                     float(rel_eps), max_out, _ptr(ot, _c_i64p),
                                     _ptr(oj, _c_i64p), _ptr(oh, _c_f64p))
    assert n <= max_out, "too many near-zero hidden units (%d)" % n
    return sorted((int(ot[i]), int(oj[i]), float(oh[i])) for i in range(n))


def backward(x, W_r, W_in, W_out, dy, fwd: Dict, alpha: float, d_aux: float = 1.0,
             expert_sel: Optional[Sequence[int]] = None,
             token_sel: Optional[Sequence[int]] = None,
             relu_flips: Optional[Sequence] = None) -> Dict:
    """Whole backward pass for L = sum <dy, y> + d_aux * aux_loss.

    With expert_sel (and optionally token_sel, extra single tokens), weight
    gradients are returned only for the experts of expert_sel (stacked in the
    given order); dx rows of unselected tokens are NaN and their gate gradient is
    taken as 0 in dW_r / db_r (exact only if dy is zero on those tokens).
    relu_flips: (token, hidden unit) pairs whose ReLU gate 1[h > 0] is inverted.
    """
    x32, W_r32, W_in32, W_out32, dy32 = _f32(x), _f32(W_r), _f32(W_in), _f32(W_out), _f32(dy)
    T, d = x32.shape
    ffn = fwd.get("ffn", "relu")
    E, _, f = _ffn_dims(W_in32, W_out32, ffn)
    f1 = W_in32.shape[2]
    e = np.ascontiguousarray(fwd["expert_index"], dtype=np.int32)
    dr = np.ascontiguousarray(fwd["dropped"], dtype=np.uint8)
    g = np.ascontiguousarray(fwd["gate"], dtype=np.float64)
    p = np.ascontiguousarray(fwd["probs"], dtype=np.float64)
    n_groups = int(fwd.get("n_groups", 1))
    if "group_counts" in fwd:
        counts_g = np.ascontiguousarray(fwd["group_counts"], dtype=np.int64)
    else:
        counts_g = np.ascontiguousarray(fwd["expert_counts"], dtype=np.int64).reshape(1, -1)
    assert counts_g.shape == (n_groups, E)
    tmask = _token_mask(e, E, expert_sel, token_sel)
    if expert_sel is None and token_sel is not None:
        expert_sel = []
    if expert_sel is None:
        sel_slot = None
        nsel = E
    else:
        expert_sel = list(expert_sel)
        sel_slot = np.full(E, -1, dtype=np.int32)
        for s, ex in enumerate(expert_sel):
            sel_slot[ex] = s
        nsel = len(expert_sel)
    flips = list(relu_flips or [])
    flip_t = np.ascontiguousarray([p[0] for p in flips], dtype=np.int64)
    flip_j = np.ascontiguousarray([p[1] for p in flips], dtype=np.int64)
    dx = np.empty((T, d), dtype=np.float64)
    dW_r = np.empty((d, E), dtype=np.float64)
    db_r = np.empty(E, dtype=np.float64)
    dW_in = np.empty((nsel, d, f1), dtype=np.float64)
    dW_out = np.empty((nsel, f, d), dtype=np.float64)
    dgate = np.empty(T, dtype=np.float64)
    dlog = np.empty((T, E), dtype=np.float64)
    _load().swo_backward(T, d, f, E, _ptr(x32, _c_f32p), _ptr(W_r32, _c_f32p),
                         _ptr(W_in32, _c_f32p), _ptr(W_out32, _c_f32p), _ptr(dy32, _c_f32p),
                         float(d_aux), float(alpha), _ptr(e, _c_i32p), _ptr(dr, _c_u8p),
                         _ptr(g, _c_f64p), _ptr(p, _c_f64p), n_groups, _ptr(counts_g, _c_i64p),
                         _ptr(sel_slot, _c_i32p), _ptr(tmask, _c_u8p), len(flips),
                         _ptr(flip_t, _c_i64p), _ptr(flip_j, _c_i64p), _noise(fwd.get("noise")),
                         FFN_KINDS[ffn], _ptr(dx, _c_f64p), _ptr(dW_r, _c_f64p),
                         _ptr(db_r, _c_f64p), _ptr(dW_in, _c_f64p), _ptr(dW_out, _c_f64p),
                         _ptr(dgate, _c_f64p), _ptr(dlog, _c_f64p))
    return dict(dx=dx, dW_r=dW_r, db_r=db_r, dW_in=dW_in, dW_out=dW_out, dgate=dgate,
                dlogits=dlog)
