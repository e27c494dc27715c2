"""ctypes binding of libswitchffn.so -- marshalling only, no arithmetic."""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libswitchffn.so")

SW_F32, SW_BF16 = 0, 1
SW_FFN_RELU, SW_FFN_GEGLU = 0, 1
SW_FLAG_FUSED_DISPATCH = 1


class SwitchError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, switch_status_string(status), status))


class SwitchConfig(ctypes.Structure):
    """Mirror of the C struct switch_config."""
    _fields_ = [
        ("T", ctypes.c_int64),
        ("d_model", ctypes.c_int64),
        ("d_ff", ctypes.c_int64),
        ("E", ctypes.c_int64),
        ("capacity_factor", ctypes.c_double),
        ("alpha", ctypes.c_float),
        ("act_dtype", ctypes.c_int32),
        ("ffn_kind", ctypes.c_int32),
        ("n_groups", ctypes.c_int64),
        ("expert_dropout", ctypes.c_float),
        ("jitter_eps", ctypes.c_float),
        ("seed", ctypes.c_uint64),
        ("ntlb_rounds", ctypes.c_int32),
        ("flags", ctypes.c_int32),
    ]


def library_path() -> str:
    return _LIB_PATH


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        # nothing built yet: build in-tree once, then load; there is no fallback
        from . import build as _build
        _build.build(verbose=False)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, cfgp = ctypes.c_void_p, ctypes.POINTER(SwitchConfig)
    lib.switch_capacity.restype = ctypes.c_int
    lib.switch_capacity.argtypes = [cfgp, ctypes.POINTER(ctypes.c_int64)]
    lib.switch_workspace_size.restype = ctypes.c_int
    lib.switch_workspace_size.argtypes = [cfgp, ctypes.POINTER(ctypes.c_size_t)]
    lib.switch_forward.restype = ctypes.c_int
    lib.switch_forward.argtypes = [cfgp] + [vp] * 13 + [vp, ctypes.c_size_t, vp]
    lib.switch_forward_static.restype = ctypes.c_int
    lib.switch_forward_static.argtypes = [cfgp] + [vp] * 13 + [vp]
    lib.switch_backward.restype = ctypes.c_int
    lib.switch_backward.argtypes = [cfgp, vp, ctypes.c_float] + [vp] * 10 + [vp, ctypes.c_size_t, vp]
    lib.switch_status_string.restype = ctypes.c_char_p
    lib.switch_status_string.argtypes = [ctypes.c_int]
    lib.switch_profile_enable.restype = ctypes.c_int
    lib.switch_profile_enable.argtypes = [ctypes.c_int]
    lib.switch_profile_collect.restype = ctypes.c_int
    lib.switch_profile_collect.argtypes = []
    lib.switch_profile_count.restype = ctypes.c_int
    lib.switch_profile_count.argtypes = []
    lib.switch_profile_get.restype = ctypes.c_int
    lib.switch_profile_get.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_char_p),
                                       ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(ctypes.c_int64)]
    _lib = lib
    return lib


def _p(t) -> Optional[int]:
    """Device (or host) address of a tensor-like (anything with data_ptr()), an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def switch_status_string(status: int) -> str:
    return _load().switch_status_string(int(status)).decode()


def switch_capacity(cfg: SwitchConfig) -> int:
    out = ctypes.c_int64(0)
    st = _load().switch_capacity(ctypes.byref(cfg), ctypes.byref(out))
    if st != 0:
        raise SwitchError(st, "switch_capacity")
    return out.value


def switch_workspace_size(cfg: SwitchConfig) -> int:
    out = ctypes.c_size_t(0)
    st = _load().switch_workspace_size(ctypes.byref(cfg), ctypes.byref(out))
    if st != 0:
        raise SwitchError(st, "switch_workspace_size")
    return out.value


def switch_forward(cfg: SwitchConfig, x, W_r, b_r, W_in, W_out, y, expert_index, gate,
                   position_in_expert, dropped, expert_counts, aux_loss, router_logits,
                   workspace, workspace_bytes: int, hip_stream: int = 0, check: bool = True) -> int:
    st = _load().switch_forward(ctypes.byref(cfg), _p(x), _p(W_r), _p(b_r), _p(W_in), _p(W_out),
                                _p(y), _p(expert_index), _p(gate), _p(position_in_expert),
                                _p(dropped), _p(expert_counts), _p(aux_loss), _p(router_logits),
                                _p(workspace), int(workspace_bytes), hip_stream or None)
    if check and st != 0:
        raise SwitchError(st, "switch_forward")
    return st


SW_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024   # include/switchffn.h


def switch_forward_static(cfg: SwitchConfig, x, W_r, b_r, W_in, W_out, y, expert_index, gate,
                          position_in_expert, dropped, expert_counts, aux_loss, router_logits,
                          hip_stream: int = 0, check: bool = True) -> int:
    """switch_forward on the library's own fixed scratch array: no workspace argument."""
    st = _load().switch_forward_static(ctypes.byref(cfg), _p(x), _p(W_r), _p(b_r), _p(W_in),
                                       _p(W_out), _p(y), _p(expert_index), _p(gate),
                                       _p(position_in_expert), _p(dropped), _p(expert_counts),
                                       _p(aux_loss), _p(router_logits), hip_stream or None)
    if check and st != 0:
        raise SwitchError(st, "switch_forward_static")
    return st


def switch_backward(cfg: SwitchConfig, dy, d_aux: float, x, W_r, b_r, W_in, W_out, dx, dW_r, db_r,
                    dW_in, dW_out, workspace, workspace_bytes: int, hip_stream: int = 0,
                    check: bool = True) -> int:
    st = _load().switch_backward(ctypes.byref(cfg), _p(dy), float(d_aux), _p(x), _p(W_r), _p(b_r),
                                 _p(W_in), _p(W_out), _p(dx), _p(dW_r), _p(db_r), _p(dW_in),
                                 _p(dW_out), _p(workspace), int(workspace_bytes),
                                 hip_stream or None)
    if check and st != 0:
        raise SwitchError(st, "switch_backward")
    return st


def switch_profile_enable(on: bool) -> None:
    st = _load().switch_profile_enable(1 if on else 0)
    if st != 0:
        raise SwitchError(st, "switch_profile_enable")


def switch_profile_collect() -> None:
    st = _load().switch_profile_collect()
    if st != 0:
        raise SwitchError(st, "switch_profile_collect")


def switch_profile_read() -> Dict[str, Tuple[float, int]]:
    """{kernel name: (total milliseconds, launches)} accumulated since enable."""
    lib = _load()
    out: Dict[str, Tuple[float, int]] = {}
    for i in range(lib.switch_profile_count()):
        name = ctypes.c_char_p()
        ms = ctypes.c_double()
        n = ctypes.c_int64()
        st = lib.switch_profile_get(i, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(n))
        if st != 0:
            raise SwitchError(st, "switch_profile_get")
        out[name.value.decode()] = (ms.value, n.value)
    return out
