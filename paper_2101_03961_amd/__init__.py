"""MI355X-native Switch FFN layer (arXiv 2101.03961): Python binding of the C ABI.

The functions here have the names and argument order of ``include/switchffn.h``
and do argument marshalling only; every step of the layer runs in the HIP
kernels of ``libswitchffn.so``.  There is no CPU or PyTorch fallback: if the
library is missing or cannot be loaded, importing the binding raises.
"""
from .binding import (  # noqa: F401
    SW_BF16,
    SW_F32,
    SW_FFN_GEGLU,
    SW_FFN_RELU,
    SW_FLAG_FUSED_DISPATCH,
    SwitchConfig,
    SwitchError,
    library_path,
    switch_backward,
    switch_capacity,
    SW_STATIC_SCRATCH_BYTES,
    switch_forward,
    switch_forward_static,
    switch_profile_collect,
    switch_profile_enable,
    switch_profile_read,
    switch_status_string,
    switch_workspace_size,
)
