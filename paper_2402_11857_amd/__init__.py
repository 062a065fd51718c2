"""MI355X-native LIEC-SGD compressed step: thin Python binding over the C-ABI HIP library.

The binding marshals arguments only; every step of the method runs in the HIP
kernels of ``libliec.so``.  There is no CPU fallback: if the library is missing
the first use raises.
"""
from .binding import (  # noqa: F401
    COMP_IDENTITY,
    COMP_SIGN,
    COMP_TOPK,
    COMP_BLOCKSIGN,
    COMP_RANDK,
    LiecContext,
    LiecError,
    LiecInfo,
    device_copy,
    lib,
    library_path,
    liec_create,
    liec_create_ex,
    liec_destroy,
    liec_get_info,
    liec_get_worker_desc,
    liec_l2_norm_static,
    liec_set_lr,
    liec_set_random,
    liec_get_random,
    liec_message_bytes,
    liec_comm_cost,
    liec_set_blocks,
    liec_get_block_scales,
    liec_step,
    liec_step_sync,
)
