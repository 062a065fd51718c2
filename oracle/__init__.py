"""CPU oracle for the LIEC-SGD compressed step.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the bench's CPU-baseline leg may import
this package; the product (``paper_2402_11857_amd``) never does.
"""
from .liec_oracle import (  # noqa: F401
    IDENTITY,
    SIGN,
    TOPK,
    BLOCKSIGN,
    RANDK,
    Desc,
    build,
    build_all_cores,
    step_all_cores,
    compress,
    compress_blocksign,
    error_update,
    pack_sign,
    pack_topk,
    pack_randk,
    randk_priorities,
    unpack_topk,
    unpack_sign,
    server_average,
    step,
    step_blocks,
    step_sync,
    worker_update,
)
