"""Event-tensor decode megakernel for AMD MI355X: thin Python binding of the C ABI (include/etc.h).

Argument marshalling only.  Every step of the decode path runs in the HIP library
``libetc.so``; there is no Python or CPU fallback: a missing library raises.
"""
from .binding import (  # noqa: F401
    DEBUG_EXEC_COUNT, DEBUG_LAYER_HIDDEN, DEBUG_ROUTING, DEBUG_TRACE, SCHED_DYNAMIC, SCHED_STATIC, SCHED_UNFUSED,
    Decoder, EtcError, EventGraph, MoeLayer, ROWSUM_NOALLOC_MAX_N, lib, lib_path, moe_layer_plan_build, plan_build,
    rowsum_launch_noalloc,
)
