"""MI355X-native context-switch swap (bidirectional evict/restore through a bounded pinned ring).

The work is done by ``libnixie.so`` (hand-written HIP for gfx950 behind a C ABI, declared in
``include/nixie.h``); this package only marshals arguments.  There is no CPU fallback: if the
library has not been built, loading it raises.
"""
from .nixie import (  # noqa: F401
    NixieError, Opts, Plan, Ring, Layout, Sched, Pool, Space, tier_register, tier_unregister, host_copy, place, TIER_GPU, TIER_PINNED, TIER_PAGEABLE, lib, lib_path, link_peak, hash_buffers, hash_buffers_noalloc, strerror,
    ORDER_TABLE, ORDER_LARGE_FIRST, ORDER_ADDRESS, ORDER_REVERSE,
    SPLIT_BY_BYTES, SERIALIZE, DIAG_RING_ONLY, DIAG_STALL_DRAIN, HOST_PLAIN_MEMCPY, IN_PLACE, NO_DIRECT, HOST_SPIN, NO_FLEX_WGS,
    EINVAL, EOVERLAP, ENOMEM, EHIP, ETIMEOUT, EMISMATCH, EBUSY, EUNMAPPED, DECLARED_SYMBOLS,
)
