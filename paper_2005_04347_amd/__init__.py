"""MI355X-native full activation of arbitrary-structure sparse neural networks.

The product is the C-ABI library ``libasnn.so`` (HIP, gfx950; headers in
``include/asnn.h``, sources in ``csrc/``).  This package is the thin ctypes
binding above it; build the library with ``python -m paper_2005_04347_amd.build``.
"""
from .binding import (  # noqa: F401
    AsnnError,
    BoundActivation,
    FLAG_ACC_F32,
    FLAG_DATAFLOW,
    FLAG_LEVEL_LAUNCHES,
    FLAG_RAW_INPUTS,
    FLAG_WORKGROUP,
    HEAVY_INDEGREE,
    MEDIUM_INDEGREE,
    Network,
    PackedGraph,
    STATIC_SCRATCH,
    STATIC_SCRATCH_BYTES,
    asnn_activate,
    asnn_activate_schedule,
    asnn_activate_static,
    asnn_activate_status,
    asnn_activate_workspace,
    asnn_build_levels,
    asnn_device_copy,
    asnn_device_gather,
    asnn_device_gather_store,
    asnn_device_read,
    asnn_compact_required,
    asnn_filter_required,
    asnn_relabel_ids,
    asnn_required_set,
    asnn_pack_csr,
    load,
)
