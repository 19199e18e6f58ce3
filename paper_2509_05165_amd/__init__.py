"""MI355X-native KVCompose compression pass: thin ctypes binding over libkvc.so.

The binding only marshals arguments; every step of the pass runs in the HIP
kernels of the C-ABI library declared in include/kvc.h.
"""
from .binding import (  # noqa: F401
    KVC_F32, KVC_BF16, KVC_AGG_MAX, KVC_AGG_MEAN, KVC_ORDER_RANK, KVC_ORDER_POSITION, KvcError, KvcParams, lib, lib_path,
    kvc_version, kvc_status_string, kvc_last_error, kvc_budget, kvc_workspace_size,
    kvc_score, kvc_head_rank, kvc_composite, kvc_global_select, kvc_global_select_static,
    kvc_gather, kvc_compress,
    kvc_profile_enable, kvc_profile_collect, kvc_copy_probe, kvc_mfma_probe,
    KVC_MFMA_PROBE_OPERAND_BYTES, KVC_MFMA_PROBE_SINK_FLOATS,
)
