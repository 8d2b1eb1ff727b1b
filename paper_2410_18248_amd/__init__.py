"""MI355X-native paged decode attention + KV swap under the LAMPS scheduler
(arXiv 2410.18248).  All compute is in ``liblamps.so`` (hand-written HIP for
gfx950 behind the C ABI of ``include/lamps.h``); this package only marshals
arguments.  Build the library with ``python -m paper_2410_18248_amd.build``.
"""
from .binding import (  # noqa: F401
    LAMPS_DISCARD, LAMPS_HANDLING_AUTO, LAMPS_POLICY_FCFS, LAMPS_POLICY_FIXED, LAMPS_POLICY_LAMPS, LAMPS_POLICY_SJF,
    LAMPS_POLICY_SJF_TOTAL, LAMPS_PRESERVE, LAMPS_SWAP, LampsCostModel, LampsSched, LampsSchedConfig,
    LAMPS_BF16, LAMPS_F32, LAMPS_LAYOUT_PLAIN, LAMPS_LAYOUT_TILED, Lamps, LampsConfig, LampsError, lib_path, load_library,
    lamps_block_bytes, lamps_decode_attn_static, lamps_kv_bytes_per_token, lamps_kv_layout, lamps_pool_bytes, lamps_workspace_bytes,
)
