"""SP-KV decode path for AMD MI355X: ctypes binding over the C-ABI library libspkv.so.

Importing the package loads nothing; the library is loaded on first use and a missing
library is an error (there is no fallback path).  Build it with
`python -m paper_2605_14037_amd.build` or `__graft_entry__.build()`.
"""

from .binding import (  # noqa: F401
    SPKVCache, SPKVConfig, SPKVStats, SPKVError, load_library, library_path,
    required_bytes, strerror, layout_offset, debug_copy, debug_read, utility_logits, soft_gated_attention,
    EXPORTED_SYMBOLS,
    OPT_ITEM_TARGET, OPT_KERNEL_TIMING, OPT_SPLIT_ONLY, OPT_SINK_TOKENS, OPT_MERGE_WAVES, OPT_STEP_LAUNCHES,
)
