"""MI355X-native forward pass of the gated-linear-attention token mixer of DiG.

The compute lives in hand-written HIP kernels behind the C ABI declared in
``include/gla.h`` (built into ``libgla.so`` next to ``csrc/``); this package
only marshals arguments.  Importing the package does not load the library;
calling any entry point without a built library raises.
"""
from .binding import (  # noqa: F401
    GlaError, gla_fwd, gla_fwd_static, gla_fwd_ex, gla_fwd_layout, gla_fwd_workspace_bytes, gla_fwd_timed, gla_calibrate_mfma,
    gla_bwd, gla_bwd_layout, gla_bwd_workspace_bytes, gla_bwd_gates, gla_bwd_gates_workspace_bytes, gla_fwd_fused, gla_fwd_fused_gates, gla_fwd_multi, gla_fwd_gates, gla_srem_dwconv,
    gla_set_option, gla_get_option, gla_status_string, gla_version, gla_block_scan_dir,
    SCHEDULE_BLOCK_PROCESS, SCHEDULE_BLOCK_SCAN,
    library_path, load_library, lib_symbols,
    SCAN_ROW_FWD, SCAN_ROW_REV, SCAN_COL_FWD, SCAN_COL_REV, DT_F32, DT_BF16,
    OPT_CHUNKS_PER_SPAN, OPT_ENGINE, OPT_CARRY, OPT_BWD_SPLIT, OPT_RANGE_FALLBACK, ENGINE_AUTO, ENGINE_RECURRENT, ENGINE_MFMA, ENGINE_MFMA_FP16,
    CARRY_AUTO, CARRY_KERNEL, CARRY_IN_OUTPUT_PASS, LAYOUT_BHTD, LAYOUT_BTHD,
)
