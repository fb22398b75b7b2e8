"""MI355X-native hierarchical block LDL^T log-determinant (thin Python binding).

Every step of the path runs inside ``libmemdet.so`` (hand-written HIP for
gfx950); this package only marshals arguments.  PyTorch tensors are used as
device / pinned-host memory and for the current stream handle.
"""
from .binding import (  # noqa: F401
    MDET_F32, MDET_F64, MDET_F16, MDET_BF16, FLAG_NO_LOOKAHEAD, FLAG_FORCE_OUT_OF_CORE, FLAG_PROFILE, FLAG_COMPUTE_F64, FLAG_ASSUME_SPD, FLAG_SCALED_COPY, FLAG_PIVOT, FLAG_GENERAL, FLAG_PIVOT_BLOCK,
    MemdetError, LogdetResult, PlanInfo, Status,
    lib, lib_path, load,
    mdet_plan, mdet_workspace_query, mdet_logdet_device, mdet_logdet_host,
    mdet_logdet_provider, mdet_logdet_provider_device, mdet_logdet_file, mdet_host_layout_offset, mdet_paper_block_rule,
    mdet_paper_fma_count, mdet_step_schur_update, mdet_step_panel_factor, mdet_step_panel_factor_pivoted, mdet_step_panel_factor_general,
    mdet_step_logdet_reduce, mdet_strerror, mdet_version,
    mdet_sequence_workspace_query, mdet_principal_logdets, mdet_flodance_fit, mdet_flodance_eval,
    mdet_step_copy, mdet_step_mfma_peak, mdet_logdet_device_noalloc,
    pack_lower_block_columns, pack_general_block_columns,
)
from .api import memdet, parse_bytes, FitLogdet  # noqa: E402,F401
