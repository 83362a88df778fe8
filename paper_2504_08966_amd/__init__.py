"""MI355X-native PACT token reduction: thin ctypes binding over libpact.so (HIP, gfx950).

The binding marshals arguments only; every step of the path runs in the library's
kernels.  PyTorch supplies device memory and the stream.
"""
from .binding import (  # noqa: F401
    PactParams, PACT_F32, PACT_BF16, PACT_FLAG_NO_MERGE, PACT_FLAG_SCORE_NO_NORM, PACT_FLAG_SCORE_NORM_ONLY, PACT_FLAG_KEY_STATS, REPORT_FIELDS, PactError,
    lib_path, load_library, pact_workspace_bytes, pact_score, pact_prune, dbdpc_cluster,
    pact_reincorporate, pact_merge, pact_reduce, pact_reduce_static, new_outputs, pact_reduce_varlen, pact_strerror,
    pact_attention_handoff, pact_calibration_copy, pact_plan_workgroups, pact_profile_enable, pact_profile_reset, pact_profile_read, read_report, new_report,
    alloc_workspace,
)
