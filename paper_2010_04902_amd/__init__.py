"""ByzShield parameter-server aggregation (majority vote + coordinate-wise median) on MI355X.

Thin Python binding over the C-ABI of libbyzshield.so; every step of the path runs in the
library's HIP kernels / host code.  PyTorch is used for device memory and streams only.
"""
from .binding import (  # noqa: F401
    BYZ_AGG_EARLY_MAJORITY,
    BYZ_AGG_TRIM,
    BYZ_AGG_TRIMMED_MEAN,
    BYZ_SCHEME_FRC,
    BYZ_SCHEME_MOLS,
    BYZ_SCHEME_RAMANUJAN,
    BYZ_MAX_F,
    BYZ_MAX_F_WIDE,
    Assignment,
    ByzError,
    byz_aggregate,
    byz_aggregate_has_single_pass,
    byz_aggregate_opts,
    byz_aggregate_took_exact_path,
    byz_aggregate_workspace_bytes,
    byz_build_assignment,
    byz_bulyan,
    byz_bulyan_workspace_bytes,
    byz_calibration_copy,
    byz_gamma_bound,
    byz_median,
    byz_multi_krum,
    byz_multi_krum_workspace_bytes,
    byz_profile_collect,
    byz_profile_enable,
    byz_strerror,
    byz_trimmed_mean,
    byz_vote,
    byz_vote_tolerant,
    byz_worst_case,
    library_path,
)
