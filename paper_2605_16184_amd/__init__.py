"""MI355X-native Shampoo / SOAP preconditioner pipeline (thin Python binding over the C ABI in
``include/asteria.h``).  Every step of the path runs in the HIP library; this package only
marshals arguments.  PyTorch is used for device memory and streams.
"""
from .binding import (  # noqa: F401
    AsteriaError,
    RootOpts,
    lib,
    library_path,
    stats_update,
    inverse_root,
    inverse_root_plan,
    inverse_root_static,
    static_scratch_bytes,
    precondition,
    soap_refresh,
    soap_step,
    stats_update_workspace_bytes,
    inverse_root_workspace_bytes,
    precondition_workspace_bytes,
    soap_refresh_workspace_bytes,
    soap_step_workspace_bytes,
    status_string,
    version,
    Blocks,
    Factors,
    PBlocks,
    SBlocks,
    profile_enable,
    profile_collect,
    profile_i8_flops,
)
