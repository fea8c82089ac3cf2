"""MI355X-native FDA monitor: HIP kernels behind a C ABI (include/fda.h) and a thin
ctypes binding with the same entry-point names (binding.py)."""
from .binding import (  # noqa: F401
    FDA_BF16, FDA_F32, FDA_DESC_PLAIN_TABLE, FDA_VARIANT_LINEAR, FDA_VARIANT_SKETCH, FdaError, FdaDesc,
    FdaEstimate, FdaPlanInfo, fda_create, fda_destroy, fda_estimate_variance,
    fda_estimate_variance_mean, fda_estimate_variance_static, fda_get_plan, fda_last_error, fda_last_mean_state_path,
    fda_last_state_path, fda_local_state, fda_mean_state, fda_plan, fda_profile_enable, fda_profile_read, fda_state_floats,
    fda_step, FDA_STEP_MEAN_STATE, fda_calib_stream, fda_calib_lds_atomics, LDS_OPS, LDS_PATTERNS, fda_strerror, fda_sync, fda_sync_xi, fda_sync_from_mean, fda_update_xi, fda_workspace_bytes, library_path, load_library,
)
from .monitor import FdaMonitor  # noqa: F401,E402
