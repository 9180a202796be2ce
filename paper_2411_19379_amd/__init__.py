"""MI355X-native SSM-layer prefill with cached-state resume and state
checkpoints.  All compute runs in the HIP library `libssm_prefill.so`; this
package is the thin ctypes binding over its C ABI (include/ssm_prefill.h)."""
from .binding import (  # noqa: F401
    SSM_DT_BF16,
    SSM_DT_F32,
    SSM_ERR_UNSUPPORTED_SHAPE,
    SSM_PATH_MFMA_BF16,
    SSM_PATH_VALU_F32,
    SSM_ST_BF16,
    SSM_ST_F16,
    SSM_ST_F32,
    Plan,
    SsmError,
    SsmShape,
    library_path,
    load_library,
    prefill,
    ssm_last_error,
    ssm_plan_create,
    ssm_plan_destroy,
    ssm_plan_info,
    ssm_plan_tile,
    ssm_plan_workspace_bytes,
    ssm_conv1d_prefill,
    ssm_prefill,
    ssm_prefill_noalloc,
    ssm_state_advance,
)
