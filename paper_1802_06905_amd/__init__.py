"""cacnn for MI355X: thin Python binding over the C-ABI library libcacnn.so (see include/cacnn.h).

Only argument marshalling happens here; every step of the convolution and of the pooling runs in the HIP kernels.  PyTorch is used by
callers for device memory and streams only.
"""
from .binding import (  # noqa: F401
    CACNN_BF16_F32ACC,
    CACNN_F32,
    CACNN_POOL_AVG,
    CACNN_POOL_MAX,
    CacnnError,
    Bound,
    Division,
    Machine,
    Plan,
    PoolBound,
    ClosedForm,
    MachineL2,
    L2Plan,
    Problem,
    cacnn_conv_forward,
    cacnn_conv_forward_with_plan,
    cacnn_lower_bound,
    cacnn_parallel_bound,
    cacnn_pool_forward,
    cacnn_pool_lower_bound,
    cacnn_two_level_plan,
    cacnn_plan_variant,
    cacnn_closed_form_tiling,
    cacnn_probe_copy,
    cacnn_probe_mfma,
    cacnn_status_string,
    cacnn_tile_plan,
    cacnn_tune,
    cacnn_variant_count,
    cacnn_variant_name,
    cacnn_work_division,
    library_path,
)
