"""MI355X-native hot path of AdLoCo: gradient statistics for adaptive batching and the
multi-instance DiLoCo outer step, behind the C ABI of include/adloco.h.

The Python layer only marshals arguments (device pointers of torch tensors, the current
HIP stream); every step of the path runs in the HIP kernels of libadloco.so.
"""
from .binding import (  # noqa: F401
    ADLOCO_ACCUMULATE, ADLOCO_SUM_ONLY, ADLOCO_ALLOW_SHRINK, ADLOCO_BF16, ADLOCO_BIASED_VAR, ADLOCO_BROADCAST,
    ADLOCO_F16, ADLOCO_F32, ADLOCO_GRAD_PROVIDED, ADLOCO_KIND_EMBED, ADLOCO_KIND_LINEAR, ADLOCO_KIND_VECTOR,
    ADLOCO_MAX_INSTANCES, AdlocoError, Context, IpAcc, IpTestResult, LinearDesc,
    NormTestResult, StatsAcc, adloco_check_merge, adloco_grad_stats, adloco_inner_product_decide,
    adloco_inner_product_test, adloco_inner_products, adloco_inner_step, adloco_merge,
    adloco_norm_test, adloco_norm_test_decide, adloco_norm_test_noalloc, adloco_outer_step, adloco_round, adloco_switch_mode,
    adloco_pack_drift, adloco_outer_step_drift, adloco_merge_drift, adloco_version, lib_path, load_library, make_layer_descs,
)
