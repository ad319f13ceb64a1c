"""MI355X-native CO2 outer update: thin Python binding over libco2.so.

The package marshals arguments only; every step of the update runs in the HIP
kernels behind the C ABI declared in include/co2.h.  There is no CPU fallback:
if the library cannot be built or loaded, importing the binding's functions
raises.
"""
from .binding import (  # noqa: F401
    CO2_OK, CO2_EINVAL, CO2_EWORKSPACE, CO2_EHIP, CO2_ESCRATCH, CO2_STATIC_SCRATCH_BYTES, CO2_MAX_K, CO2_MAX_NORM_BUFS,
    CO2_FLAG_NONE, CO2_FLAG_CARRIED_NORMS, CO2_FLAG_CURRENT_ROUND, CO2_FLAG_ANCHOR_PULL, CO2_FLAG_NORM_CLIP, CO2_MAX_BUFFER_SET, BufferSet,
    Co2Error, Co2Params, SegmentTable, HipEvent, make_params, lib, lib_path, strerror, workspace_bytes,
    co2_outer_step, co2_outer_step_static, co2_outer_step_bf16, co2_outer_step_f16, co2_pseudo_grad_norms, co2_inner_adamw, co2_sqrt_to_f32, co2_copy_f32,
)
