"""MI355X-native NVFP4 + LoRA linear with AQN RMSNorm (QeRL rollout hot path).

The work is done by hand-written HIP kernels in libqerl_nvfp4.so behind the C
ABI of include/qerl_nvfp4.h; this package only marshals torch GPU tensors to it.
"""
from .binding import (  # noqa: F401
    EXPORTED_SYMBOLS, LIB_PATH, PackedWeight, QerlError, Workspace, nvfp4_lora_linear_packed, nvfp4_lora_linear_packed_noalloc, nvfp4_lora_linear_packed_swiglu, nvfp4_prepack_t, nvfp4_lora_linear_backward, PackedWeightT, nvfp4_lora_linear_packed_group, nvfp4_prepack, aqn_rmsnorm, aqn_rmsnorm_lora_down, aqn_rmsnorm_nvfp4_lora_linear_group, aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes, aqn_rmsnorm_nvfp4_lora_mlp, workspace_status, aqn_sigma, aqn_sigma_schedule, aqn_noise_fill, load_library, mxfp4_quantize, mxfp4_dequantize, mxfp8_quantize, mxfp4_prepack, mxfp4_linear_native, MxPackedWeight,
    nvfp4_dequantize, nvfp4_lora_linear, nvfp4_lora_linear_workspace_bytes, nvfp4_quantize,
    nvfp4_quantize_workspace_bytes, mxfp4_lora_linear_native, nvfp4_lora_linear_backward_group,
)
