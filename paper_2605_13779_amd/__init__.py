"""MI355X-native batched multi-adapter LoRA apply (thin Python binding over libmlora.so).

Every step of the hot path runs in the HIP kernels behind the C ABI declared in
``include/mlora.h``; this package only marshals arguments.  PyTorch is used for device memory
and streams.  There is no CPU fallback: importing :mod:`paper_2605_13779_amd.binding`
raises if the library has not been built.
"""
from .binding import (  # noqa: F401
    MLoraError, Site, Plan, load_library, set_tuning,
    lora_slots_upload, lora_slots_evict, lora_apply_decode, lora_apply_decode_noalloc, lora_apply_segmented,
    moe_lora_apply_packed, lora_plan_decode, lora_apply_decode_planned, moe_plan_route,
    moe_lora_apply_planned, moe_lora_apply_multi, lora_apply_decode_multi, lora_plan_apply_decode_multi, moe_down_workspace_bytes, moe_lora_apply_down,
    pack_experts, lora_slots_upload_experts, ExpertTensors, SiteDesc, Resident, lora_slot_lookup,
)
