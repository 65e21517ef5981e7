"""MI355X-native batched heterogeneous-adapter LoRA delta (HIP, gfx950).

The compute lives in liblora.so (paper_2604_07173_amd/csrc, C ABI in include/lora.h); this
package is the thin ctypes binding over it.  There is no CPU fallback: without the built
library every call raises.
"""
from .binding import (  # noqa: F401
    LoraError, PoolDesc, Pool, Segments, lib_path, load_library,
    lora_pool_bytes, lora_register_pool, lora_pool_load_unit, lora_pool_load_adapter_layer,
    lora_pool_adapter_layer_bytes, lora_pool_load_adapter_async, lora_pool_set_adapter,
    lora_pool_set_activation_policy, lora_pool_activation_policy,
    lora_pool_wait_layer,
    lora_pool_layer_ready, lora_pool_read_unit, lora_pool_unit_layout, lora_pool_destroy,
    lora_segments_ws_bytes, lora_segments_launches, lora_build_segments, lora_v_bytes, lora_shrink, lora_expand, lora_apply,
    lora_group_ws_bytes, lora_apply_group, lora_group_launches,
    lora_build_apply_group, lora_build_apply_launches, lora_moe_build_apply,
    lora_moe_ws_bytes, lora_moe_apply, lora_moe_apply_static, lora_moe_shrink,
    lora_moe_combine_ws_bytes, lora_moe_down_combine, lora_moe_expand, lora_strerror,
    LORA_DTYPE_BF16, LORA_DTYPE_F32, LORA_MOE_UPGATE, LORA_MOE_DOWN, LORA_ACT_AUTO, LORA_ACT_RESIDENT, LORA_ACT_STREAMING, LORA_MAX_ROWS, LORA_MAX_ROWS_LONG, LORA_STATIC_WS_BYTES,
    EXPORTED_SYMBOLS,
    ProvisionError, lora_provision_iar, lora_provision_min_cache, lora_provision_memory_bytes,
)
