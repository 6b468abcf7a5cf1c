"""MI355X decode-step library: thin Python binding of the C ABI in
include/decodekit.h.  Every step of the path runs in the HIP kernels of
libdecodekit.so; this package only marshals arguments (torch is used for
device memory and streams).  There is no CPU fallback: importing works
anywhere, but any call needs the built library and raises if it is missing.
"""
from .binding import (  # noqa: F401
    DecodeKitError, lib, version, last_error,
    ModelConfig as DkModelConfig, LayerWeights, WeightPtrs,
    kv_pool_bytes, create_kv_pool, destroy_kv_pool,
    kv_alloc_block, kv_alloc_block_id, kv_retain_block, kv_release_block, kv_refcount,
    kv_free_blocks, kv_offset, kv_validate_tables, append_kv,
    create_model, create_model_q4, destroy_model, read_stream, gemm_plan_query, workspace_bytes, decode_step, decode_step_static, STATIC_SCRATCH_BYTES, step_routing, step_algorithmic_bytes, profile_read, fused_status, workspace_reset, prefill_chunk, debug_set_wait_limit, debug_set_stage_stamps, STAGE_STAMPS, sample_tokens, sample_scratch_bytes,
    STEP_ADVANCE, STEP_PROFILE, STEP_NO_FUSED, KERNEL_CLASSES, STATUS,
    EngineConfig, prefix_index_create, prefix_index_destroy, prefix_index_match, prefix_index_insert,
    prefix_index_evict_lru, prefix_index_size, engine_device_bytes, engine_create, engine_destroy,
    engine_submit, engine_step, engine_poll, engine_forget, engine_stats, engine_set_sampling,
)
from .q4 import pack_q4, q4_bytes  # noqa: F401
from .runtime import DeviceModel, DeviceKV, Decoder, Prefiller  # noqa: F401
