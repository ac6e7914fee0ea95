"""MI355X-native hot path under micro-request execution: mixed-batch paged-KV attention,
KV append and chunked KV pack/unpack, as hand-written HIP kernels behind a C ABI (``include/dsv_attn.h``).

This package is only the thin Python binding; importing it does not load the library.  Every
call goes to ``libdsv_attn.so``; there is no CPU or eager fallback, and a missing library raises.
"""
from .binding import (  # noqa: F401
    DSV_OUT_BF16, DSV_OUT_F32, ChunkDescs, DsvError, KVPool, attn_mixed_batch,
    attn_mixed_batch_workspace_bytes, build_info, dsv_profile_events, KERNEL_PLAN, KERNEL_ROWS,
    KERNEL_TILES, KERNEL_MERGE, KERNEL_MIXED, KERNEL_STAGE, kv_append, kv_pack_chunks, kv_unpack_chunks,
    library_path, load_library, attn_mixed_batch_fp8kv, attn_mixed_batch_fp8kv_workspace_bytes,
    kv_append_fp8, kv_pack_chunks_fp8, kv_unpack_chunks_fp8, AttnPlan, attn_mixed_batch_plan,
    attn_mixed_batch_planned, attn_mixed_batch_fp8kv_planned, attn_mixed_batch_static,
    attn_mixed_batch_static_max_bytes, dsv_check_block_tables, kv_unpack_chunks_ordered,
    kv_unpack_chunks_ordered_workspace_bytes, dsv_calib_hbm, dsv_calib_mfma, dsv_calib_mfma_data, dsv_calib_paged_read,
    attn_mixed_batch_plan_info,
)
