"""PEVLM prefill attention for AMD MI355X (gfx950): Python binding of libpevlm.so.

The binding only marshals arguments; every step of the path (sequential RoPE, block-parallel
prefill attention, split-KV question attention + merge) runs in the HIP kernels behind the C ABI
declared in include/pevlm.h.  There is no CPU fallback: loading fails if the library is missing.
"""
from .binding import (  # noqa: F401
    Heads,
    Layout,
    PevlmError,
    StreamItem,
    WorkItem,
    lib_path,
    load_library,
    pevlm_block_prefill_attn,
    pevlm_block_prefill_attn_blocks,
    pevlm_block_prefill_attn_mrope,
    pevlm_block_prefill_attn_rope,
    pevlm_block_prefill_rope_workspace_bytes,
    pevlm_block_prefill_workspace_bytes,
    pevlm_last_error,
    pevlm_prefill_tile_rows,
    pevlm_prefill_stream_items_host,
    pevlm_prefill_uses_stream_kernel,
    pevlm_prefill_worklist_host,
    pevlm_probe_copy,
    pevlm_probe_mfma_bf16,
    pevlm_query_attn,
    pevlm_query_attn_static,
    pevlm_query_attn_mrope,
    pevlm_query_attn_rope,
    pevlm_query_attn_window,
    pevlm_query_window_workspace_bytes,
    pevlm_query_worklist_window_host,
    pevlm_prefill_worklist_blocks_host,
    pevlm_query_rope_workspace_bytes,
    pevlm_query_tile_rows,
    pevlm_query_workspace_bytes,
    pevlm_query_worklist_host,
    pevlm_rope_mrope,
    pevlm_rope_seq,
    pevlm_set_prefill_kernel,
    pevlm_version,
    pevlm_visible_pairs,
)
from .cost_model import (  # noqa: F401
    choose_block_len,
    choose_sink_and_block,
    predict_block_prefill_ms,
    prefill_work,
    stream_work,
    useful_flops,
    video_layout,
)
