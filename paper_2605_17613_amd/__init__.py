"""MI355X-native hot path of VeriCache (draft / verify / accept / swap-in) - Python binding.

The compute lives in the HIP library built from csrc/; this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    VcError, Context, load, library_path,
    vc_draft_attn, vc_draft_workspace_bytes, vc_draft_attn_static, vc_draft_static_scratch_bytes, vc_verify_attn, vc_verify_workspace_bytes, vc_verify_plan, vc_verify_attn_range, vc_verify_finish,
    vc_accept_len, vc_accept_workspace_bytes, vc_swap_in, vc_swap_in_rows, vc_pack_rows, vc_swap_wait, vc_mark, vc_swap_after, vc_swap_query, vc_swap_sync, vc_keep_from_dropped,
    vc_version, vc_time_main_kernel, vc_compress_quant, vc_decompress_quant, vc_topk_keep,
    vc_iter_time_model, Sched, vc_set_tunable, vc_get_tunable, vc_stream_status, vc_validate_comp_kv, vc_validate_full_kv, vc_accept_sample, vc_accept_sample_workspace_bytes,
)
