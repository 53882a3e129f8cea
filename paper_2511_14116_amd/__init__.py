"""MI355X-native cyclic/hybrid decode-attention share (thin binding over libfailsafe.so).

Every step of the path runs in the native library (host builders in C++, kernels in
HIP for gfx950); this package only marshals arguments.  There is no fallback: if the
library is not built, importing the binding's functions raises.
"""
from .binding import (  # noqa: F401
    FS_OK, FS_EINVAL, FS_ECAPACITY, FS_EHIP, FS_EUNSUPPORTED,
    FS_MODE_TP, FS_MODE_DP, FS_KV_BF16, FS_KV_FP8_E4M3, FS_V_ANY, FS_V_FP16_RANGE,
    FsError, FsShape, FsKvView, ITEM_DTYPE, PAIR_DTYPE, RECORD_DTYPE, PREFILL_ENTRY_DTYPE, PREFILL_ITEM_DTYPE, PREFILL_PAIR_DTYPE,
    fs_build_prefill_worklist, fs_choose_prefill_chunk, fs_prefill_attention, fs_prefill_attention_fused, fs_prefill_tile_tokens,
    fs_route_request, fs_route_requests, fs_schedule_prefill, fs_plan_kv_reload, fs_replace_failed_gpu, fs_plan_ffn_reload,
    library_path, load_library,
    fs_build_placement, fs_build_placement_hybrid_heads, fs_build_worklist, fs_build_worklist_units, fs_build_launch_records, fs_choose_chunk_tokens, fs_decode_attention, fs_decode_attention_persistent, fs_decode_attention_fused, fs_decode_attention_fused_static, fs_decode_attention_units, fs_decode_attention_records, fs_merge_lse,
    BoundCall, bind_build_placement, bind_build_placement_hybrid_heads, bind_build_worklist, bind_build_worklist_units, bind_build_prefill_worklist, bind_choose_prefill_chunk, bind_route_requests, bind_schedule_prefill, bind_decode_attention, bind_decode_attention_persistent, bind_decode_attention_fused, bind_decode_attention_units, bind_build_launch_records, bind_decode_attention_records, bind_merge_lse,
    fs_kv_elem_offset, fs_pack_kv_slots, fs_stream_read_probe, fs_set_option, fs_get_option, fs_last_error, fs_abi_version,
)
from .layout import slot_permutation, pack_slots  # noqa: F401
