"""ThinK key-cache channel pruning and pruned-cache decode attention for MI355X.

Thin ctypes binding over libthk.so (hand-written HIP, gfx950).  Every step of
the path runs in the library's kernels; this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    THK_BF16, THK_F32, THK_OP_DECODE, THK_OP_PRUNE, THK_OP_SCORE, THK_OP_PRUNE_VALUE, THK_OP_SCORE_VALUE, THK_STREAM_COPY, THK_STREAM_READ, THK_STREAM_WRITE, ThkError, lib_path, load,
    make_shape, thk_cache_append, thk_compact_keys, thk_compact_rows, thk_copy_rows, thk_decode_attn, thk_decode_attn_kv, thk_bench_stream, thk_decode_attn_static, thk_decode_on_matrix_cores, thk_default_split, thk_keep_count, thk_last_hip_error, thk_profile_next, thk_prune, thk_prune_is_fused, thk_prune_launches, thk_prune_value, thk_reload_env,
    thk_score, thk_score_magnitude, thk_score_value, thk_select_topk, thk_shape, thk_status_string,
    thk_tail_append, thk_tail_flush, thk_version, thk_workspace_bytes)
