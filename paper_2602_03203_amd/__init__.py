"""MI355X-native budgeted-KV decode + evict path (ForesightKV generation loop).

`binding` exposes the C ABI of libfk.so (fk_append, fk_decode_attn, fk_score_kv,
fk_select_keep, fk_compact); `build` compiles it in-tree with hipcc for gfx950.
"""
from .binding import (CacheDesc, FkError, fk_append, fk_compact, fk_decode_attn, fk_decode_attn_workspace,  # noqa: F401
                      fk_decode_step, fk_decode_window, fk_decode_step_static, new_attn_workspace, fk_decode_step_feat, fk_decode_window_feat, fk_score_kv_feat, fk_compact_feat,
                      feat_heads, new_feat, new_feat_workspace, fk_golden_steps, fk_golden_scores, fk_golden_trace,
                      fk_score_kv, fk_select_keep, fk_select_keep_workspace, fk_select_keep_ws, fk_select_keep_sampled, fk_stream_read, lib, prepare, status_string, version)
