"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def fklib():
    from paper_2602_03203_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2602_03203_amd import build
        build.build()
    return binding


def declared_functions():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(fk_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(fklib):
    names = declared_functions()
    assert {"fk_append", "fk_decode_attn", "fk_score_kv", "fk_select_keep", "fk_compact"} <= set(names)
    L = fklib.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(fklib.SYMBOLS) == names          # the Python binding covers the same set
    assert "gfx950" in fklib.version()


def test_status_strings(fklib):
    assert fklib.status_string(0) == "ok"
    assert len({fklib.status_string(i) for i in range(5)}) == 5


def test_argument_validation_without_gpu(fklib):
    L = fklib.lib()
    D = fklib.fk_cache_desc
    good = D(2, 8, 2, 128, 512, fklib.FK_BF16)
    assert L.fk_decode_step(ctypes.byref(good), 0, 0, 0, 0, 0, 0, 0, 0, 512, 1.0, 0, 0, 0, 0) == fklib.FK_ERR_INVALID_ARG
    # null buffers
    assert L.fk_append(ctypes.byref(good), 0, 0, 0, 0, 0, 0, 0, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_decode_attn(ctypes.byref(good), 0, 0, 0, 0, 512, 1.0, 0, 0, 0, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_compact(ctypes.byref(good), 0, 0, 0, 0, 0, 256, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_select_keep(ctypes.byref(good), 0, 0, 0, 512, 256, 32, 0, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_score_kv(ctypes.byref(good), 0, 0, 0, 512, None, 0, 0) == fklib.FK_ERR_INVALID_ARG
    # bad descriptors
    for bad, code in [(D(0, 8, 2, 128, 512, 1), fklib.FK_ERR_INVALID_ARG), (D(2, 7, 2, 128, 512, 1), fklib.FK_ERR_INVALID_ARG),
                      (D(2, 8, 2, 96, 512, 1), fklib.FK_ERR_UNSUPPORTED), (D(2, 8, 2, 128, 512, 5), fklib.FK_ERR_UNSUPPORTED),
                      (D(2, 32, 2, 128, 512, 1), fklib.FK_ERR_UNSUPPORTED), (D(2, 8, 2, 128, 1 << 24, 1), fklib.FK_ERR_UNSUPPORTED)]:
        assert L.fk_append(ctypes.byref(bad), 16, 16, 16, 16, 16, 16, 16, 0) == code
        assert L.fk_decode_attn_workspace(ctypes.byref(bad), 100) == 0
    # budget / recent / max_len ranges (pointers are fake but non-null and aligned: rejected before use)
    p = 4096
    assert L.fk_select_keep(ctypes.byref(good), p, p, p, 512, 600, 32, p, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_select_keep(ctypes.byref(good), p, p, p, 512, 256, 300, p, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_select_keep(ctypes.byref(good), p, p, p, 513, 256, 32, p, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_compact(ctypes.byref(good), p, p, p, p, p, 0, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_decode_attn(ctypes.byref(good), p, p, p, p, 0, 1.0, p, p, 1 << 30, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_decode_attn(ctypes.byref(good), p + 4, p, p, p, 512, 1.0, p, p, 1 << 30, 0) == fklib.FK_ERR_INVALID_ARG   # misaligned q
    # workspace too small / missing
    need = L.fk_decode_attn_workspace(ctypes.byref(good), 512)
    assert need > 0
    assert L.fk_decode_attn(ctypes.byref(good), p, p, p, p, 512, 1.0, p, p, need - 1, 0) == fklib.FK_ERR_WORKSPACE
    assert L.fk_decode_attn(ctypes.byref(good), p, p, p, p, 512, 1.0, p, 0, 0, 0) == fklib.FK_ERR_WORKSPACE
    # scorer: hidden not a multiple of 8 in bf16 is unsupported; null weights invalid
    S = fklib.fk_scorer
    assert L.fk_score_kv(ctypes.byref(good), p, p, p, 512, ctypes.byref(S(p, p, p, p, 44, 1)), p, 0) == fklib.FK_ERR_UNSUPPORTED
    assert L.fk_score_kv(ctypes.byref(good), p, p, p, 512, ctypes.byref(S(0, p, p, p, 64, 1)), p, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_score_kv(ctypes.byref(good), p, p, p, 512, ctypes.byref(S(p, p, p, p, 4096, 1)), p, 0) == fklib.FK_ERR_UNSUPPORTED


def test_argument_validation_of_the_next_row_calls(fklib):
    """Sampled selection, the feature path and the Golden Eviction builder reject bad arguments on the host."""
    L = fklib.lib()
    D = fklib.fk_cache_desc
    good = D(2, 8, 2, 128, 512, fklib.FK_BF16)
    p = 4096
    big = D(1, 8, 2, 128, 1 << 20, fklib.FK_BF16)
    assert L.fk_select_keep_sampled(ctypes.byref(good), p, 0, p, p, 512, 256, 32, 64, p, 0) == fklib.FK_ERR_INVALID_ARG   # no noise
    assert L.fk_select_keep_sampled(ctypes.byref(good), p, p, p, p, 512, 256, 32, -1, p, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_select_keep_sampled(ctypes.byref(big), p, p, p, p, 1 << 20, 256, 32, 64, p, 0) == fklib.FK_ERR_UNSUPPORTED
    # feature path
    need = L.fk_decode_step_feat_workspace(ctypes.byref(good))
    assert need >= 2 * 2 * 512 * 4 * 4
    assert L.fk_decode_step_feat_workspace(ctypes.byref(D(2, 7, 2, 128, 512, 1))) == 0
    args = [p] * 8
    assert L.fk_decode_step_feat(ctypes.byref(good), *args, 512, 1.0, 0, 0, 128, p, p, need, 0) == fklib.FK_ERR_INVALID_ARG   # no state
    assert L.fk_decode_step_feat(ctypes.byref(good), *args, 512, 1.0, p, 128, 128, p, p, need, 0) == fklib.FK_ERR_INVALID_ARG  # chunk_pos
    assert L.fk_decode_step_feat(ctypes.byref(good), *args, 512, 1.0, p, 0, 0, p, p, need, 0) == fklib.FK_ERR_INVALID_ARG      # chunk_len
    assert L.fk_decode_step_feat(ctypes.byref(good), *args, 512, 1.0, p, 0, 128, p, p, need - 1, 0) == fklib.FK_ERR_WORKSPACE
    S = fklib.fk_scorer
    assert L.fk_score_kv_feat(ctypes.byref(good), p, p, 0, p, 512, ctypes.byref(S(p, p, p, p, 64, 1)), p, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_score_kv_feat(ctypes.byref(good), p, p, p, p, 512, ctypes.byref(S(p, p, p, p, 44, 1)), p, 0) == fklib.FK_ERR_UNSUPPORTED
    assert L.fk_compact_feat(ctypes.byref(good), p, p, p, 0, p, p, 256, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_compact_feat(ctypes.byref(good), p, p, p, p, p, p, 513, 0) == fklib.FK_ERR_INVALID_ARG
    # windows of the feature path: the window must end inside the chunk
    assert L.fk_decode_window_feat(ctypes.byref(good), *args, 4, 512, 1.0, p, 126, 128, p, p, need, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_decode_window_feat(ctypes.byref(good), *args, 0, 512, 1.0, p, 0, 128, p, p, need, 0) == fklib.FK_OK   # no step: no launch
    assert L.fk_decode_window_feat(ctypes.byref(good), p, p, p, p, p, 0, p, p, 4, 512, 1.0, p, 0, 128, p, p, need, 0) == fklib.FK_ERR_INVALID_ARG
    # selection of few long rows: workspace sizes are a host-side plan; a short workspace is refused before any launch
    long_rows = D(1, 8, 4, 128, 131072, fklib.FK_BF16)
    ws = L.fk_select_keep_workspace(ctypes.byref(long_rows), 131072, 2048, 128)
    assert ws >= 4 * 2 * (2048 - 128) * 4                      # at least two chunks of survivors per row
    assert L.fk_select_keep_workspace(ctypes.byref(good), 512, 256, 32) == 0           # short rows are not split
    assert L.fk_select_keep_workspace(ctypes.byref(long_rows), 131072, 2048, 2048) == 0   # nothing to select
    assert L.fk_select_keep_workspace(ctypes.byref(long_rows), 131073, 2048, 128) == 0    # bad arguments
    assert L.fk_select_keep_ws(ctypes.byref(long_rows), p, p, p, 131072, 2048, 128, p, p, ws - 1, 0) == fklib.FK_ERR_WORKSPACE
    assert L.fk_select_keep_ws(ctypes.byref(long_rows), p, p, p, 131072, 2048, 128, p, 0, 0, 0) == fklib.FK_ERR_WORKSPACE
    assert L.fk_select_keep_ws(ctypes.byref(long_rows), p, p, p, 131072, 4096, 5000, p, p, ws, 0) == fklib.FK_ERR_INVALID_ARG
    # Golden Eviction
    assert L.fk_golden_steps(8192, 2048, 128) == 47 and L.fk_golden_steps(2176, 2048, 128) == 0
    assert L.fk_golden_steps(0, 2048, 128) == -1 and L.fk_golden_steps(100, 8, 16) == -1
    assert L.fk_golden_scores(0, 1, 8, 2, 512, 512, 64, 16, p, p, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_golden_scores(p, 1, 8, 3, 512, 512, 64, 16, p, p, 0) == fklib.FK_ERR_INVALID_ARG       # heads do not divide
    assert L.fk_golden_scores(p, 1, 8, 2, 512, 510, 64, 16, p, p, 0) == fklib.FK_ERR_INVALID_ARG       # ld < T
    assert L.fk_golden_scores(p, 1, 8, 2, 510, 516, 64, 16, p, p, 0) == fklib.FK_ERR_INVALID_ARG       # ld not a multiple of 8
    assert L.fk_golden_scores(p, 7, 8, 2, 512, 512, 64, 16, p, p, 0) == fklib.FK_ERR_UNSUPPORTED       # dtype
    assert L.fk_golden_scores(p, 1, 8, 2, 512, 512, 16, 64, p, p, 0) == fklib.FK_ERR_INVALID_ARG       # L > B
    assert L.fk_golden_scores(p, 1, 8, 2, 64, 64, 64, 16, p, p, 0) == fklib.FK_OK                       # M == 0: nothing to do
    assert L.fk_golden_trace(0, 2, 512, 64, 16, p, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_golden_trace(p, 2, 100000, 20000, 16, p, 0) == fklib.FK_ERR_UNSUPPORTED
    assert L.fk_golden_trace(p, 2, 64, 64, 16, p, 0) == fklib.FK_OK
