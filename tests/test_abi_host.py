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
    text = open(os.path.join(ROOT, "include", "fk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fk_[a-z_]+)\s*\(", text)))


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
    # scorer: hidden not a multiple of 32 in bf16 is unsupported; null weights invalid
    S = fklib.fk_scorer
    assert L.fk_score_kv(ctypes.byref(good), p, p, p, 512, ctypes.byref(S(p, p, p, p, 48, 1)), p, 0) == fklib.FK_ERR_UNSUPPORTED
    assert L.fk_score_kv(ctypes.byref(good), p, p, p, 512, ctypes.byref(S(0, p, p, p, 64, 1)), p, 0) == fklib.FK_ERR_INVALID_ARG
    assert L.fk_score_kv(ctypes.byref(good), p, p, p, 512, ctypes.byref(S(p, p, p, p, 4096, 1)), p, 0) == fklib.FK_ERR_UNSUPPORTED
