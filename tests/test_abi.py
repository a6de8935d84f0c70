"""CPU-only checks of the C ABI: the library builds, loads and exports every
symbol the header declares; argument validation that needs no GPU."""
import ctypes
import os
import re

import pytest

import paper_2511_16947_amd as fm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "finemoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fine_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(fm.LIB_PATH):
        from paper_2511_16947_amd import build
        build.build()
    return fm.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert set(names) == set(fm.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_workspace_queries(lib):
    assert fm.fine_version() >= 100
    s = fm.Shape(256, 128, 256, 8, 2, 4, fm.FINE_F32)
    for which in (fm.WS_TOPK, fm.WS_SCHED, fm.WS_FFN, fm.WS_BACKWARD):
        assert fm.fine_workspace_bytes(s, which) > 0
    assert fm.fine_workspace_bytes(s, 99) == 0
    # G does not divide T, K > E, bf16 with d not a multiple of 64: rejected
    assert fm.fine_workspace_bytes(fm.Shape(250, 128, 256, 8, 2, 4, fm.FINE_F32), fm.WS_SCHED) == 0
    assert fm.fine_workspace_bytes(fm.Shape(256, 128, 256, 2, 3, 4, fm.FINE_F32), fm.WS_SCHED) == 0
    assert fm.fine_workspace_bytes(fm.Shape(256, 100, 256, 8, 2, 4, fm.FINE_BF16), fm.WS_FFN) == 0
    # the gate's workspace: room for the partial logits when blocks share a token tile (bf16, more than
    # 64 experts, few tokens, a long enough k range), a token amount otherwise
    gate = lambda T, d, E, dt=fm.FINE_BF16: fm.fine_workspace_bytes(fm.Shape(T, d, 64, E, 2, 1, dt), fm.WS_TOPK)
    assert gate(4096, 7168, 256) == 4 * 4096 * 256 * 4          # 128 tiles: 4 parts of the 112 steps
    assert gate(4096, 2048, 128) == 4 * 4096 * 128 * 4          # 32 steps: 4 parts of 8
    assert gate(40, 4608, 160) == 8 * 64 * 256 * 4              # 2 tiles of 32 tokens, 8 parts; 160 experts padded to 256
    assert gate(4096, 512, 256) == 256                          # 8 steps: not worth splitting
    assert gate(32768, 7168, 256) == 256                        # 1024 tiles fill the chip
    assert gate(4096, 7168, 64) == 256                          # 64 experts: the waves of a block split k already
    assert gate(4096, 7168, 256, fm.FINE_F32) == 256


def test_null_pointers_are_rejected_without_touching_the_gpu(lib):
    s = fm.Shape(256, 128, 256, 8, 2, 4, fm.FINE_F32).c()
    rc = lib.fine_permute(ctypes.byref(s), None, None, None, None)
    assert rc == fm.FINE_INVALID_ARG
    rc = lib.fine_combine(ctypes.byref(s), None, None, None, None, None)
    assert rc == fm.FINE_INVALID_ARG
    bad = fm.Shape(256, 128, 256, 8, 9, 4, fm.FINE_F32).c()
    assert lib.fine_permute(ctypes.byref(bad), None, None, None, None) == fm.FINE_INVALID_ARG
    # both scheduling entry points: outputs and workspace are required, x_prev is optional
    none12 = [None] * 12
    assert lib.fine_sched_warm(ctypes.byref(s), *none12, None, 0, None) == fm.FINE_INVALID_ARG
    assert lib.fine_sched(ctypes.byref(s), *none12[:11], None, 0, None) == fm.FINE_INVALID_ARG
    buf = ctypes.c_void_p(4096)        # non-null, 16-byte aligned; the size check below fails before any use
    assert lib.fine_sched_warm(ctypes.byref(s), buf, None, None, *([buf] * 9), buf, 16, None) == fm.FINE_WORKSPACE_TOO_SMALL
    # the placement entry points check their arguments on the host as well
    assert lib.fine_replica_counts(ctypes.byref(s), None, 4, None, None) == fm.FINE_INVALID_ARG
    assert lib.fine_eval_placements(ctypes.byref(s), 1, None, None, None, None, None) == fm.FINE_INVALID_ARG
    assert lib.fine_place_search(ctypes.byref(s), None, None, 4, 8, 0, None, None, None, None, None) == fm.FINE_INVALID_ARG
    one = ctypes.c_void_p(16)          # any non-null address: the checks below fail before it is used
    assert lib.fine_replica_counts(ctypes.byref(s), one, 1, one, None) == fm.FINE_INVALID_ARG       # 4 slots, 8 experts
    assert lib.fine_place_search(ctypes.byref(s), one, one, 4, 0, 0, one, one, one, one, None) == fm.FINE_INVALID_ARG
    wide = fm.Shape(256, 128, 256, 1024, 2, 64, fm.FINE_F32).c()     # flow tables of 1024 experts x 64 ranks: no room
    assert lib.fine_place_search(ctypes.byref(wide), one, one, 32, 8, 0, one, one, one, one, None) == fm.FINE_UNSUPPORTED
    assert lib.fine_eval_placements(ctypes.byref(wide), 1, one, one, one, one, None) == fm.FINE_UNSUPPORTED
    assert lib.fine_eval_placements(ctypes.byref(s), 0, None, one, None, None, None) == fm.FINE_OK    # nothing to score


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(fm, "_lib", None)
    monkeypatch.setattr(fm, "LIB_PATH", str(tmp_path / "libfinemoe.so"))
    with pytest.raises(FileNotFoundError):
        fm.fine_version()
