"""The C-ABI library loads and exports every function include/eesd.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "eesd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(eesd_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_round_calls():
    names = _declared()
    for n in ("eesd_create", "eesd_prefill", "eesd_draft_step", "eesd_verify", "eesd_accept", "eesd_rollback", "eesd_generate"):
        assert n in names


def test_library_exports_every_declared_function():
    import paper_2406_03853_amd as pk
    assert os.path.exists(pk.lib_path()), "libeesd.so is not built (python -m paper_2406_03853_amd.build)"
    L = ctypes.CDLL(pk.lib_path())
    missing = [n for n in _declared() if not hasattr(L, n)]
    assert not missing, missing
    # the binding knows them all too
    assert sorted(pk.binding.EXPORTS) == _declared()


def test_struct_sizes_match_the_header_layout():
    import paper_2406_03853_amd.binding as b
    # 15 int32/float fields (60) + pad to 8 + seed + 2 doubles + 7 int32 + pad to 8 = 120
    assert ctypes.sizeof(b._Config) == 120
    assert ctypes.sizeof(b._Layer) == 48
    assert ctypes.sizeof(b._Weights) == 4 * 8 + 48 + 2 * 8
    assert ctypes.sizeof(b._Stats) == 4 * 8 + 9 * 8


def test_null_arguments_are_rejected_without_a_gpu():
    import paper_2406_03853_amd as pk
    L = pk.lib()
    assert L.eesd_create(None, None, None, None) == -1
    assert L.eesd_prefill(None, None, 0, None) == -1
    assert L.eesd_set_tunable(b"no_such_knob", 1) == -1
    assert L.eesd_last_error(None) == b"no context"
