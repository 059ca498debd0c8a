"""The C-ABI library loads and exports every symbol that include/kge.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    txt = open(os.path.join(ROOT, "include", "kge.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(kge_[a-z_]+)\s*\(", txt)))


@pytest.fixture(scope="module")
def lib():
    import paper_2211_12281_amd.binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_2211_12281_amd.build import build
        build()
    return ctypes.CDLL(b.LIB_PATH)


def test_header_declares_the_boundary_calls():
    d = _declared()
    for name in ["kge_score", "kge_loss_bwd", "kge_sparse_adam", "kge_topk", "kge_sample_negatives",
                 "kge_partition_triples", "kge_workspace_bytes", "kge_status_string"]:
        assert name in d


def test_library_exports_every_declared_symbol(lib):
    for name in _declared():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_symbols():
    import paper_2211_12281_amd.binding as b
    assert sorted(b.EXPORTS) == _declared()


def test_host_only_entry_points(lib):
    import paper_2211_12281_amd as kge
    assert kge.status_string(0) == "ok" and "workspace" in kge.status_string(-3)
    assert kge.workspace_bytes(2, None, 1000, 64) > 4 * 4 * 1000
    assert kge.workspace_bytes(2, None, -1, 64) == 0
    assert kge.workspace_bytes(99, None, 1, 1) == 0
    # argument validation happens on the host, before any GPU call
    assert lib.kge_sample_negatives(ctypes.c_uint64(1), ctypes.c_uint64(0), 7, ctypes.c_int64(5), ctypes.c_int64(5),
                                    ctypes.c_int64(4), None, None) == -1
    assert lib.kge_score(None, None, None, None, ctypes.c_int64(1), None, ctypes.c_int64(0), None, None, None,
                         ctypes.c_size_t(0), None) == -1


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2211_12281_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", "/nonexistent/libkge.so")
    with pytest.raises(b.KgeError):
        b.load()
