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


def test_profile_slots_are_selected_by_mask(lib):
    """kge_profile_enable: 0 off, negative every slot, positive a bit mask of slots; nothing is recorded without a GPU
    call, so collecting returns zero launches."""
    import paper_2211_12281_amd as kge
    for on in (True, ["block_fwd"], ["adam", "sort"], False):
        kge.profile_enable(on)
    with pytest.raises(KeyError):
        kge.profile_enable(["no_such_slot"])
    kge.profile_enable(False)
    ms, n = ctypes.c_double(1.0), ctypes.c_int64(7)
    assert lib.kge_profile_collect(1, ctypes.byref(ms), ctypes.byref(n)) == 0 and n.value == 0 and ms.value == 0.0
    assert lib.kge_profile_collect(99, ctypes.byref(ms), ctypes.byref(n)) == -1


def test_calibration_calls_validate_their_arguments(lib):
    out = ctypes.c_double(0.0)
    assert lib.kge_calibrate_mfma(0, None, ctypes.c_int64(0), ctypes.byref(out), None) == -1
    assert lib.kge_calibrate_mfma(16, ctypes.c_void_p(4096), ctypes.c_int64(1000), ctypes.byref(out), None) == -1   # sink too small
    assert lib.kge_calibrate_mfma_varied(0, None, ctypes.c_int64(0), ctypes.byref(out), None) == -1
    assert lib.kge_calibrate_mfma_varied(16, ctypes.c_void_p(4096), ctypes.c_int64(1000), ctypes.byref(out), None) == -1
    assert lib.kge_calibrate_copy(None, None, ctypes.c_size_t(1 << 20), ctypes.byref(out), None) == -1
    assert lib.kge_calibrate_copy(ctypes.c_void_p(4096), ctypes.c_void_p(8200), ctypes.c_size_t(1 << 20), ctypes.byref(out),
                                  None) == -1                                                                      # unaligned


def test_alignment_rules_are_checked_on_the_host(lib):
    """Misaligned table pointers are refused before anything is launched (fake addresses: nothing dereferences them)."""
    import paper_2211_12281_amd.binding as b
    cfg = b.KgeAdamCfgT(1e-3, 0.9, 0.999, 1e-8, 1)
    p = ctypes.c_void_p
    ok = 0x10000000
    call = lambda th, sh, m, v, g: lib.kge_sparse_adam(p(th), p(sh), p(m), p(v), ctypes.c_int64(100), 8, ctypes.c_int64(8), p(ok),
                                                      p(g), ctypes.c_int64(4), ctypes.byref(cfg), None, ctypes.c_size_t(0), None)
    assert call(ok, ok, ok, ok, ok) == -3                       # everything aligned: gets as far as the missing workspace
    for bad in [(ok + 4, ok, ok, ok, ok), (ok, ok + 2, ok, ok, ok), (ok, ok, ok + 8, ok, ok), (ok, ok, ok, ok + 4, ok),
                (ok, ok, ok, ok, ok + 12)]:
        assert call(*bad) == -1
    # kge_topk: rows of the entity table must be 16-byte aligned
    m = b.KgeModelT()
    m.scorer, m.p_norm, m.dtype, m.dim, m.rel_dim = b.SCORERS["distmult"], 2, 1, 64, 64
    m.n_ent, m.n_rel, m.ent, m.rel, m.ent_ld, m.rel_ld = 1000, 10, ok, ok, 67, 64
    topk = lambda: lib.kge_topk(ctypes.byref(m), p(ok), p(ok), ctypes.c_int64(8), ctypes.c_int64(0), ctypes.c_int64(1000), 10,
                                p(ok), p(ok), None, None, None, ctypes.c_size_t(0), None)
    assert topk() == -2                                         # unsupported: row stride of 134 bytes
    m.ent_ld = 72
    assert topk() == -3                                         # aligned rows: gets as far as the missing workspace


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2211_12281_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", "/nonexistent/libkge.so")
    with pytest.raises(b.KgeError):
        b.load()
