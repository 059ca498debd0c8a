"""kge_sparse_adam_static (the entry point that allocates nothing: its scratch is a buffer built into the library)
against kge_sparse_adam with a caller-owned workspace, through the C ABI: same kernels, so the same bits; and against
the oracle to the usual bar.  Two calls in a row share the built-in buffer, the second one smaller."""
import ctypes as C

import numpy as np
import pytest
import torch

import kge_synth as ks
from helpers import RTOL_F32, norm_err

pytestmark = pytest.mark.gpu
F = np.float32


def _inputs(n_rows, d, M, seed):
    g = np.random.default_rng(seed)
    theta = g.normal(size=(n_rows, d)).astype(F) * F(0.1)
    m = (g.normal(size=(n_rows, d)) * 1e-3).astype(F)
    v = (g.normal(size=(n_rows, d)) ** 2 * 1e-5).astype(F)
    idx = ks.ZipfIds(n_rows, 1.1).draw(g, M)
    grads = (g.normal(size=(M, d)) * 1e-2).astype(F)
    return theta, m, v, idx, grads


def _raw_static(lib, b, th, sh, m, v, idx, grads, lr, step):
    """The call itself, through ctypes: device pointers and sizes only."""
    cfg = b.KgeAdamCfgT(lr, 0.9, 0.999, 1e-8, step)
    p = lambda t: None if t is None else C.c_void_p(t.data_ptr())
    return lib.kge_sparse_adam_static(p(th), p(sh), p(m), p(v), th.shape[0], th.shape[1], th.stride(0), p(idx), p(grads),
                                      idx.numel(), C.byref(cfg), C.c_void_p(torch.cuda.current_stream().cuda_stream))


def test_static_scratch_entry_point_matches_the_workspace_one(orc):
    import paper_2211_12281_amd as kge
    import paper_2211_12281_amd.binding as b
    lib = kge.load()
    # the larger call first, then a smaller one over the same built-in buffer (stale sort buffers and piece sums of
    # the first call lie behind and between what the second one uses)
    for n_rows, d, M, step, shadow in [(50000, 256, 24576, 3, True), (3000, 64, 5000, 4, False), (40, 4, 1, 5, False)]:
        theta, m, v, idx, grads = _inputs(n_rows, d, M, seed=M)
        assert kge.workspace_bytes(b.OP_SPARSE_ADAM, None, M, d) <= kge.sparse_adam_static_limit()
        dev = lambda a: torch.from_numpy(a.copy()).cuda()
        ref = [dev(theta), dev(m), dev(v)]
        got = [dev(theta), dev(m), dev(v)]
        sh_ref = torch.zeros((n_rows, d), dtype=torch.bfloat16, device="cuda") if shadow else None
        sh_got = torch.zeros((n_rows, d), dtype=torch.bfloat16, device="cuda") if shadow else None
        d_idx, d_grads = dev(idx), dev(grads)
        kge.sparse_adam(ref[0], sh_ref, ref[1], ref[2], d_idx, d_grads, 1e-3, step=step)
        assert _raw_static(lib, b, got[0], sh_got, got[1], got[2], d_idx, d_grads, 1e-3, step) == 0
        torch.cuda.synchronize()
        for a, c in zip(ref, got):
            assert bool((a == c).all())
        if shadow:
            assert bool((sh_ref.view(torch.int16) == sh_got.view(torch.int16)).all())
        # and against the oracle, to the bar of the other Adam tests
        lr, b1, b2, eps = float(F(1e-3)), float(F(0.9)), float(F(0.999)), float(F(1e-8))
        rth, rm, rv, touched = orc.sparse_adam(theta, m, v, idx, grads, lr, b1, b2, eps, step)
        gth, gm, gv = (x.cpu().numpy() for x in got)
        assert np.array_equal(gth[~touched], theta[~touched])
        upd, rupd = gth[touched].astype(np.float64) - theta[touched], rth[touched] - theta[touched]
        allowed = RTOL_F32 * np.max(np.abs(rupd)) + np.spacing(np.abs(gth[touched]).astype(F)).astype(np.float64)
        assert np.all(np.abs(upd - rupd) <= allowed)
        assert norm_err(gm[touched], rm[touched]) <= RTOL_F32 and norm_err(gv[touched], rv[touched]) <= RTOL_F32


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import paper_2211_12281_amd as kge
    import paper_2211_12281_amd.binding as b
    lib = kge.load()
    n_rows, d, M = 1000, 256, 200000                 # needs about 16 MB of sort buffers and piece sums
    assert kge.workspace_bytes(b.OP_SPARSE_ADAM, None, M, d) > kge.sparse_adam_static_limit()
    th = torch.zeros((n_rows, d), device="cuda"); m = torch.zeros_like(th); v = torch.zeros_like(th)
    idx = torch.zeros(M, dtype=torch.int32, device="cuda")
    grads = torch.ones((M, d), device="cuda")
    assert _raw_static(lib, b, th, None, m, v, idx, grads, 1e-3, 1) == -5
    torch.cuda.synchronize()
    assert float(th.abs().max()) == 0.0 and float(m.abs().max()) == 0.0          # nothing was launched
    assert "static scratch" in kge.status_string(-5)
