"""Pins of the oracle's feature-projection encoder (arXiv 2211.12281, Section 3.1 "Encoder", eq. (embedding),
and "Regularisation": dropout on the projection, L3 norms of e, e_S and M e_F)."""
import numpy as np
import pytest


def _case(n_ent=40, d=8, fd=12, B=5, N=7, seed=3):
    g = np.random.default_rng(seed)
    q = lambda a: (np.round(a * 2 ** 12) / 2 ** 12).astype(np.float32)       # exact grid: exact finite differences
    ent, feat = q(g.normal(size=(n_ent, d)) * 0.3), q(g.normal(size=(n_ent, fd)) * 0.5)
    mh, mt = q(g.normal(size=(d, fd)) * 0.2), q(g.normal(size=(d, fd)) * 0.2)
    idx = g.integers(0, n_ent, 2 * B + N).astype(np.int32)
    idx[B] = idx[0]; idx[2 * B] = idx[0]                                      # one entity as head, tail and negative
    return ent, feat, mh, mt, idx, B, N


def test_forward_is_shallow_plus_matrix_product(orc):
    ent, feat, mh, mt, idx, B, N = _case()
    om, proj, e = orc.encode(ent, feat, mh, mt, idx, B, N)
    F, S = feat[idx].astype(np.float64), ent[idx].astype(np.float64)
    ref = np.concatenate([F[:B] @ mh.astype(np.float64).T, F[B:] @ mt.astype(np.float64).T])   # heads M_H, rest M_T
    assert np.allclose(proj, ref, rtol=0, atol=1e-14)
    assert np.allclose(e, S + ref, rtol=0, atol=1e-14) and om == 0.0
    # zero projections: the encoder is the shallow table
    _, _, e0 = orc.encode(ent, feat, np.zeros_like(mh), np.zeros_like(mt), idx, B, N)
    assert np.array_equal(e0, S)
    # the same entity encodes differently as head and as tail unless M_H = M_T
    assert not np.allclose(e[0], e[B]) and np.allclose(e[B], e[2 * B])
    _, _, es = orc.encode(ent, feat, mt, mt, idx, B, N)
    assert np.allclose(es[0], es[B])


def test_dropout_mask_statistics_and_scaling(orc):
    ent, feat, mh, mt, idx, B, N = _case(n_ent=60, d=64, fd=8, B=40, N=60)
    _, proj, e0 = orc.encode(ent, feat, mh, mt, idx, B, N)
    p = 0.25
    _, proj_p, e = orc.encode(ent, feat, mh, mt, idx, B, N, p=p, seed=7, step=3, tag=11)
    assert np.array_equal(proj, proj_p)                                       # the projection itself is not dropped
    D = (e - ent[idx]) / proj                                                 # recovered factors
    kept = np.isclose(D, 1 / (1 - p), rtol=1e-9)
    assert np.all(kept | np.isclose(D, 0.0, atol=1e-9))
    assert abs(kept.mean() - (1 - p)) < 4 * np.sqrt(p * (1 - p) / D.size)     # keep rate 1 - p
    assert abs((D * 1.0).mean() - 1.0) < 0.03                                 # unbiased scaling
    # deterministic in (seed, step, tag); another step gives another mask
    assert np.array_equal(e, orc.encode(ent, feat, mh, mt, idx, B, N, p=p, seed=7, step=3, tag=11)[2])
    assert not np.array_equal(e, orc.encode(ent, feat, mh, mt, idx, B, N, p=p, seed=7, step=4, tag=11)[2])
    # rows and columns are masked independently: no all-kept or all-dropped rows / columns in 140 x 64
    assert 0 < kept.sum(axis=1).min() and kept.sum(axis=1).max() < 64 and 0 < kept.sum(axis=0).min()


def test_regulariser_value_is_sum_of_library_norms(orc):
    ent, feat, mh, mt, idx, B, N = _case()
    om, proj, e = orc.encode(ent, feat, mh, mt, idx, B, N, p=0.3, seed=1, step=2, tag=3, reg_t=0.5, reg_s=0.25, reg_f=2.0)
    n3 = lambda a: np.linalg.norm(a, ord=3, axis=1).sum()
    assert abs(om - (0.5 * n3(e) + 0.25 * n3(ent[idx].astype(np.float64)) + 2.0 * n3(proj))) < 1e-12 * om


@pytest.mark.parametrize("p", [0.0, 0.3])
def test_backward_matches_central_differences(orc, p):
    """Scalar test function J = sum(c o e) + regulariser, with fixed random c: dJ/de = c, so encode_bwd(c) must
    give dJ/dM_H, dJ/dM_T and (after summing the slots of a row) dJ/de_S; checked entry by entry."""
    ent, feat, mh, mt, idx, B, N = _case()
    g = np.random.default_rng(9)
    c = g.normal(size=(2 * B + N, ent.shape[1]))
    kw = dict(p=p, seed=5, step=6, tag=7, reg_t=0.3, reg_s=0.2, reg_f=0.4)

    def J(ent_, mh_, mt_):
        om, _, e = orc.encode(ent_, feat, mh_, mt_, idx, B, N, **kw)
        return float((c * e).sum() + om)

    g_s, g_mh, g_mt = orc.encode_bwd(ent, feat, mh, mt, idx, B, N, c, **kw)
    dense = np.zeros(ent.shape); np.add.at(dense, idx, g_s)
    step = 2.0 ** -10
    for name, arr, grad in (("ent", ent, dense), ("mh", mh, g_mh), ("mt", mt, g_mt)):
        for _ in range(25):
            i, j = int(g.integers(0, arr.shape[0])), int(g.integers(0, arr.shape[1]))
            if name == "ent" and i not in idx:
                assert grad[i, j] == 0.0
                continue
            keep = arr[i, j]
            arr[i, j] = np.float32(keep + step); jp = J(ent, mh, mt)
            arr[i, j] = np.float32(keep - step); jm = J(ent, mh, mt)
            arr[i, j] = keep
            fd = (jp - jm) / (2 * step)
            assert abs(fd - grad[i, j]) < 2e-5 * max(1.0, np.abs(grad).max()), (name, i, j, fd, grad[i, j])


def test_projection_gradient_is_an_outer_product_sum(orc):
    """Without regularisers and dropout: g_mh = de_heads^t F_heads, g_mt = de_rest^t F_rest, g_s = de."""
    ent, feat, mh, mt, idx, B, N = _case()
    de = np.random.default_rng(2).normal(size=(2 * B + N, ent.shape[1]))
    g_s, g_mh, g_mt = orc.encode_bwd(ent, feat, mh, mt, idx, B, N, de)
    F = feat[idx].astype(np.float64)
    assert np.array_equal(g_s, de)
    assert np.allclose(g_mh, de[:B].T @ F[:B], atol=1e-13) and np.allclose(g_mt, de[B:].T @ F[B:], atol=1e-13)
