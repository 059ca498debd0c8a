"""Pins of the oracle's L3 regulariser (arXiv 2211.12281, Section 3.1 "Regularisation"):
Omega_S = sum_b (||h_b||_3 + ||t_b||_3) + sum_i ||t'_i||_3 added to the micro-batch loss with weight lambda_S."""
import numpy as np
import pytest

from helpers import small_graph


def test_norm_equals_library_p_norm(orc):
    g = np.random.default_rng(3)
    for d in (1, 7, 32, 256):
        x = g.normal(size=d).astype(np.float32)
        n, _ = orc.l3_norm(x)
        assert abs(n - np.linalg.norm(x.astype(np.float64), ord=3)) <= 1e-14 * max(1.0, n)


def test_norm_closed_forms(orc):
    # constant vector: |c| d^(1/3); a single non-zero entry: its magnitude; zero vector: 0 with zero gradient
    n, _ = orc.l3_norm(np.full(27, -0.5, dtype=np.float32))
    assert abs(n - 0.5 * 3.0) < 1e-15
    n, grad = orc.l3_norm(np.array([0, 0, -2.0, 0], dtype=np.float32), lam=1.0)
    assert n == 2.0 and np.array_equal(grad, [0, 0, -1.0, 0])
    n, grad = orc.l3_norm(np.zeros(5, dtype=np.float32), lam=1.0)
    assert n == 0.0 and not grad.any()


def test_gradient_is_homogeneous_and_matches_differences(orc):
    g = np.random.default_rng(5)
    x = (np.round(g.normal(size=24) * 2 ** 10) / 2 ** 10).astype(np.float32)
    lam = 0.75
    n, grad = orc.l3_norm(x, lam=lam)
    # Euler: a norm is homogeneous of degree one, x . grad = ||x||
    assert abs(np.dot(x.astype(np.float64), grad) - lam * n) < 1e-13
    step = 2.0 ** -14
    for j in range(24):
        xp, xm = x.copy(), x.copy()
        xp[j] += step; xm[j] -= step
        fd = lam * (orc.l3_norm(xp)[0] - orc.l3_norm(xm)[0]) / (2 * step)
        assert abs(fd - grad[j]) < 1e-7
    # the sign follows the entry, the magnitude grows with it
    assert np.all(np.sign(grad) == np.sign(x))


@pytest.mark.parametrize("scorer,loss", [("distmult", "sampled_softmax"), ("transe", "logsigmoid")])
def test_regularised_loss_is_sum_of_parts(orc, scorer, loss):
    """The regularised loss and gradient are the unregularised ones plus lambda times the norms (gradients)
    of the gathered rows, slot by slot; duplicates of a row are counted once per slot."""
    G = small_graph(scorer, 300, 5, 16, 20, 30, amp=0.3)
    G["t"][2] = G["h"][0]; G["neg"][4] = G["h"][0]
    kw = dict(n_ent_for_c=300) if loss == "sampled_softmax" else dict(gamma=2.0, adv_temp=0.5)
    args = (scorer, loss, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"])
    lam = 0.05
    plain = orc.loss_bwd(*args, **kw)
    reg = orc.loss_bwd(*args, reg_l3=lam, **kw)
    slots = np.concatenate([G["h"], G["t"], G["neg"]])
    omega = sum(np.linalg.norm(G["ent"][s].astype(np.float64), ord=3) for s in slots)
    assert abs(reg["loss"] - (plain["loss"] + lam * omega)) < 1e-12 * max(1.0, abs(reg["loss"]))
    extra = reg["g_ent"] - plain["g_ent"]
    for i, s in enumerate(slots):
        assert np.allclose(extra[i], orc.l3_norm(G["ent"][s], lam=lam)[1], rtol=0, atol=1e-15)
    assert np.array_equal(reg["g_rel"], plain["g_rel"])          # relations are not regularised


def test_regularised_loss_matches_central_differences(orc):
    n_ent, dim = 200, 16
    G = small_graph("complex", n_ent, 4, dim, 16, 24, grid_bits=20, amp=0.5)
    G["neg"][3] = G["h"][1]
    kw = dict(n_ent_for_c=n_ent, reg_l3=0.2)
    out = orc.loss_bwd("complex", "sampled_softmax", G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"], **kw)
    dense = np.zeros((n_ent, dim)); np.add.at(dense, out["g_ent_idx"], out["g_ent"])
    step = 2.0 ** -17
    g = np.random.default_rng(11)
    rows = np.unique(out["g_ent_idx"])
    for _ in range(30):
        row, col = int(g.choice(rows)), int(g.integers(0, dim))
        keep = G["ent"][row, col]
        L = []
        for sgn in (1, -1):
            G["ent"][row, col] = np.float32(keep + sgn * step)
            L.append(orc.loss_bwd("complex", "sampled_softmax", G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"],
                                  G["neg"], want_grads=False, **kw)["loss"])
        G["ent"][row, col] = keep
        fd = (L[0] - L[1]) / (2 * step)
        assert abs(fd - dense[row, col]) < 1e-6 * np.max(np.abs(dense)), (row, col, fd, dense[row, col])
