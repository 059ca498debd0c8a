"""Finite-difference pin of the oracle's backward pass on a 1k-entity graph: every scorer and both
losses, including rows that occur several times in the micro-batch (the derivative with respect to
a table row is the SUM of the per-slot gradients that target it)."""
import numpy as np
import pytest

from helpers import small_graph

STEP = 2.0 ** -17     # exactly representable: table values sit on a 2^-20 grid


def _loss(orc, scorer, loss, G, kw):
    return orc.loss_bwd(scorer, loss, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"],
                        want_grads=False, **kw)["loss"]


@pytest.mark.parametrize("scorer", ["transe", "transh", "rotate", "distmult", "complex"])
@pytest.mark.parametrize("loss", ["logsigmoid", "sampled_softmax"])
def test_gradients_match_central_differences(orc, scorer, loss):
    n_ent, n_rel, dim, B, N = 1000, 10, 32, 64, 64
    amp = 0.5 if scorer in ("distmult", "complex") else 0.1   # larger values: non-trivial softmax weights
    G = small_graph(scorer, n_ent, n_rel, dim, B, N, grid_bits=20, amp=amp)
    # force duplicates: a head that is also a tail and a negative, a repeated negative
    G["t"][3] = G["h"][0]; G["neg"][5] = G["h"][0]; G["neg"][6] = G["neg"][7]; G["h"][9] = G["h"][0]
    G["r"][9] = G["r"][0]
    # adv_temp = 0 here: with a > 0 the weights are held constant (StopGrad), so the loss is not
    # the function whose derivative is taken; that case has its own test below.
    kw = dict(gamma=4.0, adv_temp=0.0) if loss == "logsigmoid" else dict(n_ent_for_c=n_ent)
    if scorer in ("distmult", "complex") and loss == "logsigmoid":
        kw["gamma"] = 0.0
    out = orc.loss_bwd(scorer, loss, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"], **kw)
    k = G["rel"].shape[1]
    dense_ent = np.zeros((n_ent, dim)); np.add.at(dense_ent, out["g_ent_idx"], out["g_ent"])
    dense_rel = np.zeros((n_rel, k)); np.add.at(dense_rel, out["g_rel_idx"], out["g_rel"])
    tables = [("ent", dense_ent)]
    tables.append(("rel", dense_rel))
    if scorer == "transh":
        dense_w = np.zeros((n_rel, dim)); np.add.at(dense_w, out["g_rel_idx"], out["g_relw"])
        tables.append(("relw", dense_w))
    g = np.random.default_rng(7)
    worst = 0.0
    for name, dense in tables:
        rows = np.unique(out["g_ent_idx"] if name == "ent" else out["g_rel_idx"])
        picks = [(int(G["h"][0]), j) for j in (0, dim // 2, dense.shape[1] - 1)] if name == "ent" else []
        picks += [(int(G["neg"][6]), 1)] if name == "ent" else []
        for _ in range(40 if name == "ent" else 12):
            picks.append((int(g.choice(rows)), int(g.integers(0, dense.shape[1]))))
        scale = np.max(np.abs(dense))
        for (row, col) in picks:
            keep = G[name][row, col]
            G[name][row, col] = np.float32(keep + STEP); lp = _loss(orc, scorer, loss, G, kw)
            G[name][row, col] = np.float32(keep - STEP); lm = _loss(orc, scorer, loss, G, kw)
            G[name][row, col] = keep
            fd = (lp - lm) / (2 * STEP)
            err = abs(fd - dense[row, col]) / scale
            worst = max(worst, err)
            assert err < 1e-6, (name, row, col, fd, dense[row, col])
    # an untouched row has zero gradient and zero finite difference
    untouched = np.setdiff1d(np.arange(n_ent), out["g_ent_idx"])[0]
    assert np.all(dense_ent[untouched] == 0)


def test_gradient_is_zero_at_zero_distance(orc):
    # sub-gradient 0 at the kink of the norm: t = h + r exactly
    ent = np.array([[0.25, 0.5], [0.75, 0.25], [0.1, 0.2]], dtype=np.float32)
    rel = np.array([[0.5, -0.25]], dtype=np.float32)
    out = orc.loss_bwd("transe", "logsigmoid", ent, rel, None, [0], [0], [1], np.zeros(0, np.int32), gamma=1.0)
    assert np.all(out["g_ent"] == 0) and np.all(out["g_rel"] == 0)


def test_self_adversarial_weights_are_held_constant(orc):
    """With a > 0 the gradient is that of the surrogate in which the softmax weights are frozen at
    their current values (StopGrad in the log-sigmoid loss)."""
    n_ent, n_rel, dim, B, N = 300, 5, 16, 16, 24
    gamma, a = 3.0, 0.8
    G = small_graph("transe", n_ent, n_rel, dim, B, N, grid_bits=20, amp=0.3)
    out = orc.loss_bwd("transe", "logsigmoid", G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"],
                       gamma=gamma, adv_temp=a)
    dense = np.zeros((n_ent, dim)); np.add.at(dense, out["g_ent_idx"], out["g_ent"])
    _, s0 = orc.score_batch("transe", G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"])
    w = np.exp(a * s0 - (a * s0).max(1, keepdims=True)); w /= w.sum(1, keepdims=True)

    def logsig(x):
        return np.minimum(x, 0) - np.log1p(np.exp(-np.abs(x)))

    def surrogate():
        p, s = orc.score_batch("transe", G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"])
        return float(np.mean(-logsig(gamma + p) - (w * logsig(-gamma - s)).sum(1)))

    g = np.random.default_rng(3)
    rows = np.unique(out["g_ent_idx"])
    for _ in range(30):
        row, col = int(g.choice(rows)), int(g.integers(0, dim))
        keep = G["ent"][row, col]
        G["ent"][row, col] = np.float32(keep + STEP); lp = surrogate()
        G["ent"][row, col] = np.float32(keep - STEP); lm = surrogate()
        G["ent"][row, col] = keep
        assert abs((lp - lm) / (2 * STEP) - dense[row, col]) / np.max(np.abs(dense)) < 1e-6
