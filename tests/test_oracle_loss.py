"""Pins for the oracle's losses (Section 3.1, "Loss Functions") and their score-derivatives."""
import math

import numpy as np
import torch

from helpers import small_graph


def test_sampled_softmax_equal_scores_gives_log_num_entities(orc):
    # all N+1 scores equal: L = log(1 + N * (|E|-1)/N) = log |E|
    for n_ent, N in [(1000, 64), (91230610, 1024), (17, 16)]:
        L, dfp, ds = orc.loss_one("sampled_softmax", 0.0, 0.0, n_ent, 0.37, np.full(N, 0.37))
        assert abs(L - math.log(n_ent)) < 1e-12
        # probabilities: positive 1/|E|, each negative ((|E|-1)/N)/|E|
        assert abs(dfp - (1.0 / n_ent - 1.0)) < 1e-12
        assert np.allclose(ds, (n_ent - 1) / N / n_ent, rtol=0, atol=1e-12)


def test_sampled_softmax_shift_invariance_and_gradient_sum(orc):
    g = np.random.default_rng(0)
    s = g.normal(size=50) * 3
    L0, dfp0, ds0 = orc.loss_one("sampled_softmax", 0.0, 0.0, 10**6, 1.3, s)
    L1, dfp1, ds1 = orc.loss_one("sampled_softmax", 0.0, 0.0, 10**6, 1.3 + 7.5, s + 7.5)
    assert abs(L0 - L1) < 1e-12 and abs(dfp0 - dfp1) < 1e-13 and np.max(np.abs(ds0 - ds1)) < 1e-13
    assert abs(dfp0 + ds0.sum()) < 1e-13          # gradients of a shift-invariant function sum to 0
    # large scores do not overflow
    L2, _, ds2 = orc.loss_one("sampled_softmax", 0.0, 0.0, 10**6, 900.0, s + 1000.0)
    assert np.isfinite(L2) and np.all(np.isfinite(ds2))


def test_sampled_softmax_with_all_entities_is_textbook_cross_entropy(orc):
    # N = |E| - 1  ->  c = 0  ->  plain softmax cross-entropy with the positive as class 0
    g = np.random.default_rng(1)
    N = 40
    fp, s = 0.3, g.normal(size=N)
    L, dfp, ds = orc.loss_one("sampled_softmax", 0.0, 0.0, N + 1, fp, s)
    logits = torch.tensor(np.r_[fp, s], dtype=torch.float64, requires_grad=True)
    ref = torch.nn.functional.cross_entropy(logits[None, :], torch.tensor([0]))
    ref.backward()
    assert abs(L - ref.item()) < 1e-13
    assert np.max(np.abs(np.r_[dfp, ds] - logits.grad.numpy())) < 1e-14


def test_logsigmoid_closed_forms(orc):
    # f = 0, gamma = 0, a = 0: L = log 2 + sum (1/N) log 2 = 2 log 2
    L, dfp, ds = orc.loss_one("logsigmoid", 0.0, 0.0, 0, 0.0, np.zeros(10))
    assert abs(L - 2 * math.log(2)) < 1e-15
    assert abs(dfp + 0.5) < 1e-15 and np.allclose(ds, 0.05, rtol=0, atol=1e-16)


def test_logsigmoid_against_torch(orc):
    g = np.random.default_rng(2)
    for gamma, a in [(0.0, 0.0), (6.0, 0.0), (10.0, 1.0), (2.0, 0.5)]:
        N = 33
        fp, s = float(g.normal() * 3 - 4), g.normal(size=N) * 4 - 6
        L, dfp, ds = orc.loss_one("logsigmoid", gamma, a, 0, fp, s)
        tfp = torch.tensor(fp, dtype=torch.float64, requires_grad=True)
        ts = torch.tensor(s, dtype=torch.float64, requires_grad=True)
        w = torch.softmax(a * ts, dim=0).detach()
        ref = -torch.nn.functional.logsigmoid(gamma + tfp) - (w * torch.nn.functional.logsigmoid(-gamma - ts)).sum()
        ref.backward()
        assert abs(w.sum().item() - 1) < 1e-14
        assert abs(L - ref.item()) < 1e-12
        assert abs(dfp - tfp.grad.item()) < 1e-14
        assert np.max(np.abs(ds - ts.grad.numpy())) < 1e-14
        if a == 0.0:
            assert np.allclose(ds / (1 / (1 + np.exp(-(gamma + s)))), 1.0 / N, rtol=1e-12)


def test_logsigmoid_extreme_arguments_are_finite(orc):
    L, dfp, ds = orc.loss_one("logsigmoid", 0.0, 1.0, 0, -800.0, np.array([700.0, -700.0, 0.0]))
    assert np.isfinite(L) and np.isfinite(dfp) and np.all(np.isfinite(ds))
    assert abs(L - (800.0 + 700.0)) < 1e-9      # -log sigma(-800) = 800; weight ~1 on the 700 score


def test_batch_loss_is_scaled_sum_of_per_triple_losses(orc):
    G = small_graph("transe", n_ent=200, n_rel=5, dim=8, B=12, N=10)
    pos, neg = orc.score_batch("transe", G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"])
    for loss, kw in [("logsigmoid", dict(gamma=3.0, adv_temp=0.7)), ("sampled_softmax", dict(n_ent_for_c=200))]:
        out = orc.loss_bwd("transe", loss, G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"],
                           want_grads=False, **kw)
        per = [orc.loss_one(loss, kw.get("gamma", 0.0), kw.get("adv_temp", 0.0), kw.get("n_ent_for_c", 0),
                            pos[b], neg[b])[0] for b in range(12)]
        assert np.max(np.abs(out["per_triple"] - per)) < 1e-14
        assert abs(out["loss"] - sum(per) / 12) < 1e-14
        out2 = orc.loss_bwd("transe", loss, G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"],
                            want_grads=False, loss_scale=0.25, **kw)
        assert abs(out2["loss"] - 0.25 * sum(per)) < 1e-13


def test_no_negatives(orc):
    G = small_graph("distmult", n_ent=50, n_rel=3, dim=8, B=4, N=0)
    out = orc.loss_bwd("distmult", "logsigmoid", G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"])
    pos, _ = orc.score_batch("distmult", G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"])
    assert abs(out["loss"] - np.mean(np.log1p(np.exp(-pos)))) < 1e-14
    assert out["g_ent"].shape == (8, 8)
