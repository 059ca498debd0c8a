"""Pins for the 1-norm variants of the distance scorers (Table 2, p = 1): hand-computed values, numpy's
1-norm on independently built difference vectors, norm-equivalence bounds against the 2-norm scorers,
reductions between scorers, homogeneity, the sub-gradient at the kink and central finite differences."""
import math

import numpy as np
import pytest

from helpers import small_graph

F = np.float32
STEP = 2.0 ** -17


def test_hand_computed(orc):
    # h + r - t = (1.5, -2, 0.25): 1-norm 3.75
    assert orc.score_one("transe_l1", F([1, 2, 0.5]), F([0.5, -1, 0]), None, F([0, 3, 0.25])) == -3.75
    # one complex coordinate, h = 1, phase pi/2 -> q = i; t = 1: x = -1 + i -> |Re| + |Im| = 2
    assert abs(orc.score_one("rotate_l1", F([1, 0]), F([math.pi / 2]), None, F([1, 0])) + 2.0) < 1e-7
    # w = (0,2) -> unit normal (0,1); h_perp = (3,0), t_perp = (1,0); u = (2.5, 0.25)
    assert abs(orc.score_one("transh_l1", F([3, 4]), F([0.5, 0.25]), F([0, 2]), F([1, -5])) + 2.75) < 1e-15


def _diff_vector(scorer, h, r, w, t):
    """The vector whose norm the scorer takes, built with numpy (complex arithmetic for RotatE)."""
    h, r, t = h.astype(np.float64), r.astype(np.float64), t.astype(np.float64)
    if scorer == "transe":
        return h + r - t
    if scorer == "rotate":
        c = h.size // 2
        x = (h[:c] + 1j * h[c:]) * np.exp(1j * r) - (t[:c] + 1j * t[c:])
        return np.concatenate([x.real, x.imag])
    wh = w.astype(np.float64) / np.linalg.norm(w.astype(np.float64))
    return (h - wh * (wh @ h)) + r - (t - wh * (wh @ t))


@pytest.mark.parametrize("scorer", ["transe", "rotate", "transh"])
def test_scores_equal_library_norms(orc, scorer):
    g = np.random.default_rng(11)
    d = 24
    for _ in range(20):
        h, t = g.uniform(-1, 1, d).astype(F), g.uniform(-1, 1, d).astype(F)
        r = g.uniform(-3, 3, d // 2 if scorer == "rotate" else d).astype(F)
        w = g.uniform(-1, 1, d).astype(F) if scorer == "transh" else None
        x = _diff_vector(scorer, h, r, w, t)
        s1, s2 = orc.score_one(scorer + "_l1", h, r, w, t), orc.score_one(scorer, h, r, w, t)
        assert abs(s1 + np.linalg.norm(x, ord=1)) < 1e-12
        assert abs(s2 + np.linalg.norm(x, ord=2)) < 1e-12
        # ||x||_2 <= ||x||_1 <= sqrt(d) ||x||_2
        assert -s2 <= -s1 * (1 + 1e-15) and -s1 <= math.sqrt(d) * -s2 * (1 + 1e-15)


def test_reductions_between_scorers(orc):
    g = np.random.default_rng(12)
    d = 16
    h, t, r = (g.uniform(-1, 1, d).astype(F) for _ in range(3))
    zero_ph = np.zeros(d // 2, F)
    # RotatE with zero phases = TransE with r = 0
    assert orc.score_one("rotate_l1", h, zero_ph, None, t) == orc.score_one("transe_l1", h, np.zeros(d, F), None, t)
    # TransH with h, t, r orthogonal to the normal = TransE
    w = np.zeros(d, F); w[0] = 3.0
    h2, t2, r2 = h.copy(), t.copy(), r.copy()
    h2[0] = t2[0] = r2[0] = 0.0
    assert abs(orc.score_one("transh_l1", h2, r2, w, t2) - orc.score_one("transe_l1", h2, r2, None, t2)) < 1e-15
    # one coordinate: both norms coincide
    assert orc.score_one("transe_l1", F([0.3]), F([0.4]), None, F([-0.5])) == orc.score_one("transe", F([0.3]), F([0.4]), None, F([-0.5]))
    # the score is absolutely homogeneous of degree 1 in (h, r, t) for TransE
    s = orc.score_one("transe_l1", h, r, None, t)
    assert abs(orc.score_one("transe_l1", F(2) * h, F(2) * r, None, F(2) * t) - 2 * s) < 1e-12


@pytest.mark.parametrize("scorer", ["transe_l1", "transh_l1", "rotate_l1"])
@pytest.mark.parametrize("loss", ["logsigmoid", "sampled_softmax"])
def test_gradients_match_central_differences(orc, scorer, loss):
    n_ent, n_rel, dim, B, N = 400, 6, 16, 24, 24
    G = small_graph(scorer, n_ent, n_rel, dim, B, N, grid_bits=20, amp=0.1)
    G["t"][3] = G["h"][0]; G["neg"][5] = G["h"][0]; G["neg"][6] = G["neg"][7]; G["h"][9] = G["h"][0]
    G["r"][9] = G["r"][0]
    kw = dict(gamma=2.0, adv_temp=0.0) if loss == "logsigmoid" else dict(n_ent_for_c=n_ent)

    def f():
        return orc.loss_bwd(scorer, loss, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"],
                            want_grads=False, **kw)["loss"]
    out = orc.loss_bwd(scorer, loss, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"], **kw)
    k = G["rel"].shape[1]
    dense = {"ent": np.zeros((n_ent, dim)), "rel": np.zeros((n_rel, k))}
    np.add.at(dense["ent"], out["g_ent_idx"], out["g_ent"]); np.add.at(dense["rel"], out["g_rel_idx"], out["g_rel"])
    if scorer == "transh_l1":
        dense["relw"] = np.zeros((n_rel, dim)); np.add.at(dense["relw"], out["g_rel_idx"], out["g_relw"])
    g = np.random.default_rng(5)
    checked = 0
    for name, dn in dense.items():
        rows = np.unique(out["g_ent_idx"] if name == "ent" else out["g_rel_idx"])
        scale = np.max(np.abs(dn))
        for _ in range(30 if name == "ent" else 10):
            row, col = int(g.choice(rows)), int(g.integers(0, dn.shape[1]))
            keep = G[name][row, col]
            vals = []
            for delta in (STEP, -STEP, 2 * STEP, -2 * STEP):
                G[name][row, col] = F(keep + delta); vals.append(f())
            G[name][row, col] = keep
            fd1, fd2 = (vals[0] - vals[1]) / (2 * STEP), (vals[2] - vals[3]) / (4 * STEP)
            # the loss is piecewise smooth: a kink of some |x_j| inside the stencil shows as a disagreement of
            # the two difference quotients; such points say nothing about the gradient and are skipped
            if abs(fd1 - fd2) > 1e-7 * scale:
                continue
            checked += 1
            assert abs(fd1 - dn[row, col]) / scale < 1e-6, (name, row, col, fd1, dn[row, col])
    assert checked >= 30


def test_subgradient_at_the_kink_is_zero(orc):
    # coordinate 0 of h + r - t is exactly zero, coordinate 1 is not
    ent = np.array([[0.25, 0.5], [0.75, 0.25]], dtype=F)
    rel = np.array([[0.5, -0.5]], dtype=F)
    out = orc.loss_bwd("transe_l1", "logsigmoid", ent, rel, None, [0], [0], [1], np.zeros(0, np.int32), gamma=1.0,
                       loss_scale=1.0)
    # L = softplus(-(gamma + f)), f = -0.25: dL/df = -sigma(-(gamma + f)); df/dx = -sign(x), x = (0, -0.25)
    gp = -1.0 / (1.0 + math.exp(1.0 - 0.25))
    assert out["g_ent"][0, 0] == 0 and out["g_rel"][0, 0] == 0 and out["g_ent"][1, 0] == 0
    assert abs(out["g_ent"][0, 1] - gp) < 1e-15 and abs(out["g_ent"][1, 1] + gp) < 1e-15


def test_topk_orders_by_the_one_norm(orc):
    g = np.random.default_rng(3)
    n_ent, d = 300, 8
    ent = g.uniform(-1, 1, (n_ent, d)).astype(F); rel = g.uniform(-1, 1, (4, d)).astype(F)
    h, r = np.array([5, 17], np.int32), np.array([1, 3], np.int32)
    idx, score, rank = orc.topk("transe_l1", ent, rel, None, h, r, 0, n_ent, 10, true_t=np.array([7, 9], np.int32))
    for q in range(2):
        key = np.abs(ent[h[q]].astype(np.float64) + rel[r[q]] - ent.astype(np.float64)).sum(axis=1)
        order = np.lexsort((np.arange(n_ent), key))
        assert np.array_equal(idx[q], order[:10])
        assert np.allclose(score[q], -key[order[:10]], rtol=0, atol=1e-12)
        assert rank[q] == 1 + int(np.where(order == [7, 9][q])[0][0])


def test_sign_flip_justification_accepts_only_coordinates_near_zero(orc):
    """The helper that the GPU tests use to accept a flipped sign: a deviation of 2 |dL/dS| at a column whose coordinate
    lies within rounding of zero passes; the same deviation anywhere else, or a larger one at that column, fails."""
    from helpers import l1_sign_flips_justified, small_graph
    G = small_graph("transe", 300, 4, 16, 12, 20, amp=0.4)
    b, n, j = 5, 7, 3
    # put coordinate j of pair (b, n) a hair above zero: h + r - t = 1e-9-ish (well inside the band, not a tie)
    G["ent"][G["neg"][n], j] = np.float32(G["ent"][G["h"][b], j] + G["rel"][G["r"][b], j]) - np.float32(2e-8)
    kw = dict(n_ent_for_c=300)
    args = (G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"])
    ref = orc.loss_bwd("transe_l1", "sampled_softmax", *args, **kw)
    x = (np.float64(G["ent"][G["h"][b], j]) + np.float64(G["rel"][G["r"][b], j])) - np.float64(G["ent"][G["neg"][n], j])
    assert 0 < abs(x) < 1e-7
    # dL/dS(b, n) from the head's gradient: flipping sign(x) moves g_head[b, j] and g_neg[n, j] by 2 dL/dS each
    pos, S = orc.score_batch("transe_l1", *args)
    c = np.log(299 / 20)
    z = np.concatenate([pos[:, None], S + c], axis=1); p = np.exp(z - z.max(axis=1, keepdims=True)); p /= p.sum(axis=1, keepdims=True)
    gbn = p[b, 1 + n] / 12
    same = lambda: {"g_ent": ref["g_ent"].copy(), "g_rel": ref["g_rel"].copy()}
    assert l1_sign_flips_justified(orc, "transe", "sampled_softmax", *args, kw, same(), ref, 1e-5) == 0
    got = same()
    sgn = np.sign(x)
    got["g_ent"][b, j] += 2 * sgn * gbn; got["g_rel"][b, j] += 2 * sgn * gbn; got["g_ent"][2 * 12 + n, j] -= 2 * sgn * gbn
    assert l1_sign_flips_justified(orc, "transe", "sampled_softmax", *args, kw, got, ref, 1e-5) == 3
    bad = same(); bad["g_ent"][b, j + 1] += 2 * gbn                       # right size, wrong column
    with pytest.raises(AssertionError):
        l1_sign_flips_justified(orc, "transe", "sampled_softmax", *args, kw, bad, ref, 1e-5)
    bad = same(); bad["g_ent"][b, j] += 6 * sgn * gbn                     # right column, three times the allowance
    with pytest.raises(AssertionError):
        l1_sign_flips_justified(orc, "transe", "sampled_softmax", *args, kw, bad, ref, 1e-5)
