"""Pins for the oracle's scoring functions (Table 2): hand-computed values, reductions between
scorers, the relation-property identities of Table 2, and the algebraic block forms."""
import math

import numpy as np
import pytest

import kge_synth as ks
from helpers import small_graph

F = np.float32


def test_transe_distmult_hand_computed(orc):
    h, r, t = F([1, 2, 3]), F([2, 0, -1]), F([0, 1, 4])
    # h + r - t = (3, 1, -2), squared norm 14
    assert orc.score_one("transe", h, r, None, t) == -math.sqrt(14.0)
    # 1*2*0 + 2*0*1 + 3*(-1)*4 = -12
    assert orc.score_one("distmult", h, r, None, t) == -12.0


def test_complex_hand_computed(orc):
    # h = (1+2i, 3-i), r = (0.5-i, 2), t = (2+i, -1+3i), layout [re | im]
    h, r, t = F([1, 3, 2, -1]), F([0.5, 2, -1, 0]), F([2, -1, 1, 3])
    # (1+2i)(0.5-i) = 2.5;   2.5 * conj(2+i) = 5 - 2.5i            -> Re 5
    # (3-i)*2 = 6-2i;  (6-2i) * conj(-1+3i) = (6-2i)(-1-3i) = -12 - 16i -> Re -12
    assert orc.score_one("complex", h, r, None, t) == -7.0


def test_rotate_hand_computed(orc):
    # one complex component: h = 1, phase pi/2 -> q = i
    h, r = F([1, 0]), F([math.pi / 2])
    assert abs(orc.score_one("rotate", h, r, None, F([0, 1]))) < 1e-7
    assert abs(orc.score_one("rotate", h, r, None, F([1, 0])) + math.sqrt(2.0)) < 1e-7


def test_transh_hand_computed(orc):
    # w = (0,2) -> unit normal (0,1); h_perp = (3,0), t_perp = (1,0); u = (2.5, 0.25)
    v = orc.score_one("transh", F([3, 4]), F([0.5, 0.25]), F([0, 2]), F([1, -5]))
    assert abs(v + math.sqrt(2.5 ** 2 + 0.25 ** 2)) < 1e-15


def _rand(g, d, n=1):
    return g.uniform(-1, 1, size=(n, d)).astype(np.float32)


def test_complex_with_zero_imaginary_parts_is_distmult(orc):
    g = np.random.default_rng(1)
    for _ in range(20):
        c = 8
        hre, rre, tre = _rand(g, c)[0], _rand(g, c)[0], _rand(g, c)[0]
        z = np.zeros(c, dtype=np.float32)
        cx = orc.score_one("complex", np.r_[hre, z], np.r_[rre, z], None, np.r_[tre, z])
        dm = orc.score_one("distmult", hre, rre, None, tre)
        assert abs(cx - dm) <= 1e-15 * max(1.0, abs(dm))


def test_complex_inversion_and_symmetry(orc):
    g = np.random.default_rng(2)
    c = 6
    h, r, t = _rand(g, 2 * c)[0], _rand(g, 2 * c)[0], _rand(g, 2 * c)[0]
    rbar = np.r_[r[:c], -r[c:]]
    # f(h, r, t) = f(t, conj r, h)  (inversion column of Table 2)
    assert abs(orc.score_one("complex", h, r, None, t) - orc.score_one("complex", t, rbar, None, h)) < 1e-14
    # real r -> symmetric
    rr = np.r_[r[:c], np.zeros(c, dtype=np.float32)]
    assert abs(orc.score_one("complex", h, rr, None, t) - orc.score_one("complex", t, rr, None, h)) < 1e-14
    # a generic complex r is not symmetric
    assert abs(orc.score_one("complex", h, r, None, t) - orc.score_one("complex", t, r, None, h)) > 1e-3


def test_distmult_is_symmetric(orc):
    g = np.random.default_rng(3)
    h, r, t = _rand(g, 16)[0], _rand(g, 16)[0], _rand(g, 16)[0]
    assert abs(orc.score_one("distmult", h, r, None, t) - orc.score_one("distmult", t, r, None, h)) < 1e-15


def test_rotate_reductions(orc):
    g = np.random.default_rng(4)
    c = 8
    h, t = _rand(g, 2 * c)[0], _rand(g, 2 * c)[0]
    zero = np.zeros(c, dtype=np.float32)
    # zero phases: -||h - t|| = TransE with r = 0
    a = orc.score_one("rotate", h, zero, None, t)
    b = orc.score_one("transe", h, np.zeros(2 * c, dtype=np.float32), None, t)
    assert abs(a - b) < 1e-15
    r = g.uniform(-math.pi, math.pi, c).astype(np.float32)
    # inversion: f(h, r, t) = f(t, -r, h)
    assert abs(orc.score_one("rotate", h, r, None, t) - orc.score_one("rotate", t, -r, None, h)) < 1e-13
    # rotation preserves the norm: against t = 0 the score is -||h||
    assert abs(orc.score_one("rotate", h, r, None, np.zeros(2 * c, dtype=np.float32))
               + math.sqrt(float((h.astype(np.float64) ** 2).sum()))) < 1e-13
    # phase pi (q = -h): symmetric; fp32(pi) is not exactly pi, hence 1e-6
    rpi = np.full(c, math.pi, dtype=np.float32)
    assert abs(orc.score_one("rotate", h, rpi, None, t) - orc.score_one("rotate", t, rpi, None, h)) < 1e-6
    assert abs(orc.score_one("rotate", h, rpi, None, t)
               + math.sqrt(float(((h.astype(np.float64) + t) ** 2).sum()))) < 1e-6
    # composition: r3 = r1 + r2 chains exactly: h -> a -> b with zero distance each step
    r1 = g.uniform(-1, 1, c).astype(np.float32)
    q_re = h[:c] * np.cos(r1.astype(np.float64)) - h[c:] * np.sin(r1.astype(np.float64))
    q_im = h[:c] * np.sin(r1.astype(np.float64)) + h[c:] * np.cos(r1.astype(np.float64))
    tq = np.r_[q_re, q_im].astype(np.float32)
    assert abs(orc.score_one("rotate", h, r1, None, tq)) < 1e-6


def test_transe_inversion_and_composition(orc):
    g = np.random.default_rng(5)
    h, r, t = _rand(g, 12)[0], _rand(g, 12)[0], _rand(g, 12)[0]
    assert abs(orc.score_one("transe", h, r, None, t) - orc.score_one("transe", t, -r, None, h)) < 1e-15
    # t = h + r1 + r2 (exact in fp32 on a coarse grid) scores 0 under r3 = r1 + r2
    q = 1 / 64.0
    h, r1, r2 = [np.round(_rand(g, 12)[0] / q).astype(np.float32) * np.float32(q) for _ in range(3)]
    assert orc.score_one("transe", h, r1 + r2, None, h + r1 + r2) == 0.0


def test_transh_properties(orc):
    g = np.random.default_rng(6)
    d = 10
    h, t, w = _rand(g, d)[0], _rand(g, d)[0], _rand(g, d)[0]
    zero = np.zeros(d, dtype=np.float32)
    # r = 0 -> symmetric
    assert abs(orc.score_one("transh", h, zero, w, t) - orc.score_one("transh", t, zero, w, h)) < 1e-15
    # w parallel to h - t and r = 0: the difference is projected away
    assert abs(orc.score_one("transh", h, zero, (h - t) * np.float32(3), t)) < 1e-6  # fp32 rounding of w
    # scaling w does not matter (it is normalised inside)
    r = _rand(g, d)[0]
    assert abs(orc.score_one("transh", h, r, w, t) - orc.score_one("transh", h, r, w * np.float32(4), t)) < 1e-7
    # against an independent numpy evaluation
    w64 = w.astype(np.float64) / np.linalg.norm(w.astype(np.float64))
    hp = h - (w64 @ h) * w64
    tp = t - (w64 @ t) * w64
    assert abs(orc.score_one("transh", h, r, w, t) + np.linalg.norm(hp + r - tp)) < 1e-14


def _table2():
    import os
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "table2_relation_properties.txt"))
            if l.strip() and not l.startswith("#")]
    return {w[0]: dict(zip("S AS I C".split(), (int(x) for x in w[1:5]))) for w in rows}


@pytest.mark.parametrize("scorer", ["transe", "transh", "rotate", "distmult", "complex"])
def test_check_marks_of_table_2_have_witnesses(orc, scorer):
    """Every check mark of Table 2 (tests/golden/table2_relation_properties.txt) is realised by the oracle's scorer with an
    explicit relation: S - a non-zero r with f(h,r,t) = f(t,r,h) for all h, t; AS - an r with f(h,r,t) != f(t,r,h); I - an
    r' with f(h,r,t) = f(t,r',h); C - r3 built from r1, r2 such that f(h,r1,m) = f(m,r2,t) = 0 implies f(h,r3,t) = 0.  Two
    crosses are facts of the formulas and are checked too: TransE is symmetric for no r != 0, DistMult antisymmetric for none."""
    marks = _table2()[scorer]
    g = np.random.default_rng(11)
    d, c = 12, 6
    q = np.float32(1 / 64.0)
    grid = lambda n: (np.round(_rand(g, n)[0] / q) * q).astype(np.float32)      # sums and differences exact in fp32
    h, t = grid(d), grid(d)
    w = _rand(g, d)[0] if scorer == "transh" else None
    f = lambda hh, rr, tt: orc.score_one(scorer, hh, rr, w, tt)
    k = c if scorer == "rotate" else d
    generic = grid(k) + q                                                        # no zero entry, no multiple of pi
    if marks["S"]:
        r_sym = {"transh": np.zeros(d, F), "rotate": np.array([0, math.pi] * 3, F), "distmult": generic,
                 "complex": np.r_[generic[:c], np.zeros(c, F)]}[scorer]
        assert abs(f(h, r_sym, t) - f(t, r_sym, h)) < 1e-6 * max(1.0, abs(f(h, r_sym, t)))
        if scorer != "transh":
            assert np.any(r_sym != 0)
    else:
        assert scorer == "transe" and abs(f(h, generic, t) - f(t, generic, h)) > 1e-3
    if marks["AS"]:
        assert abs(f(h, generic, t) - f(t, generic, h)) > 1e-3
    else:
        assert scorer == "distmult" and f(h, generic, t) == f(t, generic, h)
    if marks["I"]:
        r_inv = {"transe": -generic, "rotate": -generic, "complex": np.r_[generic[:c], -generic[c:]]}[scorer]
        assert abs(f(h, generic, t) - f(t, r_inv, h)) < 1e-6 * max(1.0, abs(f(h, generic, t)))
    if marks["C"]:
        r1, r2 = grid(k), grid(k)
        if scorer == "transe":
            m, t3 = h + r1, h + r1 + r2
            assert f(h, r1, m) == 0.0 and f(m, r2, t3) == 0.0 and f(h, r1 + r2, t3) == 0.0
        else:                                                                    # rotate: the phases add
            rot = lambda x, ph: np.r_[x[:c] * np.cos(ph) - x[c:] * np.sin(ph), x[:c] * np.sin(ph) + x[c:] * np.cos(ph)].astype(np.float32)
            m = rot(h.astype(np.float64), r1.astype(np.float64))
            t3 = rot(m.astype(np.float64), r2.astype(np.float64))
            assert abs(f(h, r1, m)) < 1e-6 and abs(f(m, r2, t3)) < 1e-6 and abs(f(h, r1 + r2, t3)) < 1e-6


@pytest.mark.parametrize("scorer", ["transe", "transh", "rotate", "distmult", "complex"])
def test_block_forms_equal_direct_loops(orc, scorer):
    """The shared-negative block as (query build) + (contraction against the negative rows),
    evaluated in fp64 numpy, equals the oracle's triple-by-triple loops."""
    G = small_graph(scorer, n_ent=300, n_rel=7, dim=16, B=9, N=13)
    pos, neg = orc.score_batch(scorer, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"])
    E = G["ent"].astype(np.float64)
    R = G["rel"].astype(np.float64)
    H, Tn, Tp, Rr = E[G["h"]], E[G["neg"]], E[G["t"]], R[G["r"]]
    c = 8
    if scorer == "distmult":
        Q = H * Rr
        blk, p = Q @ Tn.T, (Q * Tp).sum(1)
    elif scorer == "complex":
        Q = np.c_[H[:, :c] * Rr[:, :c] - H[:, c:] * Rr[:, c:], H[:, :c] * Rr[:, c:] + H[:, c:] * Rr[:, :c]]
        blk, p = Q @ Tn.T, (Q * Tp).sum(1)
    elif scorer in ("transe", "rotate"):
        if scorer == "transe":
            Q = H + Rr
        else:
            Q = np.c_[H[:, :c] * np.cos(Rr) - H[:, c:] * np.sin(Rr), H[:, :c] * np.sin(Rr) + H[:, c:] * np.cos(Rr)]
        d2 = (Q ** 2).sum(1)[:, None] + (Tn ** 2).sum(1)[None, :] - 2 * Q @ Tn.T
        blk, p = -np.sqrt(d2), -np.sqrt(((Q - Tp) ** 2).sum(1))
    else:
        W = G["relw"].astype(np.float64)[G["r"]]
        W = W / np.linalg.norm(W, axis=1, keepdims=True)
        Q = H - (W * H).sum(1)[:, None] * W + Rr
        A = W @ Tn.T
        cq = (W * Q).sum(1)
        d2 = (Q ** 2).sum(1)[:, None] + (Tn ** 2).sum(1)[None, :] - 2 * Q @ Tn.T + 2 * A * cq[:, None] - A ** 2
        blk = -np.sqrt(d2)
        Ap = (W * Tp).sum(1)
        p = -np.sqrt(((Q - Tp + Ap[:, None] * W) ** 2).sum(1))
    assert np.max(np.abs(blk - neg)) < 1e-12
    assert np.max(np.abs(p - pos)) < 1e-12


def test_score_batch_matches_score_one(orc):
    G = small_graph("complex", n_ent=50, n_rel=3, dim=8, B=5, N=4)
    pos, neg = orc.score_batch("complex", G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"])
    for b in range(5):
        assert pos[b] == orc.score_one("complex", G["ent"][G["h"][b]], G["rel"][G["r"][b]], None, G["ent"][G["t"][b]])
        for n in range(4):
            assert neg[b, n] == orc.score_one("complex", G["ent"][G["h"][b]], G["rel"][G["r"][b]], None,
                                              G["ent"][G["neg"][n]])
