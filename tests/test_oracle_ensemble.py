"""Pins for the power-rank ensemble (Section 3.2, eq. (ensemble)): a hand-computed case, invariants, and a dense
brute-force evaluation over ALL entities with library sorting (the oracle only ever looks at listed entities)."""
import numpy as np
import pytest


def _lists(g, M, Q, K, n_ent, pool):
    """M lists of K distinct entities per query, drawn from a per-query pool so that the lists overlap."""
    out = np.empty((M, Q, K), dtype=np.int32)
    for q in range(Q):
        cand = g.choice(n_ent, size=pool, replace=False)
        for m in range(M):
            out[m, q] = g.permutation(cand)[:K]
    return out


def _dense(lists, p, n_ent, K_out):
    M, Q, K = lists.shape
    idx = np.empty((Q, K_out), dtype=np.int64); sc = np.empty((Q, K_out))
    for q in range(Q):
        rank = np.full((M, n_ent), K + 1, dtype=np.int64)
        for m in range(M):
            ok = lists[m, q] >= 0
            rank[m, lists[m, q][ok][::-1]] = (np.arange(K)[ok] + 1)[::-1]       # first occurrence wins
        term = np.where(rank <= K, -np.sign(p) * rank.astype(np.float64) ** p, -(p > 0) * float(K + 1) ** p)
        s = np.zeros(n_ent)
        for m in range(M):                                                         # model order, as the definition sums
            s = s + term[m]
        order = np.lexsort((np.arange(n_ent), -s))[:K_out]
        idx[q], sc[q] = order, s[order]
    return idx, sc


def test_hand_computed(orc):
    # two models, K = 3.  p = 1: s = -(sum of ranks), absent counts K + 1 = 4
    lists = np.array([[[5, 7, 9]], [[7, 2, 5]]], dtype=np.int32)
    idx, sc = orc.ensemble(lists, 1.0, K_out=4)
    # 5: -(1 + 3) = -4; 7: -(2 + 1) = -3; 9: -(3 + 4) = -7; 2: -(4 + 2) = -6
    assert idx.tolist() == [[7, 5, 2, 9]] and sc.tolist() == [[-3.0, -4.0, -6.0, -7.0]]
    # p = -1 (reciprocal ranks, absent counts 0): 5: 1 + 1/3; 7: 1/2 + 1; 9: 1/3; 2: 1/2
    idx, sc = orc.ensemble(lists, -1.0, K_out=5)
    assert idx.tolist() == [[7, 5, 2, 9, -1]]
    assert np.allclose(sc[0, :4], [1.5, 1 + 1 / 3, 0.5, 1 / 3], rtol=0, atol=1e-15) and sc[0, 4] == -np.inf


@pytest.mark.parametrize("p", [1.0, 2.0, -1.0, -0.5, 0.3])
def test_matches_dense_evaluation_over_all_entities(orc, p):
    g = np.random.default_rng(21)
    n_ent, M, Q, K = 500, 6, 25, 20
    lists = _lists(g, M, Q, K, n_ent, 45)
    lists[2, 3, 15:] = -1                               # a short list
    lists[4, 7, 9] = lists[4, 7, 2]                     # a repeated entity: its first position counts
    idx, sc = orc.ensemble(lists, p, K_out=10)
    ridx, rsc = _dense(lists, p, n_ent, 10)
    assert np.array_equal(idx, ridx)
    assert np.allclose(sc, rsc, rtol=1e-14, atol=0)


def test_invariants(orc):
    g = np.random.default_rng(22)
    lists = _lists(g, 5, 12, 16, 300, 30)
    for p in (1.0, -1.0, 2.0):
        # one model: the list itself
        idx, _ = orc.ensemble(lists[:1], p, K_out=10)
        assert np.array_equal(idx, lists[0, :, :10])
        # identical models: the common order
        idx, _ = orc.ensemble(np.repeat(lists[:1], 4, axis=0), p, K_out=10)
        assert np.array_equal(idx, lists[0, :, :10])
    # integer powers give exactly representable terms: the order of the models cannot matter
    a, sa = orc.ensemble(lists, 2.0)
    b, sb = orc.ensemble(lists[::-1], 2.0)
    assert np.array_equal(a, b) and np.array_equal(sa, sb)
    # promoting an entity to the top of one list can only move it up
    q, m = 4, 2
    base, _ = orc.ensemble(lists, -1.0, K_out=16)
    t = int(base[q, 9])
    mod = lists.copy()
    row = [x for x in mod[m, q] if x != t]
    mod[m, q] = np.array([t] + row[:15], dtype=np.int32)
    after, _ = orc.ensemble(mod, -1.0, K_out=16)
    assert int(np.where(after[q] == t)[0][0]) <= 9
