"""Pins for the oracle's full ranking (Section 3.2, "Inference") and partition bucketing."""
import numpy as np
import pytest

import kge_synth as ks
from helpers import small_graph


def _brute(orc, scorer, G, q_h, q_r, lo, hi, K, true_t):
    """Full sort of all candidate scores by (score desc, index asc)."""
    cand = np.arange(lo, hi, dtype=np.int32)
    idxs, scs, ranks = [], [], []
    for q in range(len(q_h)):
        s = np.array([orc.score_one(scorer, G["ent"][q_h[q]], G["rel"][q_r[q]],
                                    None if G["relw"] is None else G["relw"][q_r[q]], G["ent"][c]) for c in cand])
        order = np.lexsort((cand, -s))
        idxs.append(cand[order][:K]); scs.append(s[order][:K])
        st = orc.score_one(scorer, G["ent"][q_h[q]], G["rel"][q_r[q]],
                           None if G["relw"] is None else G["relw"][q_r[q]], G["ent"][true_t[q]])
        ranks.append(1 + int(np.sum(s > st)) + int(np.sum((s == st) & (cand < true_t[q]))))
    return np.array(idxs), np.array(scs), np.array(ranks)


@pytest.mark.parametrize("scorer", ["distmult", "transe", "complex", "rotate", "transh"])
def test_topk_equals_full_sort(orc, scorer):
    G = small_graph(scorer, n_ent=1000, n_rel=10, dim=32, B=16, N=0, normal=True)
    true_t = G["t"]
    idx, sc, rank = orc.topk(scorer, G["ent"], G["rel"], G["relw"], G["h"], G["r"], 0, 1000, 100, true_t)
    bi, bs, br = _brute(orc, scorer, G, G["h"], G["r"], 0, 1000, 100, true_t)
    assert np.array_equal(idx, bi) and np.array_equal(rank, br)
    assert np.max(np.abs(sc - bs)) < 1e-12
    assert np.all(np.diff(sc, axis=1) <= 0)                       # best first
    for q in range(16):                                           # rank agrees with list position
        pos = np.where(idx[q] == true_t[q])[0]
        if rank[q] <= 100:
            assert len(pos) == 1 and pos[0] + 1 == rank[q]
        else:
            assert len(pos) == 0


def test_ties_go_to_the_lower_index_and_sub_ranges(orc):
    G = small_graph("distmult", n_ent=200, n_rel=4, dim=8, B=6, N=0)
    # exact ties: copies of rows at scattered positions
    for dst, src in [(150, 3), (77, 3), (10, 120), (199, 120), (5, 6)]:
        G["ent"][dst] = G["ent"][src]
    true_t = np.array([150, 77, 3, 199, 10, 6], dtype=np.int32)
    G["h"][1] = G["h"][2] = G["h"][0]; G["r"][1] = G["r"][2] = G["r"][0]   # one query, three tied true tails
    for (lo, hi, K) in [(0, 200, 50), (2, 180, 200), (100, 101, 3)]:
        idx, sc, rank = orc.topk("distmult", G["ent"], G["rel"], None, G["h"], G["r"], lo, hi, K, true_t)
        n = hi - lo
        bi, bs, br = _brute(orc, "distmult", G, G["h"], G["r"], lo, hi, min(K, n), true_t)
        assert np.array_equal(idx[:, :min(K, n)], bi) and np.array_equal(rank, br)
        if K > n:                                               # padding past the candidate count
            assert np.all(idx[:, n:] == -1) and np.all(np.isneginf(sc[:, n:]))
    idx, _, rank = orc.topk("distmult", G["ent"], G["rel"], None, G["h"], G["r"], 0, 200, 200, true_t)
    for q in range(6):
        row = idx[q].tolist()
        assert row.index(3) < row.index(77) < row.index(150)   # identical rows: ascending index
        assert row.index(10) < row.index(120) < row.index(199)
    assert rank[0] == rank[2] + 2 and rank[1] == rank[2] + 1


@pytest.mark.parametrize("scorer", ["distmult", "transe", "rotate"])
def test_band_count_equals_a_direct_count(orc, scorer):
    """topk_band: the ranking is that of topk; the band is the number of candidates whose key (DistMult: -score; distance
    scorers: squared distance) differs from the held-out tail's by at most eps - counted here from scores evaluated one
    by one, with eps per query from zero (ties of the tail with itself and its copies only) to wider than every gap."""
    G = small_graph(scorer, n_ent=400, n_rel=5, dim=16, B=8, N=0, normal=True)
    G["ent"][333] = G["ent"][G["t"][1]]                          # an exact copy of query 1's held-out tail
    lo, hi = 3, 390
    cand = np.arange(lo, hi)
    def key(q, c):
        s = orc.score_one(scorer, G["ent"][G["h"][q]], G["rel"][G["r"][q]], None, G["ent"][c])
        return -s if scorer == "distmult" else s * s
    eps = np.array([0.0, 0.0, 1e-3, 1e-2, 5e-2, 0.3, 1e9, 2e-2])
    idx, sc, rank, band = orc.topk_band(scorer, G["ent"], G["rel"], None, G["h"], G["r"], lo, hi, 20, G["t"], eps)
    ridx, rsc, rrank = orc.topk(scorer, G["ent"], G["rel"], None, G["h"], G["r"], lo, hi, 20, G["t"])
    assert np.array_equal(idx, ridx) and np.array_equal(sc, rsc) and np.array_equal(rank, rrank)
    for q in range(8):
        kt = key(q, G["t"][q])
        keys = np.array([key(q, c) for c in cand])
        # (the square of the rounded root is not the oracle's own key: leave out candidates within 1e-12 of the edge)
        edge = np.abs(np.abs(keys - kt) - eps[q]) <= 1e-12 * max(abs(kt), 1.0)
        lo_n, hi_n = int(np.sum((np.abs(keys - kt) <= eps[q]) & ~edge)), int(np.sum((np.abs(keys - kt) <= eps[q]) | edge))
        assert lo_n <= band[q] <= hi_n, (q, band[q], lo_n, hi_n)
    assert band[6] == hi - lo and band[1] >= (2 if lo <= G["t"][1] < hi else 1)


def test_bucketing_matches_numpy(orc):
    g = ks.rng(1, ks.TAG_TRIPLE_H)
    n_ent, D, n = 1003, 4, 5000
    part = -(-n_ent // D)
    h = ks.uniform_ids(g, 0, n_ent, n); t = ks.uniform_ids(g, 0, n_ent, n)
    counts, offsets, order = orc.bucket_triples(h, t, part, D)
    bkt = (h // part) * D + (t // part)
    assert np.array_equal(counts, np.bincount(bkt, minlength=D * D))
    assert offsets[0] == 0 and np.array_equal(np.diff(offsets), counts) and offsets[-1] == n
    assert np.array_equal(order, np.argsort(bkt, kind="stable"))
    # shard sizes |E_i| = ceil(|E|/D) except the last; every head of bucket (i, j) lies in E_i
    for i in range(D):
        for j in range(D):
            sel = order[offsets[i * D + j]:offsets[i * D + j + 1]]
            assert np.all(h[sel] // part == i) and np.all(t[sel] // part == j)
