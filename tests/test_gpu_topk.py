"""kge_topk and kge_partition_triples against the oracle: indices bit-exact, scores within tolerance."""
import numpy as np
import pytest

import kge_synth as ks
from helpers import RTOL_BF16, RTOL_F32, dev_idx, gpu_model, make_case, norm_err, rank_band_eps, small_graph, to_dev

pytestmark = pytest.mark.gpu


def _check(orc, scorer, G, bf16, lo, hi, K, true_t=None):
    import paper_2211_12281_amd as kge
    model = gpu_model(scorer, G, bf16)
    tt = None if true_t is None else dev_idx(true_t)
    idx, sc, rank = kge.topk(model, dev_idx(G["h"]), dev_idx(G["r"]), lo, hi, K, tt)
    relw = G.get("relw")
    ridx, rsc, rrank = orc.topk(scorer, G["ent"], G["rel"], relw, G["h"], G["r"], lo, hi, K, true_t)
    idx, sc = idx.cpu().numpy(), sc.cpu().numpy()
    if scorer in ("rotate", "transh") and not np.array_equal(idx, ridx):
        # the key passes through cos / sin in fp64, whose last bit belongs to the math library (TransH: through the
        # normalisation of w and two fp64 dot products whose summation order is the implementation's): two candidates
        # whose keys agree to 1e-12 may legitimately swap places; anything else must be identical
        for (q, i) in np.argwhere(idx != ridx):
            one = slice(q, q + 1)
            _, s = orc.score_batch(scorer, G["ent"], G["rel"], relw, G["h"][one], G["r"][one], G["h"][one], idx[q, i:i + 1])
            assert abs(s[0, 0] - rsc[q, i]) <= 1e-12 * max(abs(rsc[q, i]), 1e-30), (q, i)
    else:
        assert np.array_equal(idx, ridx), np.argwhere(idx != ridx)[:5]
    fin = np.isfinite(rsc)
    assert np.array_equal(np.isfinite(sc), fin)
    if fin.any():
        assert np.max(np.abs(sc[fin] - rsc[fin])) <= RTOL_F32 * np.max(np.abs(rsc[fin]))   # fp64 key, rounded to fp32 once
    if true_t is not None:
        rank = rank.cpu().numpy()
        n = min(K, hi - lo)
        inside = rrank <= n
        assert np.array_equal(rank[inside], rrank[inside])          # exact whenever the tail is in the list
        assert np.all(rank[~inside] > n)
        # beyond the list the rank is counted with matrix-core values: it may differ from the exact rank by at most the
        # number of candidates whose exact key lies inside the error band of those values around the true tail's key,
        # which the oracle counts in the same pass
        if (~inside).any() and hi > lo:
            t_max = float(np.max(np.linalg.norm(G["ent"][lo:hi].astype(np.float64), axis=1)))
            eps = rank_band_eps(scorer, G["ent"][G["h"]], G["rel"][G["r"]], None if relw is None else relw[G["r"]], bf16, t_max)
            _, _, rrank2, band = orc.topk_band(scorer, G["ent"], G["rel"], relw, G["h"], G["r"], lo, hi, K, true_t, eps)
            assert np.array_equal(rrank2, rrank)
            assert np.all(np.abs(rank[~inside] - rrank[~inside]) <= band[~inside])


@pytest.mark.parametrize("scorer", ["distmult", "transe", "complex", "rotate", "transh"])
@pytest.mark.parametrize("bf16", [False, True])
def test_full_ranking_small_graph(orc, scorer, bf16):
    """64 queries over all 1,000 entities, K = 100 (the tiny configuration's brute-force ranking)."""
    G = small_graph(scorer, 1000, 10, 32, 64, 0, normal=True)
    if bf16:
        G["ent"], G["rel"] = ks.round_to_bf16(G["ent"]), ks.round_to_bf16(G["rel"])
        if G["relw"] is not None:
            G["relw"] = ks.round_to_bf16(G["relw"])
    _check(orc, scorer, G, bf16, 0, 1000, 100, G["t"])


@pytest.mark.parametrize("scorer,bf16,dim", [("distmult", True, 256), ("transe", True, 256), ("distmult", False, 64),
                                             ("transe", False, 128), ("distmult", True, 512), ("transe", False, 256),
                                             ("complex", True, 256), ("rotate", True, 256), ("complex", False, 72),
                                             ("rotate", False, 128), ("complex", True, 512), ("rotate", True, 48),
                                             ("transh", True, 256), ("transh", False, 128), ("transh", True, 80),
                                             ("transh", False, 24)])
def test_many_candidates_several_chunks(orc, scorer, bf16, dim):
    G = make_case(scorer, 60000, 20, dim, 300, 0, bf16)
    true_t = ks.uniform_ids(ks.rng(3, ks.TAG_HELDOUT), 0, 60000, 300)
    _check(orc, scorer, G, bf16, 0, 60000, 100, true_t)


def test_ties_sub_ranges_and_padding(orc):
    G = make_case("distmult", 3000, 5, 32, 10, 0, False)
    for dst, src in [(1500, 3), (77, 3), (2999, 120), (10, 120), (5, 6)]:
        G["ent"][dst] = G["ent"][src]                      # exact ties: lower index first
    true_t = np.array([1500, 77, 3, 2999, 10, 6, 0, 1, 2, 2999], dtype=np.int32)
    for (lo, hi, K) in [(0, 3000, 50), (2, 2900, 256), (100, 101, 3), (40, 70, 64), (7, 7, 5)]:
        _check(orc, "distmult", G, False, lo, hi, K, true_t)
    _check(orc, "distmult", G, False, 0, 3000, 10, None)


def test_adversarial_candidate_order_still_exact(orc):
    """Candidates sorted by increasing score for every query: each new row beats the threshold, buffers
    overflow, and the exhaustive fp64 path must take over."""
    G = make_case("distmult", 30000, 3, 32, 4, 0, False)
    G["rel"][:] = np.abs(G["rel"]) + 0.01
    G["ent"] = np.abs(G["ent"])
    order = np.argsort(G["ent"].astype(np.float64).sum(1))
    scale = np.linspace(0.1, 3.0, 30000).astype(np.float32)[:, None]
    G["ent"] = (G["ent"][order] * scale).astype(np.float32)
    G["h"] = np.array([5, 17, 100, 29999], dtype=np.int32)
    _check(orc, "distmult", G, False, 0, 30000, 20, np.array([29990, 3, 15000, 29999], dtype=np.int32))


def test_partition_bucketing(orc):
    import paper_2211_12281_amd as kge
    g = ks.rng(1, ks.TAG_TRIPLE_H)
    for (n_ent, D, n) in [(1003, 4, 5000), (90000, 16, 200000), (50, 64, 3000), (10, 1, 7)]:
        part = -(-n_ent // D)
        h, t = ks.uniform_ids(g, 0, n_ent, n), ks.uniform_ids(g, 0, n_ent, n)
        off, order = kge.partition_triples(dev_idx(h), dev_idx(t), part, D)
        rc, ro, rord = orc.bucket_triples(h, t, part, D)
        assert np.array_equal(off.cpu().numpy(), ro) and np.array_equal(order.cpu().numpy(), rord)
