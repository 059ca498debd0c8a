"""Pins of the oracle's relation-aware triple sampler (arXiv 2211.12281, Section 4, "Training"):
p((h,r,t)) = (1/n_r) * cbrt(n_r) / sum_r' cbrt(n_r') inside a partition bucket T_ij, with replacement."""
import math
from fractions import Fraction

import numpy as np

import kge_synth as ks


def _graph(n=6000, n_ent=400, n_rel=9, seed=5):
    g = np.random.default_rng(seed)
    h = g.integers(0, n_ent, n).astype(np.int32)
    t = g.integers(0, n_ent, n).astype(np.int32)
    # skewed relation frequencies, one relation absent altogether
    p = np.array([0.45, 0.2, 0.1, 0.1, 0.08, 0.04, 0.02, 0.01, 0.0])
    r = g.choice(n_rel, size=n, p=p).astype(np.int32)
    return h, r, t


def test_cube_root_weight_is_the_exact_integer_root(orc):
    for n in [0, 1, 2, 3, 7, 8, 9, 26, 27, 28, 999, 1000, 123456789, 2 ** 32 - 1]:
        w = orc.cbrt_weight(n)
        assert w ** 3 <= n << 60 < (w + 1) ** 3            # python integers: exact
    # perfect cubes give exact multiples, so small tables have exactly rational probabilities
    assert orc.cbrt_weight(8) == 2 * orc.cbrt_weight(1) and orc.cbrt_weight(27) == 3 * orc.cbrt_weight(1)
    assert abs(orc.cbrt_weight(5) / 2 ** 20 - 5 ** (1 / 3)) < 2 ** -20


def test_index_is_a_stable_sort_by_bucket_and_relation(orc):
    h, r, t = _graph()
    D, n_rel, part = 4, 9, 100
    order, offs, cdf = orc.sampler_build(h, r, t, part, D, n_rel)
    key = ((h // part) * D + (t // part)).astype(np.int64) * n_rel + r
    assert np.array_equal(order, np.argsort(key, kind="stable"))          # library routine
    assert np.array_equal(offs, np.searchsorted(key[order], np.arange(D * D * n_rel + 1)))
    cnt = np.diff(offs).reshape(D * D, n_rel)
    w = np.vectorize(orc.cbrt_weight, otypes=[np.uint64])(cnt)
    assert np.array_equal(cdf.reshape(D * D, n_rel), np.cumsum(w, axis=1, dtype=np.uint64))
    # the buckets agree with the plain partition bucketing
    _, boffs, _ = orc.bucket_triples(h, t, part, D)
    assert np.array_equal(offs[::n_rel], boffs)


def test_draws_follow_the_cube_root_law(orc):
    """Relation frequencies of many draws against cbrt(n_r)/sum cbrt (chi-square), and uniformity inside a relation."""
    h, r, t = _graph(n=20000, n_ent=200)
    D, n_rel, part = 2, 9, 100
    order, offs, cdf = orc.sampler_build(h, r, t, part, D, n_rel)
    draws = 200000
    bucket = 3
    pos = orc.sample_triples(ks.BASE_SEED, 17, 8, bucket, 1, draws, n_rel, offs, cdf, order)
    assert pos.min() >= 0
    assert np.all((h[pos] // part) * D + (t[pos] // part) == bucket)      # every draw comes from the bucket
    cnt = np.diff(offs).reshape(D * D, n_rel)[bucket].astype(np.float64)
    p = np.cbrt(cnt) / np.cbrt(cnt).sum()
    obs = np.bincount(r[pos], minlength=n_rel).astype(np.float64)
    assert obs[cnt == 0].sum() == 0
    live = cnt > 0
    chi2 = (((obs - draws * p) ** 2)[live] / (draws * p[live])).sum()
    assert chi2 < 40.0, chi2          # 7 degrees of freedom: P(chi2 > 40) ~ 1e-6; a sqrt or linear law gives > 10^4
    # a law proportional to n_r (plain uniform sampling of triples) is rejected by the same statistic
    q = cnt / cnt.sum()
    assert (((obs - draws * q) ** 2)[live] / (draws * q[live])).sum() > 1e4
    # inside the most frequent relation every triple is equally likely
    rel = int(np.argmax(cnt))
    grp = order[offs[bucket * n_rel + rel]:offs[bucket * n_rel + rel + 1]]
    hits = np.bincount(np.searchsorted(np.sort(grp), pos[r[pos] == rel]), minlength=len(grp)).astype(np.float64)
    exp = hits.sum() / len(grp)
    assert ((hits - exp) ** 2 / exp).sum() < len(grp) + 6 * math.sqrt(2 * len(grp))
    # with replacement: far more draws than triples in the bucket
    assert draws > cnt.sum() and len(np.unique(pos)) <= cnt.sum()


def test_small_table_has_exact_probabilities(orc):
    """Two relations with 1 and 8 triples: weights 1 : 2, so relation 0 is drawn iff x * 3 * 2^20 / 2^64 < 2^20,
    i.e. iff x < 2^64 / 3 -- checked against the generator's raw words."""
    h = np.zeros(9, dtype=np.int32); t = np.zeros(9, dtype=np.int32)
    r = np.array([1, 1, 0, 1, 1, 1, 1, 1, 1], dtype=np.int32)
    order, offs, cdf = orc.sampler_build(h, r, t, 10, 1, 2)
    assert list(cdf) == [2 ** 20, 3 * 2 ** 20] and list(offs) == [0, 1, 9] and order[0] == 2
    n = 3000
    pos = orc.sample_triples(99, 4, 8, 0, 1, n, 2, offs, cdf, order)
    for q in range(0, n, 7):
        w = orc.philox4x32_10(np.array([q, 0, 4, 8], dtype=np.uint32), np.array([99, 0], dtype=np.uint32))
        x, y = (int(w[1]) << 32) | int(w[0]), (int(w[3]) << 32) | int(w[2])
        if Fraction(x * 3 * 2 ** 20, 2 ** 64) < 2 ** 20:
            assert pos[q] == 2
        else:
            k = (y * 8) >> 64
            assert pos[q] == [0, 1, 3, 4, 5, 6, 7, 8][k]
    assert abs((pos == 2).mean() - 1 / 3) < 0.03


def test_microbatch_takes_equal_parts_from_every_tail_partition(orc):
    """B_i = union over j of B/D draws from T_ij (eq. (microbatch)); empty buckets give -1."""
    h, r, t = _graph(n=3000, n_ent=300)
    t[(h // 100 == 2) & (t // 100 == 1)] = 250        # empty the bucket (2, 1)
    D, n_rel, part = 3, 9, 100
    order, offs, cdf = orc.sampler_build(h, r, t, part, D, n_rel)
    per = 50
    for i in range(D):
        pos = orc.sample_triples(7, 1, 8, i * D, D, per, n_rel, offs, cdf, order)
        for j in range(D):
            seg = pos[j * per:(j + 1) * per]
            if (i, j) == (2, 1):
                assert np.all(seg == -1)
            else:
                assert np.all(h[seg] // part == i) and np.all(t[seg] // part == j)
    # the draws of a step do not depend on how the call is split: bucket-by-bucket calls differ only by
    # their counter range, so the same (bucket_lo, n_buckets) call is reproducible
    again = orc.sample_triples(7, 1, 8, 0, D, per, n_rel, offs, cdf, order)
    assert np.array_equal(again, orc.sample_triples(7, 1, 8, 0, D, per, n_rel, offs, cdf, order))
    assert not np.array_equal(again, orc.sample_triples(7, 2, 8, 0, D, per, n_rel, offs, cdf, order))


def test_sharded_negatives_cover_every_shard_equally(orc):
    n_ent, D, per = 1003, 4, 64
    part = -(-n_ent // D)
    neg = orc.sample_negatives_sharded(5, 3, 7, part, n_ent, D, per)
    for j in range(D):
        seg = neg[j * per:(j + 1) * per]
        assert seg.min() >= j * part and seg.max() < min(n_ent, (j + 1) * part)
    # slot n uses the same generator block as the plain sampler: equal to it when the shard range is passed
    for j in range(D):
        lo, hi = j * part, min(n_ent, (j + 1) * part)
        plain = orc.sample_negatives(5, 3, 7, lo, hi, D * per)
        assert np.array_equal(neg[j * per:(j + 1) * per], plain[j * per:(j + 1) * per])
