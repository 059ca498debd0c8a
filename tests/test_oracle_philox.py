"""Pins for the oracle's Philox4x32-10 and its id mapping (negative sampling, eq. (negsamples))."""
import numpy as np

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def py_philox(ctr, key):
    """Independent big-integer implementation of the published algorithm (Salmon et al., SC'11)."""
    c = [int(x) for x in ctr]
    k = [int(x) for x in key]
    for _ in range(10):
        p0 = M0 * c[0]
        p1 = M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & MASK, p1 & MASK, ((p0 >> 32) ^ c[3] ^ k[1]) & MASK, p0 & MASK]
        k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
    return c


def py_negatives(seed, step, tag, lo, hi, n):
    out = []
    for i in range(n):
        blk = i // 2
        w = py_philox([blk & MASK, blk >> 32, step & MASK, tag], [seed & MASK, (seed >> 32) & MASK])
        half = i % 2
        x = (w[2 * half + 1] << 32) | w[2 * half]
        out.append(lo + ((x * (hi - lo)) >> 64))
    return np.array(out, dtype=np.int64)


def test_single_round_hand_computed(orc):
    # ctr=(1,0,0,0), key=(0,0): M0*1 = 0x00000000_D2511F53, M1*0 = 0
    assert list(orc.philox_single_round([1, 0, 0, 0], [0, 0])) == [0, 0, 0, 0xD2511F53]
    # ctr=(2,5,3,7), key=(11,13): M0*2 = 0x1_A4A23EA6, M1*3 = 0x2_68DBA805
    # out = (2^5^11, 0x68DBA805, 1^7^13, 0xA4A23EA6) = (12, ..., 11, ...)
    assert list(orc.philox_single_round([2, 5, 3, 7], [11, 13])) == [12, 0x68DBA805, 11, 0xA4A23EA6]


def test_published_known_answers(orc):
    """The generator's published known-answer vectors (tests/golden/philox4x32_10_kat.txt)."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for w in rows:
        v = [int(x, 16) for x in w]
        assert list(orc.philox4x32_10(v[0:4], v[4:6])) == v[6:10]
        assert py_philox(v[0:4], v[4:6]) == v[6:10]


def test_block_matches_bigint_implementation(orc):
    g = np.random.default_rng(5)
    cases = [([0, 0, 0, 0], [0, 0]), ([MASK] * 4, [MASK] * 2), ([1, 2, 3, 4], [5, 6])]
    for _ in range(3000):
        cases.append((g.integers(0, 1 << 32, 4).tolist(), g.integers(0, 1 << 32, 2).tolist()))
    for i in range(3000):   # consecutive counters, as the sampler uses them
        cases.append(([i, 0, 17, 7], [221112281, 0]))
    for ctr, key in cases:
        assert list(orc.philox4x32_10(ctr, key)) == py_philox(ctr, key), (ctr, key)


def test_block_is_injective_on_a_counter_range(orc):
    # Philox is a bijection of the 128-bit counter for a fixed key: no two counters may collide.
    seen = set()
    for i in range(20000):
        seen.add(tuple(orc.philox4x32_10([i, 0, 0, 0], [42, 0]).tolist()))
    assert len(seen) == 20000


def test_ids_match_bigint_mapping(orc):
    for (seed, step, tag, lo, hi, n) in [(221112281, 0, 7, 0, 1000, 257), (2**40 + 3, 123456, 7, 100, 91230610, 300),
                                         (1, 2**32 - 1, 9, 5, 6, 11), (7, 3, 7, 0, 2**31 - 1, 64)]:
        got = orc.sample_negatives(seed, step, tag, lo, hi, n).astype(np.int64)
        assert np.array_equal(got, py_negatives(seed, step, tag, lo, hi, n))
        assert got.min() >= lo and got.max() < hi


def test_ids_are_uniform_chi_square(orc):
    n, bins = 400_000, 100
    ids = orc.sample_negatives(221112281, 5, 7, 0, bins, n)
    cnt = np.bincount(ids, minlength=bins).astype(np.float64)
    chi2 = ((cnt - n / bins) ** 2 / (n / bins)).sum()
    # 99 degrees of freedom: mean 99, sd ~14; 180 is beyond the 1e-6 tail
    assert chi2 < 180.0, chi2


def test_streams_differ_by_step_and_tag(orc):
    a = orc.sample_negatives(1, 0, 7, 0, 10**6, 64)
    assert not np.array_equal(a, orc.sample_negatives(1, 1, 7, 0, 10**6, 64))
    assert not np.array_equal(a, orc.sample_negatives(1, 0, 8, 0, 10**6, 64))
    assert not np.array_equal(a, orc.sample_negatives(2, 0, 7, 0, 10**6, 64))
    assert np.array_equal(a, orc.sample_negatives(1, 0, 7, 0, 10**6, 64))
    # a prefix of a longer draw is the shorter draw (counter-based, no hidden state)
    assert np.array_equal(a[:33], orc.sample_negatives(1, 0, 7, 0, 10**6, 33))
