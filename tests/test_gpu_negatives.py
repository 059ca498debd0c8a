"""Negative sampling on the GPU is bit-exact against the oracle's Philox (eq. (negsamples))."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed,step,tag,lo,hi,n", [
    (221112281, 0, 7, 0, 1000, 64), (221112281, 3, 7, 0, 1_000_000, 8192), (2**40 + 3, 123456, 7, 100, 91230610, 16385),
    (1, 2**32 - 1, 9, 5, 6, 11), (7, 3, 7, 0, 2**31 - 1, 1), (9, 9, 9, 0, 10, 0), (5, 1, 7, 5_625_000, 11_250_000, 4096)])
def test_negatives_bit_exact(orc, seed, step, tag, lo, hi, n):
    import paper_2211_12281_amd as kge
    got = kge.sample_negatives(seed, step, tag, lo, hi, n).cpu().numpy()
    assert np.array_equal(got, orc.sample_negatives(seed, step, tag, lo, hi, n))
