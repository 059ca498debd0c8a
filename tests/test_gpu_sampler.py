"""kge_sampler_build / kge_sample_triples / kge_sample_negatives_sharded against the oracle: bit-exact."""
import numpy as np
import pytest

import kge_synth as ks
from helpers import dev_idx

pytestmark = pytest.mark.gpu


def _graph(n, n_ent, n_rel, seed=5, zipf_rel=True):
    g = np.random.default_rng(seed)
    z = ks.ZipfIds(n_ent, 1.1)
    h, t = z.draw(g, n).astype(np.int32), z.draw(g, n).astype(np.int32)
    if zipf_rel:
        p = 1.0 / np.arange(1, n_rel + 1); p /= p.sum()
        r = g.choice(n_rel, size=n, p=p).astype(np.int32)
    else:
        r = g.integers(0, n_rel, n).astype(np.int32)
    return h, r, t


@pytest.mark.parametrize("n,n_ent,n_rel,D", [(50000, 3000, 37, 4), (5000, 1000, 1400, 2), (300000, 90000, 14, 16),
                                              (777, 64, 3, 1)])
def test_index_and_draws_match_oracle(orc, n, n_ent, n_rel, D):
    import paper_2211_12281_amd as kge
    h, r, t = _graph(n, n_ent, n_rel)
    part = -(-n_ent // D)
    order, offs, cdf = orc.sampler_build(h, r, t, part, D, n_rel)
    smp = kge.TripleSampler(dev_idx(h), dev_idx(r), dev_idx(t), part, D, n_rel)
    assert np.array_equal(smp.order.cpu().numpy(), order)
    assert np.array_equal(smp.rel_offsets.cpu().numpy(), offs)
    assert np.array_equal(smp.cdf.cpu().numpy().view(np.uint64), cdf)
    # one worker's micro-batch (all tail partitions), then a single partition pair, ragged draw counts
    for (lo, nb, per, step) in ((0, D, 129, 3), ((D - 1) * D, D, 64, 4), (D * D - 1, 1, 1000, 5), (0, D * D, 7, 6)):
        ref = orc.sample_triples(ks.BASE_SEED, step, ks.TAG_BATCH, lo, nb, per, n_rel, offs, cdf, order)
        oh, orr, ot, pos = smp.sample(ks.BASE_SEED, step, ks.TAG_BATCH, lo, nb, per, want_pos=True)
        pos = pos.cpu().numpy()
        assert np.array_equal(pos, ref)
        live = ref >= 0
        assert np.array_equal(oh.cpu().numpy()[live], h[ref[live]])
        assert np.array_equal(orr.cpu().numpy()[live], r[ref[live]])
        assert np.array_equal(ot.cpu().numpy()[live], t[ref[live]])
        assert np.all(oh.cpu().numpy()[~live] == -1)


def test_empty_input_and_empty_buckets(orc):
    import paper_2211_12281_amd as kge
    import torch
    e = torch.empty(0, dtype=torch.int32, device="cuda")
    smp = kge.TripleSampler(e, e, e, 10, 2, 5)
    assert not smp.rel_offsets.cpu().numpy().any() and not smp.cdf.cpu().numpy().any()
    oh, orr, ot = smp.sample(1, 0, 8, 0, 4, 3)
    assert np.all(oh.cpu().numpy() == -1)
    # a graph confined to one bucket: every other bucket is empty
    h = np.arange(50, dtype=np.int32) % 10
    t = 10 + np.arange(50, dtype=np.int32) % 10
    r = (np.arange(50) % 3).astype(np.int32)
    order, offs, cdf = orc.sampler_build(h, r, t, 10, 2, 3)
    smp = kge.TripleSampler(dev_idx(h), dev_idx(r), dev_idx(t), 10, 2, 3)
    ref = orc.sample_triples(9, 1, 8, 0, 4, 16, 3, offs, cdf, order)
    _, _, _, pos = smp.sample(9, 1, 8, 0, 4, 16, want_pos=True)
    assert np.array_equal(pos.cpu().numpy(), ref) and (ref[:16] == -1).all() and (ref[16:32] >= 0).all()


@pytest.mark.parametrize("n_ent,D,per", [(1003, 4, 64), (90_000_000, 16, 256), (17, 1, 5), (1000, 8, 3)])
def test_sharded_negatives_match_oracle(orc, n_ent, D, per):
    import paper_2211_12281_amd as kge
    part = -(-n_ent // D)
    ref = orc.sample_negatives_sharded(ks.BASE_SEED, 11, ks.TAG_NEG, part, n_ent, D, per)
    out = kge.sample_negatives_sharded(ks.BASE_SEED, 11, ks.TAG_NEG, part, n_ent, D, per)
    assert np.array_equal(out.cpu().numpy(), ref)
