"""kge_encode / kge_encode_bwd against the oracle, and the encoder chained with kge_loss_bwd on the compact table."""
import numpy as np
import pytest

import kge_synth as ks
from helpers import RTOL_BF16, RTOL_F32, dev_idx, norm_err, to_dev

pytestmark = pytest.mark.gpu


def _case(n_ent, d, fd, B, N, bf16, seed=0):
    ent = ks.uniform_rows(ks.BASE_SEED + seed, ks.TAG_ENT, np.arange(n_ent), d, 0.3)
    feat = ks.uniform_rows(ks.BASE_SEED + seed, 21, np.arange(n_ent), fd, 0.5)
    mh = ks.uniform_rows(ks.BASE_SEED + seed, 22, np.arange(d), fd, 0.08)
    mt = ks.uniform_rows(ks.BASE_SEED + seed, 23, np.arange(d), fd, 0.08)
    if bf16:
        ent, feat, mh, mt = (ks.round_to_bf16(x) for x in (ent, feat, mh, mt))
    g = ks.rng(ks.BASE_SEED + seed, ks.TAG_BATCH, 5)
    z = ks.ZipfIds(n_ent, 1.1)
    h, t = z.draw(g, B), z.draw(g, B)
    neg = ks.uniform_ids(g, 0, n_ent, N)
    return ent, feat, mh, mt, h, t, neg


def _encoder(ent, feat, mh, mt, bf16, **kw):
    import paper_2211_12281_amd as kge
    return kge.Encoder(to_dev(ent, bf16), to_dev(feat, bf16), to_dev(mh, bf16), to_dev(mt, bf16), **kw)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("d,fd,B,N", [(64, 96, 150, 333), (256, 768, 300, 700), (128, 32, 1, 1), (32, 768, 129, 0)])
def test_forward_matches_oracle(orc, bf16, d, fd, B, N):
    ent, feat, mh, mt, h, t, neg = _case(2000, d, fd, B, N, bf16)
    kw = dict(dropout=0.2, reg_t=0.01, reg_s=0.02, reg_f=0.03)
    enc = _encoder(ent, feat, mh, mt, bf16, dropout_tag=12, **kw)
    e, proj, reg = enc.encode(dev_idx(h), dev_idx(t), dev_idx(neg), seed=ks.BASE_SEED, step=7)
    idx = np.concatenate([h, t, neg])
    om, rproj, re = orc.encode(ent, feat, mh, mt, idx, B, N, p=0.2, seed=ks.BASE_SEED, step=7, tag=12,
                               reg_t=0.01, reg_s=0.02, reg_f=0.03)
    tol = RTOL_BF16 if bf16 else RTOL_F32
    assert norm_err(proj.cpu().numpy(), rproj) <= tol
    got_e = e.float().cpu().numpy()
    # the dropped / kept pattern is part of the result: an element kept on one side and dropped on the other would
    # differ by its whole projection
    assert norm_err(got_e, re) <= tol
    assert abs(reg.item() - om) <= tol * om


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("d,fd,B,N,p", [(64, 96, 150, 333, 0.2), (256, 768, 300, 2100, 0.0), (128, 32, 1, 1, 0.5),
                                        (32, 768, 0, 77, 0.1), (64, 64, 40, 0, 0.1)])
def test_backward_matches_oracle(orc, bf16, d, fd, B, N, p):
    ent, feat, mh, mt, h, t, neg = _case(2000, d, fd, B, N, bf16, seed=1)
    import torch
    kw = dict(dropout=p, reg_t=0.01, reg_s=0.02, reg_f=0.03)
    enc = _encoder(ent, feat, mh, mt, bf16, dropout_tag=12, **kw)
    hd, td, nd = dev_idx(h), dev_idx(t), dev_idx(neg)
    e, proj, reg = enc.encode(hd, td, nd, seed=3, step=9)
    de = ks.uniform_rows(5, 31, np.arange(2 * B + N), d, 1.0)
    g_es, g_mh, g_mt = enc.encode_bwd(hd, td, nd, proj, torch.from_numpy(de).cuda(), seed=3, step=9)
    idx = np.concatenate([h, t, neg])
    r_es, r_mh, r_mt = orc.encode_bwd(ent, feat, mh, mt, idx, B, N, de, p=p, seed=3, step=9, tag=12,
                                      reg_t=0.01, reg_s=0.02, reg_f=0.03)
    tol = RTOL_BF16 if bf16 else RTOL_F32
    errs = {"g_es": norm_err(g_es.cpu().numpy(), r_es) if 2 * B + N else 0.0}
    if B:
        errs["g_mh"] = norm_err(g_mh.cpu().numpy(), r_mh)
    else:
        assert not g_mh.cpu().numpy().any()
    errs["g_mt"] = norm_err(g_mt.cpu().numpy(), r_mt)
    assert all(v <= tol for v in errs.values()), errs


def test_encoder_feeds_the_loss_on_the_compact_table(orc):
    """e -> kge_loss_bwd on the 2B+N row table -> kge_encode_bwd, against the same chain of the oracle."""
    import paper_2211_12281_amd as kge
    import torch
    d, fd, B, N, n_ent, n_rel = 64, 128, 96, 200, 1500, 7
    ent, feat, mh, mt, h, t, neg = _case(n_ent, d, fd, B, N, False, seed=2)
    rel = ks.uniform_rows(ks.BASE_SEED, ks.TAG_REL, np.arange(n_rel), d, 0.3)
    r = ks.uniform_ids(ks.rng(1, 2, 3), 0, n_rel, B)
    enc = _encoder(ent, feat, mh, mt, False, dropout=0.1, reg_t=0.005)
    hd, td, nd = dev_idx(h), dev_idx(t), dev_idx(neg)
    e, proj, reg = enc.encode(hd, td, nd, seed=1, step=2)
    model = kge.Model("distmult", e, torch.from_numpy(rel).cuda())
    ar = lambda a, b: torch.arange(a, b, dtype=torch.int32, device="cuda")
    out = kge.loss_bwd(model, "sampled_softmax", ar(0, B), dev_idx(r), ar(B, 2 * B), ar(2 * B, 2 * B + N), n_ent_for_c=n_ent)
    g_es, g_mh, g_mt = enc.encode_bwd(hd, td, nd, proj, out["g_ent"], seed=1, step=2)
    # oracle chain
    idx = np.concatenate([h, t, neg])
    om, _, re = orc.encode(ent, feat, mh, mt, idx, B, N, p=0.1, seed=1, step=2, tag=12, reg_t=0.005)
    ref = orc.loss_bwd("distmult", "sampled_softmax", re.astype(np.float32), rel, None, np.arange(B), r, np.arange(B, 2 * B),
                       np.arange(2 * B, 2 * B + N), n_ent_for_c=n_ent)
    r_es, r_mh, r_mt = orc.encode_bwd(ent, feat, mh, mt, idx, B, N, ref["g_ent"], p=0.1, seed=1, step=2, tag=12, reg_t=0.005)
    assert abs(out["loss"].item() + reg.item() - (ref["loss"] + om)) <= 1e-5 * abs(ref["loss"] + om)
    for got, want in ((g_es, r_es), (g_mh, r_mh), (g_mt, r_mt), (out["g_rel"], ref["g_rel"])):
        assert norm_err(got.cpu().numpy(), want) <= 2e-5        # e itself is rounded to fp32 between the two stages
