"""kge_score against the oracle: all five scorers, fp32 and bf16, several tiles and ragged tails."""
import numpy as np
import pytest

from helpers import RTOL_BF16, RTOL_F32, dev_idx, gpu_model, make_case, norm_err

pytestmark = pytest.mark.gpu
SCORERS = ["transe", "transh", "rotate", "distmult", "complex"]


def _run(orc, scorer, G, bf16, want_neg=True):
    import paper_2211_12281_amd as kge
    model = gpu_model(scorer, G, bf16)
    pos, neg = kge.score(model, dev_idx(G["h"]), dev_idx(G["r"]), dev_idx(G["t"]), dev_idx(G["neg"]), want_neg)
    rp, rn = orc.score_batch(scorer, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"])
    return pos.cpu().numpy(), None if neg is None else neg.cpu().numpy(), rp, rn


@pytest.mark.parametrize("scorer", SCORERS)
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("dim,B,N", [(64, 200, 333), (256, 130, 257), (32, 64, 64)])
def test_scores_match_oracle(orc, scorer, bf16, dim, B, N):
    G = make_case(scorer, 5000, 20, dim, B, N, bf16)
    pos, neg, rp, rn = _run(orc, scorer, G, bf16)
    tol = RTOL_BF16 if bf16 else RTOL_F32
    assert norm_err(pos, rp) <= tol, ("pos", norm_err(pos, rp))
    assert norm_err(neg, rn) <= tol, ("neg", norm_err(neg, rn))


@pytest.mark.parametrize("scorer", ["transe", "transh", "complex"])
def test_large_rows_fp32_1024_bytes(orc, scorer):
    G = make_case(scorer, 3000, 10, 256, 140, 200, False)
    pos, neg, rp, rn = _run(orc, scorer, G, False)
    assert norm_err(pos, rp) <= RTOL_F32 and norm_err(neg, rn) <= RTOL_F32


@pytest.mark.parametrize("scorer", ["transe", "distmult"])
def test_edge_shapes(orc, scorer):
    import paper_2211_12281_amd as kge
    for (B, N) in [(1, 1), (1, 300), (300, 1), (5, 0)]:
        G = make_case(scorer, 1000, 5, 32, B, N, False)
        pos, neg, rp, rn = _run(orc, scorer, G, False)
        assert norm_err(pos, rp) <= RTOL_F32
        assert neg.shape == (B, N)
        if N:
            assert norm_err(neg, rn) <= RTOL_F32
    G = make_case(scorer, 1000, 5, 32, 7, 9, False)
    pos, neg, rp, _ = _run(orc, scorer, G, False, want_neg=False)
    assert neg is None and norm_err(pos, rp) <= RTOL_F32
    # B = 0 is a no-op
    model = gpu_model(scorer, G, False)
    e = dev_idx(np.zeros(0, np.int32))
    p, n = kge.score(model, e, e, e, dev_idx(G["neg"]))
    assert p.numel() == 0


@pytest.mark.parametrize("scorer", ["transe", "rotate", "transh"])
@pytest.mark.parametrize("bf16", [False, True])
def test_near_zero_distances_do_not_cancel(orc, scorer, bf16):
    """Negatives that (almost) coincide with the query: the norm-expansion form would cancel."""
    import kge_synth as ks
    G = make_case(scorer, 2000, 5, 64, 40, 70, bf16)
    E = G["ent"].astype(np.float64)
    R = G["rel"].astype(np.float64)
    for b, n in [(0, 0), (1, 5), (39, 69)]:
        h, r = E[G["h"][b]], R[G["r"][b]]
        if scorer == "transe":
            q = h + r
        elif scorer == "rotate":
            c = 32
            q = np.r_[h[:c] * np.cos(r) - h[c:] * np.sin(r), h[:c] * np.sin(r) + h[c:] * np.cos(r)]
        else:
            w = G["relw"][G["r"][b]].astype(np.float64); w /= np.linalg.norm(w)
            q = h - (w @ h) * w + r
        row = (q * (1 + 1e-4)).astype(np.float32)
        G["ent"][G["neg"][n]] = ks.round_to_bf16(row) if bf16 else row
    pos, neg, rp, rn = _run(orc, scorer, G, bf16)
    tol = RTOL_BF16 if bf16 else RTOL_F32
    assert norm_err(neg, rn) <= tol, norm_err(neg, rn)
    assert norm_err(pos, rp) <= tol
