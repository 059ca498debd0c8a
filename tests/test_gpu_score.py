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


@pytest.mark.parametrize("scorer", SCORERS)
@pytest.mark.parametrize("dim", [128, 104, 200])
def test_fp32_tables_on_the_bf16_pipe(orc, scorer, dim):
    """fp32 rows padded to 128 or 256 dimensions are contracted as two fp16 pieces per operand: against the oracle,
    and against the kernel that uses the fp32 matrix instructions (selected through the library's debug call)."""
    import paper_2211_12281_amd as kge
    G = make_case(scorer, 4000, 12, dim, 200, 333, False)
    pos, neg, rp, rn = _run(orc, scorer, G, False)
    assert norm_err(pos, rp) <= RTOL_F32 and norm_err(neg, rn) <= RTOL_F32
    kge.debug_select("score_f32_mfma", True)
    try:
        pos2, neg2, _, _ = _run(orc, scorer, G, False)
    finally:
        kge.debug_select("score_f32_mfma", False)
    assert norm_err(neg2, rn) <= RTOL_F32
    assert norm_err(neg, neg2) <= RTOL_F32 and np.array_equal(pos, pos2)


@pytest.mark.parametrize("scorer", ["transe", "transh", "distmult", "rotate"])
@pytest.mark.parametrize("scale", [1e-4, 3e3, None])
def test_fp32_score_block_does_not_depend_on_the_scale_of_the_tables(orc, scorer, scale):
    """The fp32 rows reach the matrix cores as two fp16 pieces of the row scaled by a power of two of its own: tables a
    factor 1e-4 or 3e3 away from the usual magnitudes, and rows whose columns span four decades (scale None), stay
    inside the fp32 tolerance."""
    G = make_case(scorer, 4000, 12, 256, 200, 333, False)
    if scale is None:
        col = (10.0 ** (-4.0 * np.random.default_rng(3).random(256))).astype(np.float32)
        G["ent"] = G["ent"] * col
    else:
        G["ent"] = (G["ent"] * scale).astype(np.float32)
        if scorer != "rotate":
            G["rel"] = (G["rel"] * scale).astype(np.float32)
    pos, neg, rp, rn = _run(orc, scorer, G, False)
    assert norm_err(pos, rp) <= RTOL_F32 and norm_err(neg, rn) <= RTOL_F32, norm_err(neg, rn)


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
@pytest.mark.parametrize("bf16,dim", [(False, 64), (True, 64), (False, 128), (False, 256)])
def test_near_zero_distances_do_not_cancel(orc, scorer, bf16, dim):
    """Negatives that (almost) coincide with the query: the norm-expansion form would cancel (fp32 rows of 128 and 256
    dimensions take the kernels that contract two fp16 pieces per operand: their guard is the same)."""
    import kge_synth as ks
    G = make_case(scorer, 2000, 5, dim, 40, 70, bf16)
    E = G["ent"].astype(np.float64)
    R = G["rel"].astype(np.float64)
    for b, n in [(0, 0), (1, 5), (39, 69)]:
        h, r = E[G["h"][b]], R[G["r"][b]]
        if scorer == "transe":
            q = h + r
        elif scorer == "rotate":
            c = dim // 2
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


@pytest.mark.parametrize("scorer,bf16,dim,pad", [("complex", True, 256, 8), ("transe", True, 256, 3), ("distmult", False, 64, 4),
                                                 ("transh", False, 128, 1), ("rotate", True, 64, 24)])
def test_tables_with_a_row_stride_larger_than_the_dimension(orc, scorer, bf16, dim, pad):
    """Tables that are column slices of wider arrays (ld = dim + pad; 16-byte aligned rows and unaligned ones): scores,
    loss + gradients and the top-K list must equal those of the packed tables; the padding columns hold large garbage."""
    import torch
    import paper_2211_12281_amd as kge
    G = make_case(scorer, 5000, 7, dim, 150, 300, bf16)
    dt = torch.bfloat16 if bf16 else torch.float32

    def wide(x):
        if x is None:
            return None
        full = torch.full((x.shape[0], x.shape[1] + pad), 1e4, dtype=dt, device="cuda")
        full[:, :x.shape[1]] = torch.from_numpy(x).cuda().to(dt)
        return full[:, :x.shape[1]]

    model = kge.Model(scorer, wide(G["ent"]), wide(G["rel"]), wide(G["relw"]))
    assert model.struct.ent_ld == dim + pad
    args = (dev_idx(G["h"]), dev_idx(G["r"]), dev_idx(G["t"]), dev_idx(G["neg"]))
    tol = RTOL_BF16 if bf16 else RTOL_F32
    pos, neg = kge.score(model, *args)
    rp, rn = orc.score_batch(scorer, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"])
    assert norm_err(pos.cpu().numpy(), rp) <= tol and norm_err(neg.cpu().numpy(), rn) <= tol
    out = kge.loss_bwd(model, "sampled_softmax", *args, n_ent_for_c=5000)
    ref = orc.loss_bwd(scorer, "sampled_softmax", G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"], n_ent_for_c=5000)
    assert abs(out["loss"].item() - ref["loss"]) <= tol * abs(ref["loss"])
    assert norm_err(out["g_ent"].cpu().numpy(), ref["g_ent"]) <= tol
    assert norm_err(out["g_rel"].cpu().numpy(), ref["g_rel"]) <= tol
    if (pad * (2 if bf16 else 4)) % 16 != 0:
        with pytest.raises(kge.KgeError):          # the ranking scan wants 16-byte aligned rows (checked on the host)
            kge.topk(model, args[0], args[1], 0, 5000, 20)
        return
    idx, sc, _ = kge.topk(model, args[0], args[1], 0, 5000, 20)
    ridx, rsc, _ = orc.topk(scorer, G["ent"], G["rel"], G["relw"], G["h"], G["r"], 0, 5000, 20)
    same = idx.cpu().numpy() == ridx
    if scorer in ("rotate", "transh"):
        assert np.mean(same) > 0.999            # near-ties of keys that pass through library functions may swap
    else:
        assert np.all(same)
    assert np.max(np.abs(sc.cpu().numpy() - rsc)) <= RTOL_F32 * np.max(np.abs(rsc))
