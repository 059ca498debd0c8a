"""kge_loss_bwd against the oracle: loss value and every gradient row, all scorers, both losses."""
import numpy as np
import pytest
import torch

from helpers import RTOL_BF16, RTOL_F32, dev_idx, gpu_model, make_case, norm_err

pytestmark = pytest.mark.gpu
SCORERS = ["transe", "transh", "rotate", "distmult", "complex"]


def _kw(scorer, loss, n_ent):
    if loss == "sampled_softmax":
        return dict(n_ent_for_c=n_ent)
    if scorer in ("distmult", "complex"):
        return dict(gamma=0.0, adv_temp=0.0)
    return dict(gamma=2.0, adv_temp=0.8)


def _compare(orc, scorer, loss, G, bf16, n_ent, kw=None, loss_scale=None):
    import paper_2211_12281_amd as kge
    kw = kw or _kw(scorer, loss, n_ent)
    model = gpu_model(scorer, G, bf16)
    out = kge.loss_bwd(model, loss, dev_idx(G["h"]), dev_idx(G["r"]), dev_idx(G["t"]), dev_idx(G["neg"]),
                       loss_scale=loss_scale or 0.0, **kw)
    ref = orc.loss_bwd(scorer, loss, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"],
                       loss_scale=loss_scale, **kw)
    tol = RTOL_BF16 if bf16 else RTOL_F32
    errs = {"loss": abs(out["loss"].item() - ref["loss"]) / max(abs(ref["loss"]), 1e-30)}
    for k in ("g_ent", "g_rel", "g_relw"):
        if ref[k] is not None and ref[k].size:
            errs[k] = norm_err(out[k].cpu().numpy(), ref[k])
    # heads, positive tails and negatives separately: a small block must not hide behind a large one
    B, N = len(G["h"]), len(G["neg"])
    ge = out["g_ent"].cpu().numpy()
    for name, sl in (("g_head", slice(0, B)), ("g_tail", slice(B, 2 * B)), ("g_neg", slice(2 * B, 2 * B + N))):
        if ref["g_ent"][sl].size:
            errs[name] = norm_err(ge[sl], ref["g_ent"][sl])
    assert np.array_equal(out["g_ent_idx"].cpu().numpy(), ref["g_ent_idx"])
    assert np.array_equal(out["g_rel_idx"].cpu().numpy(), ref["g_rel_idx"])
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, (bad, errs)
    return errs


@pytest.mark.parametrize("scorer", SCORERS)
@pytest.mark.parametrize("loss", ["logsigmoid", "sampled_softmax"])
@pytest.mark.parametrize("bf16", [False, True])
def test_loss_and_gradients_match_oracle(orc, scorer, loss, bf16):
    amp = 0.5 if scorer in ("distmult", "complex") else 0.1
    G = make_case(scorer, 4000, 12, 64, 200, 333, bf16, amp=amp, zipf=True)
    _compare(orc, scorer, loss, G, bf16, 4000)


@pytest.mark.parametrize("scorer,dim,bf16", [("complex", 256, True), ("transe", 256, False), ("distmult", 128, False),
                                             ("transh", 128, False), ("transh", 256, True), ("rotate", 256, True),
                                             ("distmult", 32, False), ("complex", 512, True)])
def test_other_row_sizes(orc, scorer, dim, bf16):
    G = make_case(scorer, 3000, 9, dim, 150, 260, bf16, amp=0.3 if scorer in ("distmult", "complex") else 0.1)
    _compare(orc, scorer, "sampled_softmax", G, bf16, 3000)
    _compare(orc, scorer, "logsigmoid", G, bf16, 3000)


@pytest.mark.parametrize("scorer,B,N", [("complex", 700, 3000), ("distmult", 2304, 4100), ("complex", 130, 70)])
def test_stored_weights_of_the_forward_pass_serve_the_pass_over_the_negatives(orc, scorer, B, N):
    """Sampled softmax, bilinear scorers, bf16 rows of 512 bytes: the forward kernel keeps its weights and the pass over the
    negatives contracts them with the scaled queries.  Several own tiles, forward splits and ragged tails of both passes,
    against the oracle; and against the kernel that recomputes the scores (the forward pass may be split differently there,
    which moves its reference exponents and with them the bf16 rounding of the weights)."""
    import paper_2211_12281_amd as kge
    G = make_case(scorer, 9000, 9, 256, B, N, True, amp=0.3, zipf=True)
    _compare(orc, scorer, "sampled_softmax", G, True, 9000)
    model = gpu_model(scorer, G, True)
    args = (dev_idx(G["h"]), dev_idx(G["r"]), dev_idx(G["t"]), dev_idx(G["neg"]))
    got = {k: v.clone() for k, v in kge.loss_bwd(model, "sampled_softmax", *args, n_ent_for_c=9000).items() if v is not None}
    kge.debug_select("gradt_recompute", True)
    try:
        want = kge.loss_bwd(model, "sampled_softmax", *args, n_ent_for_c=9000)
    finally:
        kge.debug_select("gradt_recompute", False)
    assert abs(got["loss"].item() - want["loss"].item()) <= 1e-5 * abs(want["loss"].item())
    for sl in (slice(0, B), slice(B, 2 * B), slice(2 * B, 2 * B + N)):
        assert norm_err(got["g_ent"][sl].cpu().numpy(), want["g_ent"][sl].cpu().numpy()) <= RTOL_BF16
    assert norm_err(got["g_rel"].cpu().numpy(), want["g_rel"].cpu().numpy()) <= RTOL_BF16


@pytest.mark.parametrize("dim,bf16,B,N", [(256, False, 150, 260), (512, True, 150, 260), (192, False, 700, 1500)])
def test_transh_rows_wider_than_512_bytes(orc, dim, bf16, B, N):
    """TransH at d = 256 in fp32 (one of the sizes of Table 3) and wider: 1,024-byte rows train on the vector-pipe route
    with the 2-norm (score block in memory); several tiles and ragged tails in the third case."""
    G = make_case("transh", 3000, 9, dim, B, N, bf16, amp=0.1, zipf=True)
    _compare(orc, "transh", "sampled_softmax", G, bf16, 3000)
    _compare(orc, "transh", "logsigmoid", G, bf16, 3000)
    _compare(orc, "transh", "logsigmoid", G, bf16, 3000, kw=dict(gamma=3.0, adv_temp=0.0, reg_l3=1e-3))


@pytest.mark.parametrize("scorer", ["transe", "complex"])
def test_edge_shapes(orc, scorer):
    for (B, N) in [(1, 1), (3, 0), (130, 1), (1, 130)]:
        G = make_case(scorer, 500, 4, 32, B, N, False, amp=0.3)
        for loss in ("logsigmoid", "sampled_softmax"):
            _compare(orc, scorer, loss, G, False, 500)
    G = make_case(scorer, 500, 4, 32, 20, 30, False, amp=0.3)
    _compare(orc, scorer, "logsigmoid", G, False, 500, loss_scale=0.37)


def test_tiny_distmult_training_config(orc):
    """1,000 entities, 10 relations, dim 32 fp32, N(0, 0.1^2), B = N = 64, log-sigmoid, margin 0."""
    import kge_synth as ks
    from helpers import small_graph
    G = small_graph("distmult", 1000, 10, 32, 64, 64, normal=True)
    G["neg"] = orc.sample_negatives(ks.BASE_SEED, 0, ks.TAG_NEG, 0, 1000, 64)
    _compare(orc, "distmult", "logsigmoid", G, False, 1000, kw=dict(gamma=0.0, adv_temp=0.0))


def test_repeated_calls_are_bitwise_identical(orc):
    import paper_2211_12281_amd as kge
    G = make_case("complex", 4000, 12, 64, 200, 333, True, amp=0.5, zipf=True)
    model = gpu_model("complex", G, True)
    args = (dev_idx(G["h"]), dev_idx(G["r"]), dev_idx(G["t"]), dev_idx(G["neg"]))
    a = kge.loss_bwd(model, "sampled_softmax", *args, n_ent_for_c=4000)
    a = {k: v.clone() for k, v in a.items() if v is not None}
    b = kge.loss_bwd(model, "sampled_softmax", *args, n_ent_for_c=4000)
    for k in a:
        assert bool((a[k] == b[k]).all()), k


@pytest.mark.parametrize("scorer,loss", [("distmult", "sampled_softmax"), ("complex", "logsigmoid"),
                                         ("transe", "logsigmoid")])
def test_wide_score_range_raises_the_reference_repeatedly(orc, scorer, loss):
    """Scores spread over tens of nats and negatives ordered by ascending score of the first query:
    the running reference exponent of the softmax weights is raised many times along the stream."""
    amp = 1.2 if scorer != "transe" else 2.5
    G = make_case(scorer, 3000, 7, 64, 130, 700, False, amp=amp)
    s0 = orc.score_batch(scorer, G["ent"], G["rel"], G["relw"], G["h"][:1], G["r"][:1], G["t"][:1], G["neg"])[1][0]
    a_t = 3.0 if scorer == "transe" else 1.0               # the weights' exponents are adv_temp * score
    assert (s0.max() - s0.min()) * a_t * 1.4427 > 20.0     # log2 units: several times the kernel's headroom of 8
    G["neg"] = G["neg"][np.argsort(s0, kind="stable")]
    kw = dict(n_ent_for_c=3000) if loss == "sampled_softmax" else dict(gamma=1.0, adv_temp=a_t)
    _compare(orc, scorer, loss, G, False, 3000, kw=kw)


@pytest.mark.parametrize("scorer", SCORERS)
@pytest.mark.parametrize("bf16", [False, True])
def test_l3_regulariser_matches_oracle(orc, scorer, bf16):
    """lambda_S * Omega_S over the 2B + N gathered rows joins loss and gradients (Section 3.1, Regularisation)."""
    loss = "sampled_softmax" if scorer in ("distmult", "complex") else "logsigmoid"
    G = make_case(scorer, 2000, 9, 64, 150, 300, bf16, amp=0.4, zipf=True)
    kw = dict(_kw(scorer, loss, 2000), reg_l3=0.03)
    errs = _compare(orc, scorer, loss, G, bf16, 2000, kw=kw)
    # the regulariser is a visible part of what is compared: without it the same call differs
    plain = orc.loss_bwd(scorer, loss, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"],
                         **_kw(scorer, loss, 2000))
    reg = orc.loss_bwd(scorer, loss, G["ent"], G["rel"], G["relw"], G["h"], G["r"], G["t"], G["neg"], **kw)
    assert norm_err(plain["g_ent"], reg["g_ent"]) > 10 * (RTOL_BF16 if bf16 else RTOL_F32), errs


def test_l3_regulariser_edge_shapes(orc):
    for B, N in ((0, 40), (33, 0), (1, 1)):
        G = make_case("transe", 500, 4, 32, B, N, False, amp=0.3)
        _compare(orc, "transe", "logsigmoid", G, False, 500, kw=dict(gamma=2.0, adv_temp=0.5, reg_l3=0.1),
                 loss_scale=0.5)


@pytest.mark.parametrize("scorer,loss", [("distmult", "sampled_softmax"), ("transe", "logsigmoid"), ("complex", "sampled_softmax")])
def test_wide_score_range_bf16_tables(orc, scorer, loss):
    """The same stress of the running reference exponent on bf16 tables, whose row-owner pass hands the coefficients
    and the rescaling factors from one wave to its partner."""
    amp = 1.2 if scorer != "transe" else 2.5
    G = make_case(scorer, 3000, 7, 64, 130, 700, True, amp=amp)
    s0 = orc.score_batch(scorer, G["ent"], G["rel"], G["relw"], G["h"][:1], G["r"][:1], G["t"][:1], G["neg"])[1][0]
    a_t = 3.0 if scorer == "transe" else 1.0
    assert (s0.max() - s0.min()) * a_t * 1.4427 > 20.0
    G["neg"] = G["neg"][np.argsort(s0, kind="stable")]
    kw = dict(n_ent_for_c=3000) if loss == "sampled_softmax" else dict(gamma=1.0, adv_temp=a_t)
    _compare(orc, scorer, loss, G, True, 3000, kw=kw)


def _outgrowing_case(orc, scorer, factor):
    """One negative far into the list scaled so that its scores tower over everything before it; returns the case and the
    largest excess (log2 units) of a row's scores over the maximum of its first 64."""
    import kge_synth as ks
    G = make_case(scorer, 6000, 9, 64, 2048, 4096, True, amp=0.3)
    big = int(G["neg"][200])
    G["ent"][big] = ks.round_to_bf16(G["ent"][big] * np.float32(factor))
    keep = (G["h"] != big) & (G["t"] != big)              # only its role as a negative is scaled
    for k in ("h", "r", "t"):
        G[k] = np.ascontiguousarray(G[k][keep])
    _, blk = orc.score_batch(scorer, G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"])
    return G, float((blk.max(axis=1) - blk[:, :64].max(axis=1)).max() * 1.4427)


@pytest.mark.parametrize("scorer", ["distmult", "complex"])
def test_scores_that_outgrow_the_first_tile(orc, scorer):
    """bf16 bilinear scorers, sampled softmax: the forward kernel weights every score against the maximum of the first 64
    negatives of its share (weights above 1 are fine while they stay finite) and does its pass a second time, against the
    exact row maxima, when the sums of weights show that a score exceeded that by more than about 2^100.
    Excess of some tens of units: one pass carries it - against the oracle at the usual bar.
    Excess of hundreds of units: the second pass - loss and the negatives' rows against the oracle at the usual bar; the
    heads' rows of this case mix magnitudes 3,000 apart, which no bf16 coefficient resolves to 2 %: they are held to the
    two-role kernel (which raises its reference as it goes) instead."""
    import paper_2211_12281_amd as kge
    G, excess = _outgrowing_case(orc, scorer, 150.0)
    assert 20 < excess < 90, excess
    _compare(orc, scorer, "sampled_softmax", G, True, 6000)
    G, excess = _outgrowing_case(orc, scorer, 3000.0)
    assert excess > 150, excess
    args = (dev_idx(G["h"]), dev_idx(G["r"]), dev_idx(G["t"]), dev_idx(G["neg"]))
    model = gpu_model(scorer, G, True)
    got = {k: v.clone() for k, v in kge.loss_bwd(model, "sampled_softmax", *args, n_ent_for_c=6000).items() if v is not None}
    kge.debug_select("two_role", True)
    try:
        want = kge.loss_bwd(model, "sampled_softmax", *args, n_ent_for_c=6000)
    finally:
        kge.debug_select("two_role", False)
    B = len(G["h"])
    ref = orc.loss_bwd(scorer, "sampled_softmax", G["ent"], G["rel"], None, G["h"], G["r"], G["t"], G["neg"], n_ent_for_c=6000)
    assert bool(torch.isfinite(got["g_ent"]).all()) and bool(torch.isfinite(got["g_rel"]).all())
    assert abs(got["loss"].item() - ref["loss"]) <= RTOL_BF16 * abs(ref["loss"])
    ge = got["g_ent"].cpu().numpy()
    assert norm_err(ge[2 * B:], ref["g_ent"][2 * B:]) <= RTOL_BF16
    errs = {"heads": norm_err(ge[:B], want["g_ent"][:B].cpu().numpy()), "tails": norm_err(ge[B:2 * B], want["g_ent"][B:2 * B].cpu().numpy()),
            "rel": norm_err(got["g_rel"].cpu().numpy(), want["g_rel"].cpu().numpy())}
    print(scorer, "second pass vs two-role kernel:", errs, "vs oracle:", norm_err(ge[:B], ref["g_ent"][:B]))
    assert max(errs.values()) <= RTOL_BF16, errs



@pytest.mark.parametrize("scorer,dim,bf16,loss,B,N", [
    ("complex", 256, True, "sampled_softmax", 300, 701),     # hot path: the gather of the negatives draws the ids
    ("transe", 256, True, "logsigmoid", 130, 260),           # two-role kernels, same gather
    ("distmult", 64, False, "sampled_softmax", 200, 333),    # fp32 tables: the draw is a launch of its own inside the call
    ("transh", 128, False, "logsigmoid", 64, 97),
    ("transe", 256, True, "logsigmoid", 0, 50),              # no queries: zero rows and the ids
    ("complex", 256, True, "sampled_softmax", 40, 0),        # no negatives: nothing is drawn
])
def test_negatives_drawn_inside_the_call_equal_the_two_calls(scorer, dim, bf16, loss, B, N):
    """kge_loss_bwd_sampled: the ids of kge_sample_negatives bit for bit, and every output of kge_loss_bwd on them
    bit for bit (same kernels on the same ids); a sub-range of the entities, and the step read from a device counter."""
    import kge_synth as ks
    import paper_2211_12281_amd as kge
    n_ent = 4000
    G = make_case(scorer, n_ent, 12, dim, max(B, 1), max(N, 1), bf16, amp=0.3, zipf=True)
    model = gpu_model(scorer, G, bf16)
    h, r, t = dev_idx(G["h"][:B]), dev_idx(G["r"][:B]), dev_idx(G["t"][:B])
    kw = _kw(scorer, loss, n_ent)
    for lo, hi, step, counter in ((0, n_ent, 5, None), (1000, 1777, 0, None), (0, n_ent, 3, 4)):
        ref_neg = kge.sample_negatives(ks.BASE_SEED, step + (counter or 0), ks.TAG_NEG, lo, hi, N)
        ref = kge.loss_bwd(model, loss, h, r, t, ref_neg, **kw)
        ref = {k: v.clone() for k, v in ref.items() if v is not None}
        neg = torch.full((N,), -1, dtype=torch.int32, device="cuda")
        draw = (ks.BASE_SEED, step, ks.TAG_NEG, lo, hi)
        if counter is not None:
            draw = draw + (torch.tensor([counter], dtype=torch.int64, device="cuda"),)
        out = kge.loss_bwd(model, loss, h, r, t, neg, draw=draw, **kw)
        assert torch.equal(neg, ref_neg), (lo, hi, step, counter)
        for k in ref:
            assert torch.equal(out[k], ref[k]), (k, lo, hi, step, counter)


def test_negatives_drawn_inside_the_call_argument_checks():
    import kge_synth as ks
    import paper_2211_12281_amd as kge
    G = make_case("complex", 500, 4, 256, 8, 8, True)
    model = gpu_model("complex", G, True)
    h, r, t = dev_idx(G["h"]), dev_idx(G["r"]), dev_idx(G["t"])
    neg = torch.zeros(8, dtype=torch.int32, device="cuda")
    for draw in ((ks.BASE_SEED, 0, ks.TAG_NEG, 10, 10), (ks.BASE_SEED, 0, ks.TAG_NEG, -1, 10), (ks.BASE_SEED, 1 << 32, ks.TAG_NEG, 0, 10),
                 (ks.BASE_SEED, 0, ks.TAG_NEG, 0, (1 << 31) + 1)):
        with pytest.raises(kge.KgeError):
            kge.loss_bwd(model, "sampled_softmax", h, r, t, neg, draw=draw, n_ent_for_c=500)


@pytest.mark.parametrize("scorer,dim,bf16,loss,B,N", [
    ("complex", 256, True, "sampled_softmax", 700, 3000),    # the sorts share the launch of the rows' finish
    ("distmult", 256, True, "sampled_softmax", 4096, 16384), # the same at the size of a full step (288 + 256 workgroups)
    ("distmult", 256, True, "logsigmoid", 300, 900),         # every other configuration: the sorts follow the call's work
    ("complex", 64, False, "sampled_softmax", 200, 333),
    ("transh", 128, False, "logsigmoid", 64, 97),
    ("complex", 256, True, "sampled_softmax", 40, 0),        # no negatives
    ("distmult", 256, True, "sampled_softmax", 0, 50),       # no queries: the relations' plan is empty
])
def test_planned_call_equals_the_sampled_call_followed_by_the_plans(scorer, dim, bf16, loss, B, N):
    """kge_loss_bwd_sampled_planned against kge_loss_bwd_sampled + kge_sparse_adam_plan_tables: every output bit for bit,
    and the plans through the updates that read them (entity rows by [h | t | drawn negatives], relation rows by r)."""
    import kge_synth as ks
    import paper_2211_12281_amd as kge
    n_ent, n_rel = 4000, 12
    G = make_case(scorer, n_ent, n_rel, dim, max(B, 1), max(N, 1), bf16, amp=0.3, zipf=True)
    model = gpu_model(scorer, G, bf16)
    h, r, t = dev_idx(G["h"][:B]), dev_idx(G["r"][:B]), dev_idx(G["t"][:B])
    kw = _kw(scorer, loss, n_ent)
    draw = (ks.BASE_SEED, 7, ks.TAG_NEG, 0, n_ent)
    k_rel = G["rel"].shape[1]
    res = {}
    for tag in ("two_calls", "planned"):
        ids = torch.full((2 * B + N,), -1, dtype=torch.int32, device="cuda")
        ids[:B] = h; ids[B:2 * B] = t
        ws_e, ws_r = kge.Workspace(), kge.Workspace()
        for w, M, d in ((ws_e, 2 * B + N, dim), (ws_r, B, k_rel)):
            w.get(kge.workspace_bytes(kge.binding.OP_SPARSE_ADAM, None, max(1, M), d)).zero_()
        plans = [(n_ent, dim, ids, ws_e), (n_rel, k_rel, r, ws_r)]
        if tag == "planned":
            out = kge.loss_bwd(model, loss, h, r, t, ids[2 * B:], draw=draw, plans=plans, **kw)
        else:
            out = kge.loss_bwd(model, loss, h, r, t, ids[2 * B:], draw=draw, **kw)
            kge.sparse_adam_plan_tables(plans)
        out = {k: v.clone() for k, v in out.items() if v is not None}
        g = torch.Generator(device="cpu").manual_seed(5)
        te = torch.randn((n_ent, dim), generator=g).cuda(); tr = torch.randn((n_rel, k_rel), generator=g).cuda()
        st = [te, torch.zeros_like(te), torch.zeros_like(te), tr, torch.zeros_like(tr), torch.zeros_like(tr)]
        kge.sparse_adam_apply_tables([(st[0], None, st[1], st[2], out["g_ent"], ws_e), (st[3], None, st[4], st[5], out["g_rel"], ws_r)],
                                     1e-2, step=2)
        torch.cuda.synchronize()
        res[tag] = (out, ids.clone(), st)
    a, b = res["two_calls"], res["planned"]
    assert torch.equal(a[1], b[1])
    for k in a[0]:
        assert torch.equal(a[0][k], b[0][k]), k
    for x, y in zip(a[2], b[2]):
        assert torch.equal(x, y)
    if B > 0 and N > 0:                                    # (no block: zero gradients, nothing moves)
        assert not torch.equal(a[2][0], torch.randn((n_ent, dim), generator=torch.Generator(device="cpu").manual_seed(5)).cuda())


def test_planned_call_rejects_the_id_arrays_it_writes_last():
    import kge_synth as ks
    import paper_2211_12281_amd as kge
    G = make_case("complex", 500, 4, 256, 8, 8, True)
    model = gpu_model("complex", G, True)
    h, r, t = dev_idx(G["h"]), dev_idx(G["r"]), dev_idx(G["t"])
    neg = torch.zeros(8, dtype=torch.int32, device="cuda")
    out = kge.loss_bwd(model, "sampled_softmax", h, r, t, neg, draw=(ks.BASE_SEED, 0, ks.TAG_NEG, 0, 500), n_ent_for_c=500)
    with pytest.raises(kge.KgeError):
        kge.loss_bwd(model, "sampled_softmax", h, r, t, neg, draw=(ks.BASE_SEED, 0, ks.TAG_NEG, 0, 500), n_ent_for_c=500, out=out,
                     plans=[(500, 256, out["g_ent_idx"], kge.Workspace())])
