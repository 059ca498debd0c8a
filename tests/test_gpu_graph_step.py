"""A whole training step (Section 4, "Training": sample the shared negatives, score, back-propagate, update) recorded
once into a HIP graph and replayed: the step number comes from a counter in device memory (kge_step_counter_add,
kge_sample_negatives_dev, kge_adam_cfg_t.step_counter).  Every replay must leave the tables with the bits of the same
step run call by call, with the program's own eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import kge_synth as ks
from helpers import make_case

pytestmark = pytest.mark.gpu


def _tables(G, bf16):
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    T = {}
    for name in ("ent", "rel"):
        p = dev(G[name])
        T[name] = {"p": p, "m": torch.zeros_like(p), "v": torch.zeros_like(p), "sh": p.to(torch.bfloat16) if bf16 else None}
    return T


def _model(kge, scorer, T, bf16):
    tbl = lambda q: q["sh"] if bf16 else q["p"]
    return kge.Model(scorer, tbl(T["ent"]), tbl(T["rel"]))


@pytest.mark.parametrize("fused", [False, True])     # the negatives from a call of their own / drawn inside kge_loss_bwd_sampled
@pytest.mark.parametrize("scorer,d,bf16,loss", [("complex", 256, True, "sampled_softmax"), ("distmult", 64, False, "logsigmoid")])
def test_replays_of_a_captured_step_match_the_step_run_call_by_call(scorer, d, bf16, loss, fused):
    import paper_2211_12281_amd as kge
    n_ent, n_rel, B, N, steps = 6000, 12, 512, 1024, 4
    G = make_case(scorer, n_ent, n_rel, d, B, N, bf16, amp=0.3)
    h, r, t = (torch.from_numpy(G[k]).cuda() for k in ("h", "r", "t"))
    kw = dict(n_ent_for_c=n_ent) if loss == "sampled_softmax" else dict(gamma=6.0, adv_temp=1.0)
    lr = 1e-2

    def out_buffers(model):
        return {"loss": torch.empty(1, device="cuda"), "g_ent": torch.empty((2 * B + N, d), device="cuda"),
                "g_ent_idx": torch.empty(2 * B + N, dtype=torch.int32, device="cuda"),
                "g_rel": torch.empty((B, model.rel.shape[1]), device="cuda"), "g_relw": None,
                "g_rel_idx": torch.empty(B, dtype=torch.int32, device="cuda")}

    # call by call
    Te = _tables(G, bf16)
    me = _model(kge, scorer, Te, bf16)
    oe = out_buffers(me)
    neg = torch.empty(N, dtype=torch.int32, device="cuda")
    want = []
    for i in range(steps):
        kge.sample_negatives(ks.BASE_SEED, 5 + i, ks.TAG_NEG, 0, n_ent, N, out=neg)
        kge.loss_bwd(me, loss, h, r, t, neg, out=oe, **kw)
        for name, gi, gg in (("ent", "g_ent_idx", "g_ent"), ("rel", "g_rel_idx", "g_rel")):
            q = Te[name]
            kge.sparse_adam(q["p"], q["sh"], q["m"], q["v"], oe[gi], oe[gg], lr, step=1 + i)
        torch.cuda.synchronize()
        want.append({"loss": oe["loss"].clone(), "neg": neg.clone(), "ent": Te["ent"]["p"].clone(), "rel": Te["rel"]["p"].clone(),
                     "ent_v": Te["ent"]["v"].clone(), "sh": Te["ent"]["sh"].clone() if bf16 else None})

    # recorded once, replayed
    Tg = _tables(G, bf16)
    mg = _model(kge, scorer, Tg, bf16)
    og = out_buffers(mg)
    negg = torch.empty(N, dtype=torch.int32, device="cuda")
    counter = torch.zeros(1, dtype=torch.int64, device="cuda")
    ws = [kge.Workspace() for _ in range(3)]

    def one_step():
        if fused:
            kge.loss_bwd(mg, loss, h, r, t, negg, out=og, ws=ws[0], draw=(ks.BASE_SEED, 5, ks.TAG_NEG, 0, n_ent, counter), **kw)
        else:
            kge.sample_negatives_dev(ks.BASE_SEED, counter, 5, ks.TAG_NEG, 0, n_ent, N, out=negg)
            kge.loss_bwd(mg, loss, h, r, t, negg, out=og, ws=ws[0], **kw)
        for j, (name, gi, gg) in enumerate((("ent", "g_ent_idx", "g_ent"), ("rel", "g_rel_idx", "g_rel"))):
            q = Tg[name]
            kge.sparse_adam(q["p"], q["sh"], q["m"], q["v"], og[gi], og[gg], lr, step=1, ws=ws[1 + j], step_counter=counter)
        kge.step_counter_add(counter, 1)

    # warm-up on scratch copies of the state (sizes the workspaces), then put the state back
    keep = {n: {k: (v.clone() if v is not None else None) for k, v in Tg[n].items()} for n in Tg}
    one_step()
    torch.cuda.synchronize()
    for n in Tg:
        for k, v in Tg[n].items():
            if v is not None:
                v.copy_(keep[n][k])
    counter.zero_()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_step()
    # (capture runs nothing: the tables and the counter are as before)
    assert int(counter.item()) == 0
    for i in range(steps):
        graph.replay()
        torch.cuda.synchronize()
        assert int(counter.item()) == i + 1
        assert bool((negg == want[i]["neg"]).all())
        assert bool((og["loss"] == want[i]["loss"]).all())
        assert bool((Tg["ent"]["p"] == want[i]["ent"]).all()) and bool((Tg["rel"]["p"] == want[i]["rel"]).all())
        assert bool((Tg["ent"]["v"] == want[i]["ent_v"]).all())
        if bf16:
            assert bool((Tg["ent"]["sh"].view(torch.int16) == want[i]["sh"].view(torch.int16)).all())
        # the program's own eager work between the replays: another call of the library on its default workspace
        kge.score(mg, h[:64], r[:64], t[:64], negg[:128])
        torch.cuda.synchronize()


def test_negatives_of_a_device_counter_equal_those_of_the_step_number():
    import paper_2211_12281_amd as kge
    counter = torch.zeros(1, dtype=torch.int64, device="cuda")
    for c, off in ((0, 0), (7, 3), (2 ** 31, 2 ** 31 - 1)):
        counter.fill_(c)
        a = kge.sample_negatives_dev(ks.BASE_SEED, counter, off, ks.TAG_NEG, 10, 9_000_001, 4097)
        b = kge.sample_negatives(ks.BASE_SEED, c + off, ks.TAG_NEG, 10, 9_000_001, 4097)
        assert bool((a == b).all())
    kge.step_counter_add(counter, 5)
    assert int(counter.item()) == 2 ** 31 + 5
