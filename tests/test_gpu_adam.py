"""kge_sparse_adam against the oracle: duplicate-aware scatter-add and the lazy Adam step."""
import numpy as np
import pytest
import torch

import kge_synth as ks
from helpers import RTOL_F32, norm_err

pytestmark = pytest.mark.gpu
F = np.float32


def update_err_ok(got_new, old, ref_new):
    """The UPDATE theta_new - theta_old must match the oracle's to RTOL_F32 of its largest entry, plus
    the rounding of the fp32 master itself: the kernel stores theta_new in fp32 (half an ulp of
    theta, which can exceed 1e-5 of a 1e-3-sized update), the oracle keeps it in fp64."""
    got_upd = got_new.astype(np.float64) - old
    ref_upd = ref_new - old
    allowed = RTOL_F32 * np.max(np.abs(ref_upd)) + np.spacing(np.abs(got_new).astype(F)).astype(np.float64)
    return bool(np.all(np.abs(got_upd - ref_upd) <= allowed))


def _state(n_rows, d, seed, warm):
    g = np.random.default_rng(seed)
    theta = g.normal(size=(n_rows, d)).astype(F) * F(0.1)
    if warm:
        m = (g.normal(size=(n_rows, d)) * 1e-3).astype(F)
        v = (g.normal(size=(n_rows, d)) ** 2 * 1e-5).astype(F)
    else:
        m = np.zeros((n_rows, d), F); v = np.zeros((n_rows, d), F)
    return theta, m, v


def _check(orc, n_rows, d, M, step, warm, shadow, zipf=True, seed=0, lr=1e-3):
    import paper_2211_12281_amd as kge
    theta, m, v = _state(n_rows, d, seed, warm)
    g = np.random.default_rng(seed + 100)
    idx = ks.ZipfIds(n_rows, 1.1).draw(g, M) if zipf else g.integers(0, n_rows, M).astype(np.int32)
    grads = (g.normal(size=(M, d)) * 1e-2).astype(F)
    b1, b2, eps = float(F(0.9)), float(F(0.999)), float(F(1e-8))
    lr = float(F(lr))
    dth, dm, dv = [torch.from_numpy(a.copy()).cuda() for a in (theta, m, v)]
    dsh = torch.zeros((n_rows, d), dtype=torch.bfloat16, device="cuda") if shadow else None
    kge.sparse_adam(dth, dsh, dm, dv, torch.from_numpy(idx).cuda(), torch.from_numpy(grads).cuda(), lr, b1, b2, eps, step)
    rth, rm, rv, touched = orc.sparse_adam(theta, m, v, idx, grads, lr, b1, b2, eps, step)
    gth, gm, gv = dth.cpu().numpy(), dm.cpu().numpy(), dv.cpu().numpy()
    # untouched rows: bit-identical to the input
    assert np.array_equal(gth[~touched], theta[~touched]) and np.array_equal(gm[~touched], m[~touched])
    assert np.array_equal(gv[~touched], v[~touched])
    if M == 0:
        return
    # touched rows: compare the UPDATE, not the value (lr would hide errors otherwise)
    assert update_err_ok(gth[touched], theta[touched], rth[touched])
    assert norm_err(gm[touched], rm[touched]) <= RTOL_F32
    assert norm_err(gv[touched], rv[touched]) <= RTOL_F32
    if shadow:
        sh = dsh.view(torch.int16).cpu().numpy().view(np.uint16)
        # the shadow is RNE(theta_new) of the fp32 master the kernel itself wrote: bit-exact
        assert np.array_equal(sh[touched], orc.bf16_rne(gth[touched]))
        assert np.all(sh[~touched] == 0)
        ref_sh = ks.bf16_bits_to_f32(orc.bf16_rne(rth[touched].astype(F)))
        assert norm_err(ks.bf16_bits_to_f32(sh[touched]), ref_sh) <= 2.0 ** -7


@pytest.mark.parametrize("n_rows,d,M", [(1000, 32, 192), (50000, 256, 24576), (300, 128, 5000), (70000, 64, 1),
                                         (1 << 20, 16, 3000), (40, 4, 1025)])
def test_update_matches_oracle(orc, n_rows, d, M):
    _check(orc, n_rows, d, M, step=7, warm=True, shadow=False)


def test_first_step_from_zero_state(orc):
    _check(orc, 2000, 32, 500, step=1, warm=False, shadow=False, zipf=False)


def test_bf16_shadow(orc):
    _check(orc, 20000, 256, 6000, step=3, warm=True, shadow=True)


def test_all_indices_equal_and_empty(orc):
    import paper_2211_12281_amd as kge
    theta, m, v = _state(50, 64, 3, True)
    idx = np.full(700, 17, np.int32)
    grads = (np.random.default_rng(5).normal(size=(700, 64)) * 1e-2).astype(F)
    dth, dm, dv = [torch.from_numpy(a.copy()).cuda() for a in (theta, m, v)]
    kge.sparse_adam(dth, None, dm, dv, torch.from_numpy(idx).cuda(), torch.from_numpy(grads).cuda(), 1e-3, step=2)
    rth, rm, rv, touched = orc.sparse_adam(theta, m, v, idx, grads, float(F(1e-3)), float(F(0.9)), float(F(0.999)),
                                           float(F(1e-8)), 2)
    assert touched.sum() == 1
    assert update_err_ok(dth.cpu().numpy()[17], theta[17], rth[17])
    _check(orc, 100, 8, 0, step=1, warm=True, shadow=False)


@pytest.mark.parametrize("runs", [[(17, 6000)], [(3, 2500), (41, 2300)], [(0, 31), (9, 2049), (30, 33), (49, 2047)]])
def test_long_runs_of_equal_ids(orc, runs):
    """Runs of equal ids far longer than the 64 chunks x 32 positions that the wave of a run's first chunk probes per
    round (the continuation of that search), alone and side by side, starting at positions that straddle chunk
    boundaries; against the oracle, and bit-identical from call to call."""
    import paper_2211_12281_amd as kge
    theta, m, v = _state(50, 64, 3, True)
    idx = np.concatenate([np.full(n, row, np.int32) for row, n in runs])
    M = idx.size
    grads = (np.random.default_rng(5).normal(size=(M, 64)) * 1e-2).astype(F)
    outs = []
    for _ in range(2):
        dth, dm, dv = [torch.from_numpy(a.copy()).cuda() for a in (theta, m, v)]
        kge.sparse_adam(dth, None, dm, dv, torch.from_numpy(idx).cuda(), torch.from_numpy(grads).cuda(), 1e-3, step=2)
        outs.append((dth.cpu().numpy(), dm.cpu().numpy(), dv.cpu().numpy()))
    assert all(np.array_equal(a, b) for a, b in zip(*outs))
    rth, rm, rv, touched = orc.sparse_adam(theta, m, v, idx, grads, float(F(1e-3)), float(F(0.9)), float(F(0.999)),
                                           float(F(1e-8)), 2)
    assert touched.sum() == len(runs)
    gth, gm, gv = outs[0]
    assert np.array_equal(gth[~touched], theta[~touched])
    assert update_err_ok(gth[touched], theta[touched], rth[touched])
    assert norm_err(gm[touched], rm[touched]) <= RTOL_F32 and norm_err(gv[touched], rv[touched]) <= RTOL_F32


@pytest.mark.parametrize("n_rows", [4096, 65536, 1 << 21])
def test_one_list_of_several_long_runs(orc, n_rows):
    """Ids that all fall into ONE list of the one-launch sort (the same low byte), longer than the list kept in LDS, with
    two long runs and hundreds of other ids - no single id to split off leaves a short remainder, so the list is ordered
    by counting passes over the output buffers (an odd and an even number of them, by the width of the ids)."""
    import paper_2211_12281_amd as kge
    g = np.random.default_rng(77)
    same_byte = 5 + 256 * np.arange(n_rows // 256)
    others = g.choice(same_byte[2:], 700)
    idx = np.concatenate([np.full(1900, same_byte[0]), others[:350], np.full(2100, same_byte[1]), others[350:]]).astype(np.int32)
    idx = idx[g.permutation(idx.size)]
    d = 32
    theta, m, v = _state(n_rows, d, 5, True)
    grads = (g.normal(size=(idx.size, d)) * 1e-2).astype(F)
    dth, dm, dv = [torch.from_numpy(a.copy()).cuda() for a in (theta, m, v)]
    kge.sparse_adam(dth, None, dm, dv, torch.from_numpy(idx).cuda(), torch.from_numpy(grads).cuda(), 1e-3, step=3)
    rth, rm, rv, touched = orc.sparse_adam(theta, m, v, idx, grads, float(F(1e-3)), float(F(0.9)), float(F(0.999)), float(F(1e-8)), 3)
    gth, gm, gv = dth.cpu().numpy(), dm.cpu().numpy(), dv.cpu().numpy()
    assert np.array_equal(gth[~touched], theta[~touched])
    assert update_err_ok(gth[touched], theta[touched], rth[touched])
    assert norm_err(gm[touched], rm[touched]) <= RTOL_F32 and norm_err(gv[touched], rv[touched]) <= RTOL_F32


def test_padded_row_stride(orc):
    """Tables whose row stride exceeds dim (ld > dim): padding columns stay untouched."""
    import paper_2211_12281_amd as kge
    n_rows, d, ld, M = 500, 24, 32, 300
    g = np.random.default_rng(11)
    full = [g.normal(size=(n_rows, ld)).astype(F) * F(0.1) for _ in range(2)] + [(g.normal(size=(n_rows, ld)) ** 2 * 1e-4).astype(F)]
    dev = [torch.from_numpy(a.copy()).cuda() for a in full]
    idx = g.integers(0, n_rows, M).astype(np.int32)
    grads = (g.normal(size=(M, d)) * 1e-2).astype(F)
    kge.sparse_adam(dev[0][:, :d], None, dev[1][:, :d], dev[2][:, :d], torch.from_numpy(idx).cuda(),
                    torch.from_numpy(grads).cuda(), 1e-3, step=4)
    rth, _, _, touched = orc.sparse_adam(full[0][:, :d], full[1][:, :d], full[2][:, :d], idx, grads, float(F(1e-3)),
                                         float(F(0.9)), float(F(0.999)), float(F(1e-8)), 4)
    got = dev[0].cpu().numpy()
    assert np.array_equal(got[:, d:], full[0][:, d:])
    assert update_err_ok(got[touched, :d], full[0][touched, :d], rth[touched])


def test_result_does_not_depend_on_scheduling(orc):
    import paper_2211_12281_amd as kge
    theta, m, v = _state(3000, 64, 9, True)
    g = np.random.default_rng(10)
    idx = ks.ZipfIds(3000, 1.1).draw(g, 8000)
    grads = (g.normal(size=(8000, 64)) * 1e-2).astype(F)
    outs = []
    for _ in range(3):
        dth, dm, dv = [torch.from_numpy(a.copy()).cuda() for a in (theta, m, v)]
        kge.sparse_adam(dth, None, dm, dv, torch.from_numpy(idx).cuda(), torch.from_numpy(grads).cuda(), 1e-3, step=5)
        outs.append(dth.cpu().numpy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_plan_on_a_side_stream_then_apply_is_bitwise_the_single_call():
    """kge_sparse_adam_plan (row ids only) on a second stream, kge_sparse_adam_apply on the main one, ordered by an
    event: the same bits as kge_sparse_adam, also when the planned workspace is reused step after step."""
    import paper_2211_12281_amd as kge
    n_rows, d, M = 50000, 64, 7000
    g = np.random.default_rng(5)
    side = torch.cuda.Stream()
    ws = kge.Workspace()
    ref = [torch.from_numpy(x).cuda() for x in _state(n_rows, d, 3, True)]
    two = [x.clone() for x in ref]
    sh_ref = ref[0].to(torch.bfloat16); sh_two = sh_ref.clone()
    for step in (1, 2, 3):
        idx = torch.from_numpy(ks.ZipfIds(n_rows, 1.1).draw(g, M)).cuda()
        grads = torch.from_numpy((g.normal(size=(M, d)) * 1e-2).astype(F)).cuda()
        kge.sparse_adam(ref[0], sh_ref, ref[1], ref[2], idx, grads, 1e-3, step=step)
        start, planned = torch.cuda.Event(), torch.cuda.Event()
        start.record()
        with torch.cuda.stream(side):
            side.wait_event(start)                       # the ids exist, the previous apply is done with the workspace
            kge.sparse_adam_plan(n_rows, d, idx, ws)
            planned.record()
        torch.cuda.current_stream().wait_event(planned)
        kge.sparse_adam_apply(two[0], sh_two, two[1], two[2], grads, ws, 1e-3, step=step)
    torch.cuda.synchronize()
    for a, b in zip(ref + [sh_ref], two + [sh_two]):
        assert bool((a == b).all())


def test_streams_passed_as_arguments_give_the_same_bits():
    """The binding takes the stream of a call as an argument (no stream context on the host): plan on a side stream,
    apply on the main one, both named explicitly, against the single call on the current stream; with the kernels of
    the update bracketed by the library's events on the given stream."""
    import paper_2211_12281_amd as kge
    n_rows, d, M = 30000, 128, 5000
    g = np.random.default_rng(11)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    ws = kge.Workspace()
    ref = [torch.from_numpy(x).cuda() for x in _state(n_rows, d, 3, True)]
    two = [x.clone() for x in ref]
    ev_ids, ev_plan = torch.cuda.Event(), torch.cuda.Event()
    kge.profile_enable(["adam"])
    for step in (1, 2):
        idx = torch.from_numpy(ks.ZipfIds(n_rows, 1.1).draw(g, M)).cuda()
        grads = torch.from_numpy((g.normal(size=(M, d)) * 1e-2).astype(F)).cuda()
        kge.sparse_adam(ref[0], None, ref[1], ref[2], idx, grads, 1e-3, step=step)
        ev_ids.record(main)
        side.wait_event(ev_ids)
        kge.sparse_adam_plan(n_rows, d, idx, ws, stream=side)
        ev_plan.record(side)
        main.wait_event(ev_plan)
        kge.sparse_adam_apply(two[0], None, two[1], two[2], grads, ws, 1e-3, step=step, stream=main)
    torch.cuda.synchronize()
    kge.profile_enable(False)
    ms, n = kge.profile_collect("adam")
    assert n == 4 and ms > 0.0                 # two single calls + two applies; the plans belong to the slot "sort"
    assert kge.profile_collect("sort")[1] == 0  # (not selected)
    for a, b in zip(ref, two):
        assert bool((a == b).all())



def test_several_tables_in_one_call_give_the_bits_of_one_call_per_table():
    """kge_sparse_adam_apply_tables (the entity table and the small relation tables of a step in two launches) against
    kge_sparse_adam_apply table by table; one table of the set is empty, one has a single row id repeated."""
    import paper_2211_12281_amd as kge
    shapes = [(50000, 256, 24576, True), (1000, 128, 4096, True), (1000, 256, 0, False), (7, 64, 300, False)]
    dev = lambda a: torch.from_numpy(a.copy()).cuda()
    sets = []
    for k, (n_rows, d, M, shadow) in enumerate(shapes):
        theta, m, v = _state(n_rows, d, 40 + k, True)
        g = np.random.default_rng(140 + k)
        idx = ks.ZipfIds(n_rows, 1.1).draw(g, M) if k != 3 else np.full(M, 5, np.int32)
        grads = (g.normal(size=(M, d)) * 1e-2).astype(F)
        one = {"idx": dev(idx), "grads": dev(grads)}
        for tag in ("ref", "got"):
            one[tag] = [dev(theta), dev(m), dev(v)]
            one[tag + "_sh"] = torch.zeros((n_rows, d), dtype=torch.bfloat16, device="cuda") if shadow else None
            one[tag + "_ws"] = kge.Workspace()
        sets.append(one)
    for s, (n_rows, d, M, _) in zip(sets, shapes):
        if M:
            kge.sparse_adam_plan(n_rows, d, s["idx"], s["ref_ws"])
            kge.sparse_adam_apply(s["ref"][0], s["ref_sh"], s["ref"][1], s["ref"][2], s["grads"], s["ref_ws"], 2e-3, step=7)
            kge.sparse_adam_plan(n_rows, d, s["idx"], s["got_ws"])
    kge.sparse_adam_apply_tables([(s["got"][0], s["got_sh"], s["got"][1], s["got"][2], s["grads"], s["got_ws"]) for s in sets],
                                 2e-3, step=7)
    torch.cuda.synchronize()
    for s in sets:
        for a, c in zip(s["ref"], s["got"]):
            assert bool((a == c).all())
        if s["ref_sh"] is not None:
            assert bool((s["ref_sh"].view(torch.int16) == s["got_sh"].view(torch.int16)).all())
    assert not bool((sets[0]["got"][0] == dev(_state(50000, 256, 40, True)[0])).all())     # something was updated


@pytest.mark.parametrize("shapes", [
    [(10_000_000, 64, 24576, "zipf"), (1000, 64, 9000, "same"), (200, 64, 4096, "zipf"), (77, 64, 0, "zipf")],
    [(10_000_000, 64, 24576, "zipf"), (1000, 64, 4096, "zipf")],          # entities and relations of a training step
    [(200, 64, 4096, "zipf"), (10_000_000, 64, 24576, "zipf"), (1000, 64, 100, "zipf"), (5000, 64, 8193, "zipf")],
], ids=["long-same-short-empty", "entities-relations", "short-long-short-long"])
def test_plans_of_several_tables_in_one_call_equal_one_call_per_table(shapes):
    """kge_sparse_adam_plan_tables against kge_sparse_adam_plan table by table, through the updates that read the plans:
    a long Zipf list, a list of one repeated id (longer than the list a workgroup orders in one step), a short list over
    few rows (no bits left to order by), an empty one; short and long lists in either order."""
    import paper_2211_12281_amd as kge
    dev = lambda a: torch.from_numpy(a.copy()).cuda()
    sets = []
    for k, (n_rows, d, M, kind) in enumerate(shapes):
        g = np.random.default_rng(240 + k)
        idx = ks.ZipfIds(n_rows, 1.1).draw(g, M) if kind == "zipf" else np.full(M, 777, np.int32)
        touched = np.unique(idx)
        rows = min(n_rows, 70000)                          # (the big table: only ids below 70,000 are kept)
        idx = idx[idx < rows] if n_rows > rows else idx
        M = idx.size
        theta, m, v = _state(rows, d, 340 + k, True)
        grads = (g.normal(size=(M, d)) * 1e-2).astype(F)
        one = {"idx": dev(idx), "grads": dev(grads), "n_rows": n_rows, "d": d}
        for tag in ("ref", "got"):
            one[tag] = [dev(theta), dev(m), dev(v)]
            one[tag + "_ws"] = kge.Workspace()
        sets.append(one)
    for s in sets:
        # (the workspaces start cleared, so that nothing a call leaves unsorted can pass for sorted: position 0 everywhere)
        for tag in ("ref_ws", "got_ws"):
            s[tag].get(kge.workspace_bytes(kge.binding.OP_SPARSE_ADAM, None, max(1, s["idx"].numel()), s["d"])).zero_()
        if s["idx"].numel():
            kge.sparse_adam_plan(s["n_rows"], s["d"], s["idx"], s["ref_ws"])
            kge.sparse_adam_apply(s["ref"][0], None, s["ref"][1], s["ref"][2], s["grads"], s["ref_ws"], 2e-3, step=3)
    kge.sparse_adam_plan_tables([(s["n_rows"], s["d"], s["idx"], s["got_ws"]) for s in sets])
    kge.sparse_adam_apply_tables([(s["got"][0], None, s["got"][1], s["got"][2], s["grads"], s["got_ws"]) for s in sets], 2e-3, step=3)
    torch.cuda.synchronize()
    for s in sets:
        for a, c in zip(s["ref"], s["got"]):
            assert bool((a == c).all())
