"""Shared test utilities: error measures and small input builders (no method arithmetic)."""
import numpy as np

import kge_synth as ks

RTOL_F32 = 1e-5   # per-tensor normalised error bound for fp32 paths
RTOL_BF16 = 2e-2  # same for bf16 compute


def norm_err(x, ref):
    """max_i |x_i - ref_i| / max(max_i |ref_i|, tiny): the per-tensor normalised error."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape, (x.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(x)), "non-finite values in result"
    return float(np.max(np.abs(x - ref)) / max(float(np.max(np.abs(ref))), 1e-300))


def row_norm_err(x, ref, floor_frac=1.0 / 32):
    """Per-ROW normalised error: max over rows of max_j |x - ref| / max(max_j |ref_row|, floor_frac * max |ref|).  Rows
    whose entries are small beside the tensor's largest are held to their own magnitude, down to the floor (an element
    of a gradient row is a sum of terms of the size of the tensor's typical entry: below 1/32 of the largest entry a
    row is mostly cancellation and its relative error says nothing)."""
    x = np.asarray(x, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape and x.ndim == 2
    if ref.size == 0:
        return 0.0
    top = max(float(np.max(np.abs(ref))), 1e-300)
    den = np.maximum(np.max(np.abs(ref), axis=1), floor_frac * top)
    return float(np.max(np.max(np.abs(x - ref), axis=1) / den))


def small_graph(scorer, n_ent=1000, n_rel=10, dim=32, B=64, N=64, seed=ks.BASE_SEED, amp=0.1,
                grid_bits=None, normal=False):
    """Tables and one micro-batch on a small graph.  grid_bits quantises table values to
    multiples of 2^-grid_bits so that finite-difference steps are exactly representable."""
    if normal:
        ent = ks.normal_table(seed, ks.TAG_ENT, n_ent, dim, amp)
    else:
        ent = ks.uniform_table(seed, ks.TAG_ENT, n_ent, dim, amp)
    rel, relw = ks.relation_tables(scorer.replace("_l1", ""), n_rel, dim, seed, amp)   # same tables for both norms
    if grid_bits is not None:
        q = float(1 << grid_bits)
        ent = (np.round(ent * q) / q).astype(np.float32)
        rel = (np.round(rel * q) / q).astype(np.float32)
        if relw is not None:
            relw = (np.round(relw * q) / q).astype(np.float32)
    g = ks.rng(seed, ks.TAG_BATCH)
    h = ks.uniform_ids(g, 0, n_ent, B)
    r = ks.uniform_ids(g, 0, n_rel, B)
    t = ks.uniform_ids(g, 0, n_ent, B)
    neg = ks.uniform_ids(ks.rng(seed, ks.TAG_NEG), 0, n_ent, N)
    return dict(ent=ent, rel=rel, relw=relw, h=h, r=r, t=t, neg=neg)


# ---------------------------------------------------------------------------------------------
# GPU-side helpers (imported lazily by the gpu tests)
# ---------------------------------------------------------------------------------------------
def to_dev(a, bf16=False):
    """numpy fp32 array -> device tensor; for bf16 the values must already be bf16-representable."""
    import torch
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32 and bf16:
        bits = ks.f32_to_bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def make_case(scorer, n_ent, n_rel, dim, B, N, bf16, seed=ks.BASE_SEED, amp=0.1, zipf=False):
    """Tables (host fp32 values, already rounded to bf16 when bf16=True) and a micro-batch."""
    G = small_graph(scorer, n_ent, n_rel, dim, B, N, seed=seed, amp=amp)
    if zipf:
        z = ks.ZipfIds(n_ent, 1.1)
        g = ks.rng(seed, ks.TAG_BATCH, 1)
        G["h"], G["t"] = z.draw(g, B), z.draw(g, B)
    if bf16:
        for k in ("ent", "rel", "relw"):
            if G[k] is not None:
                G[k] = ks.round_to_bf16(G[k])
    return G


def gpu_model(scorer, G, bf16):
    import paper_2211_12281_amd as kge
    return kge.Model(scorer, to_dev(G["ent"], bf16), to_dev(G["rel"], bf16), to_dev(G["relw"], bf16))


def dev_idx(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def rank_band_eps(scorer, ent_h, rel_r, relw_r, bf16, t_max):
    """Per query, twice the documented error bound of the matrix-core value that kge_topk compares beyond the list (in
    units of the ranking key: -score for DistMult / ComplEx, squared distance for the distance scorers).  The held-out
    tail's value and a candidate's value are each within that bound of the exact key, so the reported rank can differ
    from the exact one only by candidates whose exact key lies within the returned eps of the tail's.
    ent_h, rel_r, relw_r: the queries' head / relation / normal rows (fp64-able arrays); t_max: largest candidate norm.
    Bounds (d columns, u = rounding unit of the table type, dq = rounding of the query to the table type):
      bilinear   eps = (|dq| + d 2^-23 |q|) Tmax
      distance   eps = 2 |dq| (|q| + Tmax) + |dq|^2 + (d + 2) 2^-22 (|q| + Tmax)^2
      TransH     adds, for x = w.t - c:  dx (2 xmax + dx) + 2^-21 (xmax^2 + (|q| + Tmax)^2) + dc (2 |c| + dc)."""
    h = np.asarray(ent_h, np.float64); r = np.asarray(rel_r, np.float64)
    d = h.shape[1]
    u = (2.0 ** -9 if bf16 else 2.0 ** -24) + 2.0 ** -20        # rounding to the table type + fp32 evaluation of the query
    if scorer == "distmult":
        qn = np.linalg.norm(h * r, axis=1)
    elif scorer == "complex":
        k = d // 2
        qn = np.linalg.norm((h[:, :k] + 1j * h[:, k:]) * (r[:, :k] + 1j * r[:, k:]), axis=1)
    elif scorer == "transe":
        qn = np.linalg.norm(h + r, axis=1)
    elif scorer == "rotate":
        qn = np.linalg.norm(h, axis=1)
    else:
        qn = np.linalg.norm(h, axis=1) + np.linalg.norm(r, axis=1)      # |q'| <= |h| + |r|
    qn = qn * (1.0 + u)
    dq = u * qn
    if scorer in ("distmult", "complex"):
        eps = (dq + d * 2.0 ** -23 * qn) * t_max
    else:
        s = qn + t_max
        eps = 2.0 * dq * s + dq * dq + (d + 2) * 2.0 ** -22 * s * s
        if scorer == "transh":
            c, dw = qn, u * (1.0 + u)                                    # |c| = |u.q'| <= |q'|; rounding of the unit normal
            dc = dq + 2.0 ** -23 * c
            dx = (dw + d * 2.0 ** -23 * (1.0 + dw)) * t_max + dc
            xm = (1.0 + dw) * t_max * 1.0001 + c
            eps = eps + dx * (2.0 * xm + dx) + 2.0 ** -21 * (xm * xm + s * s) + dc * (2.0 * c + dc)
    return 2.0 * 1.01 * eps + 1e-30


def l1_sign_flips_justified(orc, scorer, loss, ent, rel, relw, h, r, t, neg, kw, got, ref, tol, max_checked=None):
    """1-norm scorers: the gradient is discontinuous where a coordinate x_j of the difference vector crosses zero, and
    the kernels evaluate x in fp32 while the oracle uses fp64, so a coordinate within fp32 rounding of zero may take
    the other sign.  Every gradient element that deviates from the oracle by more than tol (normalised by the tensor's
    largest entry) must be explained that way, FROM THE ORACLE'S SIDE: the pairs (b, n) that feed the element's row
    must hold coordinates with |x_j| <= band (band = 2^-18 of the largest table entry: 64 fp32 roundings; TransH 2^-16),
    and the
    deviation must not exceed c |dL/dS(b, n)| summed over those coordinates (c = 2 for an element that takes the sign
    directly; the rotation of RotatE and the projections of TransH spread a flipped sign over other columns with
    factors bounded by the operands' magnitudes).  An outlier with no such coordinate fails.
    got / ref: dicts with g_ent [(2B+N), d], g_rel, (g_relw).  Returns the number of outlying elements."""
    f8 = np.float64
    ent, rel = np.asarray(ent, f8), np.asarray(rel, f8)
    B, N, d = len(h), len(neg), ent.shape[1]
    k = d // 2
    pos, S = orc.score_batch(scorer + "_l1", ent, rel, relw, h, r, t, neg)
    scale = kw.get("loss_scale") or 1.0 / max(B, 1)
    if loss == "logsigmoid":
        a, gamma = kw.get("adv_temp", 0.0), kw.get("gamma", 0.0)
        w = np.exp(a * (S - S.max(axis=1, keepdims=True))) if N else S
        w = w / w.sum(axis=1, keepdims=True) if N else w
        Gn = scale * w / (1.0 + np.exp(-(gamma + S)))
        gp = -scale / (1.0 + np.exp(gamma + pos))
    else:
        c = np.log((kw["n_ent_for_c"] - 1) / N) if N else 0.0
        z = np.concatenate([pos[:, None], S + c], axis=1)
        p = np.exp(z - z.max(axis=1, keepdims=True)); p = p / p.sum(axis=1, keepdims=True)
        Gn, gp = scale * p[:, 1:], scale * (p[:, 0] - 1.0)
    H, R, T, TN = ent[h], rel[r], ent[t], ent[neg]
    if scorer == "transe":
        Qv, Wv = H + R, None
    elif scorer == "rotate":
        q = (H[:, :k] + 1j * H[:, k:]) * np.exp(1j * R)
        Qv, Wv = np.concatenate([q.real, q.imag], axis=1), None
    else:
        Wv = np.asarray(relw, f8)[r]
        Wv = Wv / np.maximum(np.linalg.norm(Wv, axis=1, keepdims=True), 1e-12)
        Qv = H - np.sum(Wv * H, axis=1, keepdims=True) * Wv + R
    def xvec(b, tails):                       # difference vectors of query b against the given tail rows [m, d]
        if Wv is None:
            return Qv[b][None, :] - tails
        return Qv[b][None, :] - tails + (tails @ Wv[b])[:, None] * Wv[b][None, :]
    big = max(float(np.abs(ent).max()), float(np.abs(rel).max()), 1e-30)
    # (TransH's x passes through two fp32 dot products over the d columns: four times the band)
    band = (2.0 ** -16 if scorer == "transh" else 2.0 ** -18) * big
    spread = 2.0 if scorer != "transh" else 8.0 * (1.0 + float(np.linalg.norm(ent[np.r_[h, t, neg]], axis=1).max()))
    if scorer == "rotate":
        spread = 2.0 * np.sqrt(2.0) * max(1.0, big * np.sqrt(2.0))
    def coords(j, is_rel):                    # coordinates whose sign can move column j
        if scorer == "transe":
            return [j]
        if scorer == "rotate":
            return [j % k, j % k + k]
        return None                           # TransH: every coordinate (through P = sign(x) . w)
    def near_zero(x, cs):
        xs = x if cs is None else x[:, cs]
        return np.sum(np.abs(xs) <= band, axis=1)
    tensors = [("g_head", got["g_ent"][:B], ref["g_ent"][:B], "head"), ("g_tail", got["g_ent"][B:2 * B], ref["g_ent"][B:2 * B], "tail"),
               ("g_neg", got["g_ent"][2 * B:], ref["g_ent"][2 * B:], "neg"), ("g_rel", got["g_rel"], ref["g_rel"], "head")]
    if ref.get("g_relw") is not None:
        tensors.append(("g_relw", got["g_relw"], ref["g_relw"], "head"))
    n_out = 0
    for name, x, rf, kind in tensors:
        if rf.size == 0:
            continue
        top = max(float(np.max(np.abs(rf))), 1e-300)
        dev = np.abs(np.asarray(x, f8) - rf)
        out = np.argwhere(dev > tol * top)
        n_out += len(out)
        if max_checked is not None and len(out) > max_checked:   # the largest deviations and an even sample of the rest
            order = np.argsort(-dev[out[:, 0], out[:, 1]])
            out = out[np.r_[order[:max_checked // 2], order[max_checked // 2::max(1, len(order) // (max_checked // 2))]]]
        for (s, j) in out:
            cs = coords(int(j), name == "g_rel")
            if kind == "head":
                allowed = spread * (np.sum(np.abs(Gn[s]) * near_zero(xvec(s, TN), cs)) + abs(gp[s]) * near_zero(xvec(s, T[s:s + 1]), cs)[0])
            elif kind == "tail":
                allowed = spread * abs(gp[s]) * near_zero(xvec(s, T[s:s + 1]), cs)[0]
            else:
                xs = np.stack([xvec(b, TN[s:s + 1])[0] for b in range(B)]) if Wv is not None else Qv - TN[s][None, :]
                allowed = spread * np.sum(np.abs(Gn[:, s]) * near_zero(xs, cs))
            assert dev[s, j] <= tol * top + allowed, (name, int(s), int(j), float(dev[s, j] / top), float(allowed / top))
    return n_out
