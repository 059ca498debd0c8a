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
