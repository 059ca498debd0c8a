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
    rel, relw = ks.relation_tables(scorer, n_rel, dim, seed, amp)
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
