"""ctypes front-end of the CPU oracle (``kge_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
``cpu_baseline`` leg.  The product package never imports this module, and this module never
imports the product package.  All arithmetic lives in the C file; this wrapper only marshals
numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kge_oracle.c")
_LIB = os.path.join(_HERE, "libkge_oracle.so")

SCORERS = {"transe": 0, "transh": 1, "rotate": 2, "distmult": 3, "complex": 4,
           "transe_l1": 5, "transh_l1": 6, "rotate_l1": 7}
LOSSES = {"logsigmoid": 0, "sampled_softmax": 1}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, no contraction, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_score_one.restype = C.c_double
        _lib.orc_loss_one.restype = C.c_double
        _lib.orc_loss_bwd.restype = C.c_double
        _lib.orc_l3_norm.restype = C.c_double
        _lib.orc_cbrt_weight.restype = C.c_uint64
        _lib.orc_encode.restype = C.c_double
        _lib.orc_bf16_rne.restype = C.c_uint16
    return _lib


def _p(a, ctype):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(ctype))


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _sid(scorer):
    return SCORERS[scorer] if isinstance(scorer, str) else int(scorer)


def _lid(loss):
    return LOSSES[loss] if isinstance(loss, str) else int(loss)


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle will use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    return os.cpu_count() or 1


# ---------------------------------------------------------------------------------------------
def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def philox_single_round(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox_single_round(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def sample_negatives(seed, step, tag, lo, hi, n):
    out = np.zeros(int(n), dtype=np.int32)
    lib().orc_sample_negatives(C.c_uint64(seed), C.c_uint64(step), C.c_uint32(tag),
                               C.c_int64(lo), C.c_int64(hi), C.c_int64(n), _p(out, C.c_int32))
    return out


def score_one(scorer, h, r, w, t):
    h, r, w, t = _f32(h), _f32(r), _f32(w), _f32(t)
    return float(lib().orc_score_one(_sid(scorer), C.c_int(h.shape[0]), _p(h, C.c_float),
                                     _p(r, C.c_float), _p(w, C.c_float), _p(t, C.c_float)))


def score_batch(scorer, ent, rel, relw, h, r, t, neg, want_neg=True):
    ent, rel, relw = _f32(ent), _f32(rel), _f32(relw)
    h, r, t, neg = _i32(h), _i32(r), _i32(t), _i32(neg)
    B, N, d = h.shape[0], neg.shape[0], ent.shape[1]
    pos = np.zeros(B, dtype=np.float64)
    ngs = np.zeros((B, N), dtype=np.float64) if want_neg else None
    lib().orc_score_batch(_sid(scorer), C.c_int(d), _p(ent, C.c_float), _p(rel, C.c_float),
                          _p(relw, C.c_float), _p(h, C.c_int32), _p(r, C.c_int32),
                          _p(t, C.c_int32), C.c_int64(B), _p(neg, C.c_int32), C.c_int64(N),
                          _p(pos, C.c_double), _p(ngs, C.c_double))
    return pos, ngs


def loss_one(loss, gamma, adv_temp, n_ent_for_c, fp, s):
    s = np.ascontiguousarray(s, dtype=np.float64)
    ds = np.zeros_like(s)
    dfp = C.c_double(0.0)
    L = lib().orc_loss_one(_lid(loss), C.c_double(gamma), C.c_double(adv_temp),
                           C.c_int64(n_ent_for_c), C.c_double(fp), _p(s, C.c_double),
                           C.c_int64(s.shape[0]), C.byref(dfp), _p(ds, C.c_double))
    return float(L), float(dfp.value), ds


def l3_norm(x, lam=0.0):
    """(||x||_3, lam * gradient) of one embedding row (Section 3.1 "Regularisation")."""
    x = _f32(x)
    g = np.zeros(x.shape[0], dtype=np.float64)
    n = lib().orc_l3_norm(C.c_int(x.shape[0]), _p(x, C.c_float), C.c_double(lam), _p(g, C.c_double))
    return float(n), g


def loss_bwd(scorer, loss, ent, rel, relw, h, r, t, neg, gamma=0.0, adv_temp=0.0,
             loss_scale=None, n_ent_for_c=0, want_grads=True, reg_l3=0.0):
    ent, rel, relw = _f32(ent), _f32(rel), _f32(relw)
    h, r, t, neg = _i32(h), _i32(r), _i32(t), _i32(neg)
    B, N, d = h.shape[0], neg.shape[0], ent.shape[1]
    k = rel.shape[1]
    if loss_scale is None:
        loss_scale = 1.0 / max(B, 1)
    g_ent = np.zeros((2 * B + N, d), dtype=np.float64) if want_grads else None
    g_rel = np.zeros((B, k), dtype=np.float64) if want_grads else None
    g_relw = np.zeros((B, d), dtype=np.float64) if (want_grads and relw is not None) else None
    per = np.zeros(B, dtype=np.float64)
    L = lib().orc_loss_bwd(_sid(scorer), _lid(loss), C.c_int(d), _p(ent, C.c_float),
                           _p(rel, C.c_float), _p(relw, C.c_float), _p(h, C.c_int32),
                           _p(r, C.c_int32), _p(t, C.c_int32), C.c_int64(B), _p(neg, C.c_int32),
                           C.c_int64(N), C.c_double(gamma), C.c_double(adv_temp),
                           C.c_double(loss_scale), C.c_int64(n_ent_for_c), C.c_double(reg_l3), _p(g_ent, C.c_double),
                           _p(g_rel, C.c_double), _p(g_relw, C.c_double), _p(per, C.c_double))
    return {"loss": float(L), "g_ent": g_ent, "g_rel": g_rel, "g_relw": g_relw,
            "g_ent_idx": np.concatenate([h, t, neg]).astype(np.int32), "g_rel_idx": r.copy(),
            "per_triple": per}


def sparse_adam(theta, m, v, idx, grads, lr, beta1=0.9, beta2=0.999, eps=1e-8, step=1):
    """Returns (theta', m', v', touched) as fp64 arrays; inputs are not modified."""
    th = np.array(theta, dtype=np.float64, order="C")
    mm = np.array(m, dtype=np.float64, order="C")
    vv = np.array(v, dtype=np.float64, order="C")
    idx, grads = _i32(idx), _f32(grads)
    n_rows, d = th.shape
    touched = np.zeros(n_rows, dtype=np.uint8)
    lib().orc_sparse_adam(_p(th, C.c_double), _p(mm, C.c_double), _p(vv, C.c_double),
                          C.c_int64(n_rows), C.c_int(d), _p(idx, C.c_int32), _p(grads, C.c_float),
                          C.c_int64(idx.shape[0]), C.c_double(lr), C.c_double(beta1),
                          C.c_double(beta2), C.c_double(eps), C.c_int64(step),
                          _p(touched, C.c_uint8))
    return th, mm, vv, touched.astype(bool)


def bf16_rne(x):
    x = _f32(x)
    out = np.zeros(x.shape, dtype=np.uint16)
    lib().orc_bf16_rne_array(_p(x, C.c_float), C.c_int64(x.size), _p(out, C.c_uint16))
    return out


def topk(scorer, ent, rel, relw, h, r, cand_lo, cand_hi, K, true_t=None):
    ent, rel, relw = _f32(ent), _f32(rel), _f32(relw)
    h, r, true_t = _i32(h), _i32(r), _i32(true_t)
    Q, d = h.shape[0], ent.shape[1]
    out_idx = np.zeros((Q, K), dtype=np.int32)
    out_score = np.zeros((Q, K), dtype=np.float64)
    rank = np.zeros(Q, dtype=np.int64) if true_t is not None else None
    lib().orc_topk(_sid(scorer), C.c_int(d), _p(ent, C.c_float), _p(rel, C.c_float),
                   _p(relw, C.c_float), _p(h, C.c_int32), _p(r, C.c_int32), C.c_int64(Q),
                   C.c_int64(cand_lo), C.c_int64(cand_hi), C.c_int32(K), _p(out_idx, C.c_int32),
                   _p(out_score, C.c_double), _p(true_t, C.c_int32), _p(rank, C.c_int64))
    return out_idx, out_score, rank


def topk_band(scorer, ent, rel, relw, h, r, cand_lo, cand_hi, K, true_t, band_eps):
    """topk(...) plus, from the same pass, the number of candidates whose ranking key lies within band_eps[q] of the
    held-out tail's key: (idx, score, rank, band)."""
    ent, rel, relw = _f32(ent), _f32(rel), _f32(relw)
    h, r, true_t = _i32(h), _i32(r), _i32(true_t)
    eps = np.ascontiguousarray(band_eps, dtype=np.float64)
    Q, d = h.shape[0], ent.shape[1]
    assert eps.shape == (Q,)
    out_idx = np.zeros((Q, K), dtype=np.int32)
    out_score = np.zeros((Q, K), dtype=np.float64)
    rank = np.zeros(Q, dtype=np.int64)
    band = np.zeros(Q, dtype=np.int64)
    lib().orc_topk_band(_sid(scorer), C.c_int(d), _p(ent, C.c_float), _p(rel, C.c_float),
                        _p(relw, C.c_float), _p(h, C.c_int32), _p(r, C.c_int32), C.c_int64(Q),
                        C.c_int64(cand_lo), C.c_int64(cand_hi), C.c_int32(K), _p(out_idx, C.c_int32),
                        _p(out_score, C.c_double), _p(true_t, C.c_int32), _p(rank, C.c_int64),
                        _p(eps, C.c_double), _p(band, C.c_int64))
    return out_idx, out_score, rank, band


def bucket_triples(h, t, part_size, D, want_order=True):
    h, t = _i32(h), _i32(t)
    n = h.shape[0]
    counts = np.zeros(D * D, dtype=np.int64)
    offsets = np.zeros(D * D + 1, dtype=np.int64)
    order = np.zeros(n, dtype=np.int64) if want_order else None
    lib().orc_bucket_triples(_p(h, C.c_int32), _p(t, C.c_int32), C.c_int64(n),
                             C.c_int64(part_size), C.c_int(D), _p(counts, C.c_int64),
                             _p(offsets, C.c_int64), _p(order, C.c_int64))
    return counts, offsets, order


def cbrt_weight(n: int) -> int:
    """floor(2^20 * n^(1/3)): the integer weight of a relation with n triples in a bucket."""
    return int(lib().orc_cbrt_weight(C.c_uint64(n)))


def sampler_build(h, r, t, part_size, D, n_rel):
    """(order, rel_offsets, cdf) of the relation-aware sampler (Section 4, "Training")."""
    h, r, t = _i32(h), _i32(r), _i32(t)
    n, groups = h.shape[0], D * D * n_rel
    order = np.zeros(n, dtype=np.int64)
    offs = np.zeros(groups + 1, dtype=np.int64)
    cdf = np.zeros(groups, dtype=np.uint64)
    lib().orc_sampler_build(_p(h, C.c_int32), _p(r, C.c_int32), _p(t, C.c_int32), C.c_int64(n),
                            C.c_int64(part_size), C.c_int(D), C.c_int64(n_rel), _p(order, C.c_int64),
                            _p(offs, C.c_int64), _p(cdf, C.c_uint64))
    return order, offs, cdf


def sample_triples(seed, step, tag, bucket_lo, n_buckets, per_bucket, n_rel, rel_offsets, cdf, order):
    out = np.zeros(n_buckets * per_bucket, dtype=np.int64)
    lib().orc_sample_triples(C.c_uint64(seed), C.c_uint64(step), C.c_uint32(tag), C.c_int64(bucket_lo),
                             C.c_int64(n_buckets), C.c_int64(per_bucket), C.c_int64(n_rel),
                             _p(np.ascontiguousarray(rel_offsets, dtype=np.int64), C.c_int64),
                             _p(np.ascontiguousarray(cdf, dtype=np.uint64), C.c_uint64),
                             _p(np.ascontiguousarray(order, dtype=np.int64), C.c_int64), _p(out, C.c_int64))
    return out


def sample_negatives_sharded(seed, step, tag, part_size, n_ent, D, per_shard):
    out = np.zeros(D * per_shard, dtype=np.int32)
    lib().orc_sample_negatives_sharded(C.c_uint64(seed), C.c_uint64(step), C.c_uint32(tag), C.c_int64(part_size),
                                       C.c_int64(n_ent), C.c_int(D), C.c_int64(per_shard), _p(out, C.c_int32))
    return out


def encode(ent_s, feat, m_h, m_t, idx, B, N, p=0.0, seed=0, step=0, tag=0, reg_t=0.0, reg_s=0.0, reg_f=0.0):
    """Feature-projection encoder (Section 3.1, eq. (embedding)) over the 2B+N slots: (reg value, proj, e)."""
    ent_s, feat, m_h, m_t, idx = _f32(ent_s), _f32(feat), _f32(m_h), _f32(m_t), _i32(idx)
    d, fd, n = ent_s.shape[1], feat.shape[1], 2 * B + N
    proj = np.zeros((n, d), dtype=np.float64)
    e = np.zeros((n, d), dtype=np.float64)
    om = lib().orc_encode(C.c_int(d), C.c_int(fd), _p(ent_s, C.c_float), _p(feat, C.c_float), _p(m_h, C.c_float),
                          _p(m_t, C.c_float), _p(idx, C.c_int32), C.c_int64(B), C.c_int64(N), C.c_double(p),
                          C.c_uint64(seed), C.c_uint64(step), C.c_uint32(tag), C.c_double(reg_t), C.c_double(reg_s),
                          C.c_double(reg_f), _p(proj, C.c_double), _p(e, C.c_double))
    return float(om), proj, e


def encode_bwd(ent_s, feat, m_h, m_t, idx, B, N, de, p=0.0, seed=0, step=0, tag=0, reg_t=0.0, reg_s=0.0, reg_f=0.0):
    """Backward of encode: (g_s [(2B+N), d], g_mh [d, fd], g_mt [d, fd])."""
    ent_s, feat, m_h, m_t, idx = _f32(ent_s), _f32(feat), _f32(m_h), _f32(m_t), _i32(idx)
    d, fd, n = ent_s.shape[1], feat.shape[1], 2 * B + N
    de = np.ascontiguousarray(de, dtype=np.float64)
    g_s = np.zeros((n, d), dtype=np.float64)
    g_mh = np.zeros((d, fd), dtype=np.float64)
    g_mt = np.zeros((d, fd), dtype=np.float64)
    lib().orc_encode_bwd(C.c_int(d), C.c_int(fd), _p(ent_s, C.c_float), _p(feat, C.c_float), _p(m_h, C.c_float),
                         _p(m_t, C.c_float), _p(idx, C.c_int32), C.c_int64(B), C.c_int64(N), C.c_double(p),
                         C.c_uint64(seed), C.c_uint64(step), C.c_uint32(tag), C.c_double(reg_t), C.c_double(reg_s),
                         C.c_double(reg_f), _p(de, C.c_double), _p(g_s, C.c_double), _p(g_mh, C.c_double),
                         _p(g_mt, C.c_double))
    return g_s, g_mh, g_mt


def ensemble(lists, p, K_out=10):
    """Power-rank ensemble of M top-K lists per query: lists int32 [M, Q, K] -> (idx [Q, K_out], score [Q, K_out])."""
    lists = np.ascontiguousarray(lists, dtype=np.int32)
    M, Q, K = lists.shape
    out_idx = np.zeros((Q, K_out), dtype=np.int32)
    out_score = np.zeros((Q, K_out), dtype=np.float64)
    lib().orc_ensemble(_p(lists, C.c_int32), C.c_int(M), C.c_int64(Q), C.c_int(K), C.c_double(p), C.c_int(K_out),
                       _p(out_idx, C.c_int32), _p(out_score, C.c_double))
    return out_idx, out_score
