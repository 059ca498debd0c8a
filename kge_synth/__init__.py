"""Seeded synthetic inputs for the knowledge-graph-embedding hot path.

This module only *produces inputs*: embedding-table values, index arrays, workload presets.  It
holds none of the method's arithmetic (no scores, losses, optimiser, ranking, negative sampling)
and is the one module that both the CPU oracle's tests and the GPU path's tests may use.

Table values are a pure function of (seed, tag, row, column), so any subset of rows of a table
that is tens of GB on the device can be regenerated on the host without holding the table:

    z   = splitmix64-finaliser(seed*K1 + tag*K2 + (row*4096 + col)*K3)        (uint64, wrapping)
    u24 = z >> 40
    val = float32(int(u24) - 2^23) * float32(amp / 2^23)                      in [-amp, amp)

The single fp32 multiply by a power-of-two-scaled constant rounds identically on every machine;
``kge_synth/fill.hip`` evaluates the same function on the device.

The graphs stand in for WikiKG90Mv2 (not available offline): same orders of magnitude for |E|,
|R|, |T| (Table 1 of arXiv 2211.12281), micro-batch / negative-sample / embedding sizes in the
range of Table 3, heavy-tailed entity degrees (Zipf) as in real knowledge graphs.
"""
from __future__ import annotations

import math

import numpy as np

BASE_SEED = 221112281

# stream tags of the value / index streams
TAG_ENT, TAG_REL, TAG_RELW = 1, 2, 3
TAG_TRIPLE_H, TAG_TRIPLE_R, TAG_TRIPLE_T = 4, 5, 6
TAG_NEG, TAG_BATCH, TAG_QUERY, TAG_HELDOUT = 7, 8, 9, 10

_K1 = np.uint64(0xD1342543DE82EF95)
_K2 = np.uint64(0x9E3779B97F4A7C15)
_K3 = np.uint64(0xBF58476D1CE4E5B9)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
COL_STRIDE = 4096  # columns per row in the element counter; dim must not exceed it


def _mix(seed: int, tag: int, idx: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        base = np.array([seed], dtype=np.uint64) * _K1 + np.array([tag], dtype=np.uint64) * _K2
        z = base + idx.astype(np.uint64) * _K3
        z ^= z >> np.uint64(30)
        z *= _M1
        z ^= z >> np.uint64(27)
        z *= _M2
        z ^= z >> np.uint64(31)
    return z


def uniform_rows(seed: int, tag: int, rows, dim: int, amp: float) -> np.ndarray:
    """fp32 [len(rows), dim] with values in [-amp, amp); row i is table row rows[i]."""
    assert dim <= COL_STRIDE
    rows = np.asarray(rows, dtype=np.uint64).reshape(-1, 1)
    cols = np.arange(dim, dtype=np.uint64).reshape(1, -1)
    z = _mix(seed, tag, rows * np.uint64(COL_STRIDE) + cols)
    k = (z >> np.uint64(40)).astype(np.int64) - (1 << 23)
    scale = np.float32(amp) / np.float32(1 << 23)
    return k.astype(np.float32) * scale


def uniform_table(seed: int, tag: int, n_rows: int, dim: int, amp: float,
                  chunk: int = 1 << 16) -> np.ndarray:
    out = np.empty((n_rows, dim), dtype=np.float32)
    for lo in range(0, n_rows, chunk):
        hi = min(n_rows, lo + chunk)
        out[lo:hi] = uniform_rows(seed, tag, np.arange(lo, hi), dim, amp)
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16); a storage-format conversion."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = u + np.uint64(0x7FFF) + lsb
    return (u >> np.uint64(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 values after a round trip through bf16 storage."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


def unit_rows(x: np.ndarray) -> np.ndarray:
    """Rows scaled to unit L2 norm in fp32 (used to initialise TransH normals)."""
    x = np.asarray(x, dtype=np.float32)
    nrm = np.sqrt((x.astype(np.float64) ** 2).sum(axis=1, keepdims=True))
    return (x / np.maximum(nrm, 1e-30)).astype(np.float32)


# ---------------------------------------------------------------------------------------------
# index streams
# ---------------------------------------------------------------------------------------------
def rng(seed: int, tag: int, step: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, tag, step]))


def _coprime_multiplier(n: int, start: int = 7654321) -> int:
    a = start % n if n > 1 else 1
    a |= 1
    while math.gcd(a, n) != 1:
        a += 2
    return a


class ZipfIds:
    """Truncated Zipf over n ids: P(rank rho) ~ rho^-s, rho = 1..n; rank -> id by the bijection
    id = (rho * A + B) mod n with gcd(A, n) = 1, so hot rows are scattered over the table."""

    def __init__(self, n: int, s: float):
        self.n = int(n)
        w = np.arange(1, self.n + 1, dtype=np.float64) ** (-float(s))
        self.cdf = np.cumsum(w)
        self.cdf /= self.cdf[-1]
        self.a = _coprime_multiplier(self.n)
        self.b = 12345 % self.n

    def ranks(self, gen: np.random.Generator, size: int) -> np.ndarray:
        u = gen.random(size)
        return np.minimum(np.searchsorted(self.cdf, u, side="right"), self.n - 1).astype(np.int64)

    def ids_of_ranks(self, ranks: np.ndarray) -> np.ndarray:
        return ((ranks.astype(np.int64) * self.a + self.b) % self.n).astype(np.int32)

    def draw(self, gen: np.random.Generator, size: int) -> np.ndarray:
        return self.ids_of_ranks(self.ranks(gen, size))


def uniform_ids(gen: np.random.Generator, lo: int, hi: int, size: int) -> np.ndarray:
    return gen.integers(lo, hi, size=size, dtype=np.int64).astype(np.int32)


# ---------------------------------------------------------------------------------------------
# workload presets (the five configurations of the build's baseline file)
# ---------------------------------------------------------------------------------------------
PRESETS = {
    # tiny DistMult training step + brute-force ranking
    "c1": dict(n_ent=1_000, n_rel=10, n_triples=5_000, dim=32, dtype="f32", B=64, N=64,
               scorers=["distmult"], loss="logsigmoid", gamma=0.0, adv_temp=0.0, lr=1e-3,
               init="normal", amp=0.1, ids="uniform", K=100),
    # scoring only, all five scorers
    "c2": dict(n_ent=1_000_000, n_rel=1_000, dim=256, dtype="f32", B=2_048, N=8_192,
               scorers=["transe", "transh", "rotate", "distmult", "complex"], init="uniform",
               amp=0.1, ids="uniform"),
    # ComplEx training step, sampled softmax, bf16 compute + fp32 master and moments
    "c3": dict(n_ent=10_000_000, n_rel=1_000, dim=256, dtype="bf16", B=4_096, N=16_384,
               scorers=["complex"], loss="sampled_softmax", lr=1e-3, init="uniform", amp=0.1,
               ids="zipf", zipf_s=1.1),
    # link-prediction inference, top-100 + rank of a held-out tail
    "c4": dict(n_ent=10_000_000, n_rel=1_000, dim=256, dtype="bf16", Q=8_192, K=100,
               scorers=["distmult", "transe"], init="uniform", amp=0.1, ids="zipf", zipf_s=1.1),
    # full-scale graph, TransH fp32, 16 partitions, one partition pair per step
    "c5": dict(n_ent=90_000_000, n_rel=1_400, n_triples=600_000_000, dim=128, dtype="f32",
               B=8_192, N=4_096, scorers=["transh"], loss="logsigmoid", gamma=10.0, adv_temp=1.0,
               lr=1e-3, init="uniform", amp=0.1, ids="zipf", zipf_s=1.1, rel_zipf_s=1.0, D=16),
}


def rel_dim(scorer: str, dim: int) -> int:
    return dim // 2 if scorer == "rotate" else dim


def relation_tables(scorer: str, n_rel: int, dim: int, seed: int = BASE_SEED, amp: float = 0.1):
    """(rel fp32 [n_rel, k], relw fp32 [n_rel, dim] or None).  RotatE relations are phases in
    [-pi, pi); TransH normals are unit rows."""
    k = rel_dim(scorer, dim)
    if scorer == "rotate":
        rel = uniform_rows(seed, TAG_REL, np.arange(n_rel), k, math.pi)
    else:
        rel = uniform_rows(seed, TAG_REL, np.arange(n_rel), k, amp)
    relw = None
    if scorer == "transh":
        relw = unit_rows(uniform_rows(seed, TAG_RELW, np.arange(n_rel), dim, 1.0))
    return rel, relw


def normal_table(seed: int, tag: int, n_rows: int, dim: int, std: float) -> np.ndarray:
    return (rng(seed, tag).standard_normal((n_rows, dim)) * std).astype(np.float32)


def compact_rows(*id_arrays):
    """Map global ids to positions in the sorted list of distinct ids.
    Returns (distinct ids, [remapped arrays...])."""
    allv = np.concatenate([np.asarray(a, dtype=np.int64).ravel() for a in id_arrays])
    uniq, inv = np.unique(allv, return_inverse=True)
    out, ofs = [], 0
    for a in id_arrays:
        n = np.asarray(a).size
        out.append(inv[ofs:ofs + n].astype(np.int32).reshape(np.asarray(a).shape))
        ofs += n
    return uniq, out
