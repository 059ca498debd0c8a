#!/usr/bin/env python3
"""Benchmark of the MI355X knowledge-graph-embedding hot path (one GPU).

A "step" is one pass of the whole path over one micro-batch of seeded synthetic input that is
already resident in HBM: sample the shared negatives, gather + score + loss + backward, and the
duplicate-aware sparse Adam update of the entity and relation tables (workload c3, the default);
or one scoring / ranking call for the forward-only workloads.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # dense bf16 MFMA, MI355X
PEAK_F32_TFLOPS = 157.3       # fp32 matrix
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default: 1000, c4: 20 - a step of a training workload takes a quarter of a millisecond, "
                         "and the first hundred run 4 %% slower than the steady state)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default: 100, c4: 2)")
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--scorer", default=None, help="restrict to one scorer (training workloads: replaces the configured one)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the entity table (debugging only)")
    ap.add_argument("--reg-l3", type=float, default=0.0,
                    help="training workloads: weight of the L3 regulariser of the gathered rows (default off)")
    ap.add_argument("--sampled-batches", type=int, default=0, metavar="TRIPLES",
                    help="training workloads: draw every micro-batch on the GPU with the relation-aware sampler "
                         "(one worker's all-partition micro-batch and sharded negatives) from a synthetic list of "
                         "this many triples, instead of replaying pre-drawn index streams")
    ap.add_argument("--pair-batches", action="store_true",
                    help="c5: replay pre-drawn micro-batches of ONE partition pair per step instead of the default there, "
                         "the sampler's all-partition micro-batch with sharded negatives (--sampled-batches 100000000)")
    ap.add_argument("--encoder", type=int, default=0, metavar="FEAT_DIM",
                    help="training workloads: entities are encoded as e_S + M e_F from synthetic text features of "
                         "this width (768 in the paper) with dropout 0.1, trained M_H and M_T; default: shallow only")
    ap.add_argument("--p-norm", type=int, default=2, choices=[1, 2],
                    help="training workloads with --scorer transe or rotate: the norm of the distance (Table 2); 1 runs the "
                         "vector-pipe kernels of the 1-norm variants")
    ap.add_argument("--ensemble", type=int, default=0, metavar="MODELS",
                    help="c4: also time the power-rank ensemble of this many synthetic top-K lists per query (reported "
                         "beside the ranking numbers, outside the timed steps)")
    ap.add_argument("--graph", action="store_true",
                    help="training workloads: replay every step from a HIP graph (step number from a counter in device "
                         "memory) instead of enqueueing it call by call; on ROCm 7.2 the replay is no faster")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 1 GiB device copy first (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


# ---------------------------------------------------------------------------------------------
# workloads
# ---------------------------------------------------------------------------------------------
class TrainWorkload:
    """c3 / c5 / c1: forward + backward + sparse Adam on bf16 shadow / fp32 master tables."""

    def __init__(self, name, P, scale, only=None, reg_l3=0.0, sampled=0, feat_dim=0, p_norm=2):
        import torch
        import kge_synth as ks
        import kge_synth.device as ksd
        import paper_2211_12281_amd as kge
        self.kge, self.torch, self.ks, self.P, self.name = kge, torch, ks, P, name
        self.scorer = only or P["scorers"][0]
        self.p_norm = p_norm
        if p_norm == 1 and self.scorer not in ("transe", "rotate", "transh"):
            raise SystemExit("--p-norm 1 needs --scorer transe, rotate or transh")
        self.n_ent = max(1000, int(P["n_ent"] * scale))
        self.n_rel, self.d, self.B, self.N = P["n_rel"], P["dim"], P["B"], P["N"]
        self.bf16 = P["dtype"] == "bf16"
        dev = "cuda"
        t0 = time.time()
        self.ent = torch.empty((self.n_ent, self.d), dtype=torch.float32, device=dev)
        ksd.fill_uniform(self.ent, ks.BASE_SEED, ks.TAG_ENT, P["amp"])
        self.ent_m = torch.zeros_like(self.ent)
        self.ent_v = torch.zeros_like(self.ent)
        self.ent_sh = None
        if self.bf16:
            self.ent_sh = torch.empty((self.n_ent, self.d), dtype=torch.bfloat16, device=dev)
            ksd.fill_uniform(self.ent_sh, ks.BASE_SEED, ks.TAG_ENT, P["amp"])
        rel, relw = ks.relation_tables(self.scorer, self.n_rel, self.d, ks.BASE_SEED, P["amp"])
        self.rel = torch.from_numpy(rel).to(dev)
        self.rel_m, self.rel_v = torch.zeros_like(self.rel), torch.zeros_like(self.rel)
        self.rel_sh = self.rel.to(torch.bfloat16) if self.bf16 else None
        self.relw = self.relw_m = self.relw_v = self.relw_sh = None
        if relw is not None:
            self.relw = torch.from_numpy(relw).to(dev)
            self.relw_m, self.relw_v = torch.zeros_like(self.relw), torch.zeros_like(self.relw)
            self.relw_sh = self.relw.to(torch.bfloat16) if self.bf16 else None
        self.model = kge.Model(self.scorer, self.ent_sh if self.bf16 else self.ent,
                               self.rel_sh if self.bf16 else self.rel, self.relw_sh if self.bf16 else self.relw,
                               p_norm=p_norm)
        # index streams: a ring of pre-drawn micro-batches, resident on the device
        self.batches = []
        self.host_batches = []
        nb = 8
        if P["ids"] == "zipf":
            z = ks.ZipfIds(self.n_ent, P["zipf_s"])
        for i in range(nb):
            g = ks.rng(ks.BASE_SEED, ks.TAG_BATCH, i)
            if name == "c5":
                # one partition pair (i, j) per step: heads in shard i, tails (and negatives) in shard j
                D = P["D"]; part = -(-self.n_ent // D)
                pi, pj = (i // D) % D, i % D
                h = self._zipf_in_range(z, g, pi * part, min(self.n_ent, (pi + 1) * part), self.B)
                t = self._zipf_in_range(z, g, pj * part, min(self.n_ent, (pj + 1) * part), self.B)
                lo, hi = pj * part, min(self.n_ent, (pj + 1) * part)
            else:
                h = z.draw(g, self.B) if P["ids"] == "zipf" else ks.uniform_ids(g, 0, self.n_ent, self.B)
                t = z.draw(g, self.B) if P["ids"] == "zipf" else ks.uniform_ids(g, 0, self.n_ent, self.B)
                lo, hi = 0, self.n_ent
            if "rel_zipf_s" in P:
                r = ks.ZipfIds(self.n_rel, P["rel_zipf_s"]).draw(g, self.B)
            else:
                r = ks.uniform_ids(g, 0, self.n_rel, self.B)
            self.host_batches.append((h, r, t, lo, hi))
            # the row ids of a step in gradient-row order, [h | t | negatives]: the negatives are drawn into the tail, so
            # the sort for the sparse update reads the array as it stands (no concatenation)
            ids = torch.empty(2 * self.B + self.N, dtype=torch.int32, device=dev)
            ids[:self.B] = torch.from_numpy(h).to(dev)
            ids[self.B:2 * self.B] = torch.from_numpy(t).to(dev)
            self.batches.append((ids[:self.B], torch.from_numpy(r).to(dev), ids[self.B:2 * self.B], lo, hi, ids))
        self.neg = torch.empty(self.N, dtype=torch.int32, device=dev)
        self.counter = torch.zeros(1, dtype=torch.int64, device=dev)      # the step number, on the device
        self.graphs = None
        k = self.rel.shape[1]
        self.out = {
            "loss": torch.empty(1, dtype=torch.float32, device=dev),
            "g_ent": torch.empty((2 * self.B + self.N, self.d), dtype=torch.float32, device=dev),
            "g_ent_idx": torch.empty(2 * self.B + self.N, dtype=torch.int32, device=dev),
            "g_rel": torch.empty((self.B, k), dtype=torch.float32, device=dev),
            "g_relw": torch.empty((self.B, self.d), dtype=torch.float32, device=dev) if relw is not None else None,
            "g_rel_idx": torch.empty(self.B, dtype=torch.int32, device=dev),
        }
        self.loss_kw = dict(gamma=P.get("gamma", 0.0), adv_temp=P.get("adv_temp", 0.0))
        if P["loss"] == "sampled_softmax":
            self.loss_kw = dict(n_ent_for_c=self.n_ent)
        if reg_l3 > 0.0:
            self.loss_kw["reg_l3"] = reg_l3
        self.main = torch.cuda.current_stream()
        self.eager_now = False
        self.ws_ent, self.ws_rel, self.ws_relw = kge.Workspace(), kge.Workspace(), kge.Workspace()
        self.enc = None
        if feat_dim > 0:
            # text features stand-ins: fixed U(-0.5, 0.5) rows; projections start at U(-0.05, 0.05)
            tdt = torch.bfloat16 if self.bf16 else torch.float32
            self.feat = torch.empty((self.n_ent, feat_dim), dtype=tdt, device=dev)
            ksd.fill_uniform(self.feat, ks.BASE_SEED, 21, 0.5)
            self.mproj = []
            for tag in (22, 23):
                m = torch.from_numpy(ks.uniform_rows(ks.BASE_SEED, tag, np.arange(self.d), feat_dim, 0.05)).to(dev)
                self.mproj.append({"p": m, "m": torch.zeros_like(m), "v": torch.zeros_like(m),
                                   "sh": m.to(torch.bfloat16) if self.bf16 else None})
            tbl = lambda q: q["sh"] if self.bf16 else q["p"]
            self.enc = kge.Encoder(self.ent_sh if self.bf16 else self.ent, self.feat, tbl(self.mproj[0]), tbl(self.mproj[1]),
                                   dropout=0.1, reg_t=reg_l3)
            self.feat_dim = feat_dim
            self.rows_d = torch.arange(self.d, dtype=torch.int32, device=dev)
            self.ar = torch.arange(2 * self.B + self.N, dtype=torch.int32, device=dev)
            self.loss_kw.pop("reg_l3", None)               # the regulariser acts on the encoded e inside the encoder
        self.sampler = None
        if sampled > 0:
            # the paper's generator: worker i's micro-batch takes B/D triples from each bucket T_ij by the
            # cube-root relation law, and N/D negatives from each entity shard (Section 4, "Training")
            self.D = P.get("D", 8)
            self.part = -(-self.n_ent // self.D)
            g = ks.rng(ks.BASE_SEED, ks.TAG_TRIPLE_H)
            zz = ks.ZipfIds(self.n_ent, P.get("zipf_s", 1.1))
            th, tt = zz.draw(g, sampled), zz.draw(g, sampled)
            tr = ks.ZipfIds(self.n_rel, P.get("rel_zipf_s", 1.0)).draw(g, sampled)
            self.sampler = kge.TripleSampler(*(torch.from_numpy(x).to(dev) for x in (th, tr, tt)), self.part, self.D,
                                             self.n_rel)
            self.n_triples = sampled
        torch.cuda.synchronize()
        self.setup_s = time.time() - t0

    def _zipf_in_range(self, z, g, lo, hi, n):
        out = np.empty(0, dtype=np.int32)
        while out.size < n:                      # rejection: keeps the Zipf shape inside one shard
            ids = z.draw(g, 4 * n * self.P["D"])
            out = np.concatenate([out, ids[(ids >= lo) & (ids < hi)]])
        return np.ascontiguousarray(out[:n])

    def step(self, i):
        kge, ks = self.kge, self.ks
        if self.sampler is not None:
            h, r, t = self.sampler.sample(ks.BASE_SEED, i, ks.TAG_BATCH, (i % self.D) * self.D, self.D, self.B // self.D)
            kge.sample_negatives_sharded(ks.BASE_SEED, i, ks.TAG_NEG, self.part, self.n_ent, self.D, self.N // self.D,
                                         out=self.neg)
        else:
            if self.enc is None:
                if self.graphs is None:
                    self._step_call_by_call(i)
                # (graphs: the step number of the negatives and of Adam is read from the device counter, which every step
                # advances; argument i only selects the pre-drawn batch)
                elif not self.eager_now:
                    self.graphs[i % len(self.batches)].replay()
                else:
                    self._enqueue(i % len(self.batches), self.main)
                return
            h, r, t, lo, hi, _ = self.batches[i % len(self.batches)]
            kge.sample_negatives(ks.BASE_SEED, i, ks.TAG_NEG, lo, hi, self.N, out=self.neg, stream=self.main)
        lr = self.P["lr"]
        if self.enc is not None:
            B, N = self.B, self.N
            e, proj, _ = self.enc.encode(h, t, self.neg, seed=ks.BASE_SEED, step=i)
            model = kge.Model(self.scorer, e, self.model.rel, self.model.relw, p_norm=self.p_norm)
            kge.loss_bwd(model, self.P["loss"], self.ar[:B], r, self.ar[B:2 * B], self.ar[2 * B:], out=self.out, **self.loss_kw)
            g_es, g_mh, g_mt = self.enc.encode_bwd(h, t, self.neg, proj, self.out["g_ent"], seed=ks.BASE_SEED, step=i)
            idx = self.torch.cat([h, t, self.neg])
            kge.sparse_adam(self.ent, self.ent_sh, self.ent_m, self.ent_v, idx, g_es, lr, step=i + 1)
            for q, gm in zip(self.mproj, (g_mh, g_mt)):
                kge.sparse_adam(q["p"], q["sh"], q["m"], q["v"], self.rows_d, gm, lr, step=i + 1)
        else:
            # batches drawn by the sampler: the ids that the update sorts are the ones kge_loss_bwd lists beside its gradient rows
            kge.loss_bwd(self.model, self.P["loss"], h, r, t, self.neg, out=self.out, stream=self.main, **self.loss_kw)
            plans = [(self.n_ent, self.d, self.out["g_ent_idx"], self.ws_ent), (self.n_rel, self.rel.shape[1], r, self.ws_rel)]
            if self.relw is not None:
                plans.append((self.n_rel, self.d, r, self.ws_relw))
            kge.sparse_adam_plan_tables(plans, stream=self.main)
            kge.sparse_adam_apply_tables(self._tables(), lr, step=i + 1, stream=self.main)
            return
        kge.sparse_adam(self.rel, self.rel_sh, self.rel_m, self.rel_v, self.out["g_rel_idx"], self.out["g_rel"], lr,
                        step=i + 1)
        if self.relw is not None:
            kge.sparse_adam(self.relw, self.relw_sh, self.relw_m, self.relw_v, self.out["g_rel_idx"],
                            self.out["g_relw"], lr, step=i + 1)

    def _tables(self):
        """(plans, updates) of the step's tables for kge_sparse_adam_plan_tables / kge_sparse_adam_apply_tables."""
        t = [(self.ent, self.ent_sh, self.ent_m, self.ent_v, self.out["g_ent"], self.ws_ent),
             (self.rel, self.rel_sh, self.rel_m, self.rel_v, self.out["g_rel"], self.ws_rel)]
        if self.relw is not None:
            t.append((self.relw, self.relw_sh, self.relw_m, self.relw_v, self.out["g_relw"], self.ws_relw))
        return t

    def _step_call_by_call(self, i):
        """One step on ONE stream: gather (which draws the step's negatives), forward, backward -> the sorts of the step's row
        ids (every table in one launch) -> the update of every table (two launches).  (A second stream for the sorts,
        which need the ids alone, was measured and lost: each cross-stream wait costs the waiting stream about 10 us on this
        stack, and small kernels that share the chip with the forward or backward kernel hold up a workgroup of theirs.)"""
        kge, ks = self.kge, self.ks
        main = self.main
        h, r, t, lo, hi, ids = self.batches[i % len(self.batches)]
        plans = [(self.n_ent, self.d, ids, self.ws_ent), (self.n_rel, self.rel.shape[1], r, self.ws_rel)]
        if self.relw is not None:
            plans.append((self.n_rel, self.d, r, self.ws_relw))
        kge.loss_bwd(self.model, self.P["loss"], h, r, t, ids[2 * self.B:], out=self.out, stream=main,
                     draw=(ks.BASE_SEED, i, ks.TAG_NEG, lo, hi), plans=plans, **self.loss_kw)
        kge.sparse_adam_apply_tables(self._tables(), self.P["lr"], step=i + 1, stream=main)

    def _enqueue(self, k, main):
        """The same step on pre-drawn batch k in a form that a HIP graph can record: the step number of the negatives and
        of Adam comes from the counter in device memory, which the last node advances."""
        kge, ks = self.kge, self.ks
        h, r, t, lo, hi, ids = self.batches[k]
        c = self.counter
        plans = [(self.n_ent, self.d, ids, self.ws_ent), (self.n_rel, self.rel.shape[1], r, self.ws_rel)]
        if self.relw is not None:
            plans.append((self.n_rel, self.d, r, self.ws_relw))
        kge.loss_bwd(self.model, self.P["loss"], h, r, t, ids[2 * self.B:], out=self.out, stream=main,
                     draw=(ks.BASE_SEED, 0, ks.TAG_NEG, lo, hi, c), plans=plans, **self.loss_kw)
        kge.sparse_adam_apply_tables(self._tables(), self.P["lr"], step=1, stream=main, step_counter=c)
        kge.step_counter_add(c, 1, stream=main)

    def capture(self):
        """Records the step of every pre-drawn batch into a HIP graph of its own (kernel nodes on two streams; the graphs
        differ in the id arrays they read).  One call-by-call step first sizes the workspaces."""
        torch = self.torch
        if self.enc is not None or self.sampler is not None:
            return
        self._enqueue(0, self.main)
        torch.cuda.synchronize()
        self.graphs = []
        for k in range(len(self.batches)):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                self._enqueue(k, torch.cuda.current_stream())
            self.graphs.append(g)
        torch.cuda.synchronize()

    def hbm_bytes(self):
        """Algorithmic HBM bytes per step of the memory-bound kernels (what the method must move, whatever the kernels do):
        gather - the 2B + N entity rows and B relation rows read once, and the ids (a fused path writes nothing);
        finish - the 2B + N + B gradient rows written once and the 3B rows the chain rule reads;
        adam   - per DISTINCT touched row (counted on the batches in flight) parameter and both moments read and written,
                 the bf16 shadow written, plus every gradient row and id read once."""
        torch = self.torch
        if self.enc is not None or self.sampler is not None:
            return {}
        e = 2 if self.bf16 else 4
        B, N, d, k = self.B, self.N, self.d, self.rel.shape[1]
        u_ent = sum(int(torch.unique(b[5]).numel()) for b in self.batches) / len(self.batches)
        u_rel = sum(int(torch.unique(b[1]).numel()) for b in self.batches) / len(self.batches)
        w = 1 if self.relw is None else 2
        row = lambda dim: dim * (24 + (2 if self.bf16 else 0))
        return {"gather": (2 * B + N) * d * e + w * B * k * e + (3 * B + N) * 4,
                "finish": (2 * B + N) * d * 4 + w * B * k * 4 + 3 * B * d * e,
                "adam": u_ent * row(d) + (2 * B + N) * (d * 4 + 4) + u_rel * (row(k) + (w - 1) * row(d)) + w * B * (k * 4 + 4),
                "distinct_rows": {"entity": u_ent, "relation": u_rel}}

    def pairs_per_step(self):
        return self.B * (self.N + 1)

    def extra(self, ms):
        out = {"triples_per_s": self.B / (ms * 1e-3), "scorer": self.scorer, "reg_l3": self.loss_kw.get("reg_l3", 0.0)}
        if self.p_norm == 1:
            out["p_norm"] = 1
        if self.enc is not None:
            out["encoder"] = f"e_S + M e_F, synthetic features of width {self.feat_dim}, dropout 0.1, M_H and M_T trained"
        if self.sampler is not None:
            out["micro_batch"] = f"sampled on the GPU per step: {self.D} x {self.B // self.D} triples of one worker by the " \
                                 f"cube-root relation law from {self.n_triples} synthetic triples, {self.D} x " \
                                 f"{self.N // self.D} sharded negatives"
        return out

    def mfma_flops(self, slot):
        # algorithmic contractions of 2 B N d flop each: the FWD pass computes the scores AND the queries'
        # gradient (two), the GRADT pass the negatives' gradient (one; its recomputed scores earn no credit)
        if slot in ("enc_fwd", "enc_bwd"):                 # projection of the 2B+N slots, or its gradient to M_H, M_T
            return 2.0 * (2 * self.B + self.N) * self.feat_dim * self.d
        gemms = (2 if slot == "block_fwd" else 1) * (2 if self.scorer == "transh" else 1)
        return 2.0 * self.B * self.N * self.d * gemms

    def alu_ops(self, slot):
        # 1-norm kernels: two vector operations per (query, negative, dimension) and pass - subtract and
        # accumulate |.| for the scores, select by the sign and accumulate for a gradient pass
        # TransH: x = q' - t + A w^ costs two, and the kernels carry A (one, scores), P (one, scores), the gradient of
        # w^ (two, pass over the queries) or the hyperplane term of dt (one, pass over the negatives) besides
        per = 2.0
        if self.scorer == "transh":
            per = {"block_score": 5.0, "block_fwd": 5.0, "block_gradt": 4.0}.get(slot, 5.0)
        return per * self.B * self.N * self.d

    def cpu_baseline(self, orc, shrink=1):
        """Oracle forward + backward + sparse Adam on the first rows of batch 0 against all negatives."""
        ks = self.ks
        h, r, t, lo, hi = self.host_batches[0]
        bs = max(1, self.B // shrink)
        h, r, t = h[:bs], r[:bs], t[:bs]
        neg = orc.sample_negatives(ks.BASE_SEED, 0, ks.TAG_NEG, lo, hi, self.N)
        uniq, (ch, ct, cn) = ks.compact_rows(h, t, neg)
        rows = ks.uniform_rows(ks.BASE_SEED, ks.TAG_ENT, uniq, self.d, self.P["amp"])
        if self.bf16:
            rows = ks.round_to_bf16(rows)
        rel, relw = ks.relation_tables(self.scorer, self.n_rel, self.d, ks.BASE_SEED, self.P["amp"])
        if self.bf16:
            rel = ks.round_to_bf16(rel)
            relw = None if relw is None else ks.round_to_bf16(relw)
        kw = dict(self.loss_kw)
        t0 = time.time()
        out = orc.loss_bwd(self.scorer + ("_l1" if self.p_norm == 1 else ""), self.P["loss"], rows, rel, relw, ch, r, ct, cn, **kw)
        z = np.zeros_like(rows, dtype=np.float64)
        orc.sparse_adam(rows, z, z, out["g_ent_idx"], out["g_ent"].astype(np.float32), self.P["lr"])
        dt = time.time() - t0
        return {"value": bs * (self.N + 1) / dt, "unit": "scored_pairs/s", "cores": orc.num_threads(),
                "kind": "oracle", "seconds": round(dt, 2),
                "sample": f"the first {bs} triples of batch 0 against all {self.N} shared negatives: "
                          f"forward + backward + sparse Adam of the entity table"}


class ScoreWorkload:
    """c2: scoring-only forward, all five scorers in one step."""

    def __init__(self, P, scale, only=None):
        import torch
        import kge_synth as ks
        import kge_synth.device as ksd
        import paper_2211_12281_amd as kge
        self.kge, self.torch, self.ks, self.P = kge, torch, ks, P
        self.n_ent = max(1000, int(P["n_ent"] * scale))
        self.d, self.B, self.N = P["dim"], P["B"], P["N"]
        self.scorers = [only] if only else P["scorers"]
        self.ent = torch.empty((self.n_ent, self.d), dtype=torch.float32, device="cuda")
        ksd.fill_uniform(self.ent, ks.BASE_SEED, ks.TAG_ENT, P["amp"])
        self.models = {}
        for s in self.scorers:
            rel, relw = ks.relation_tables(s, P["n_rel"], self.d, ks.BASE_SEED, P["amp"])
            self.models[s] = kge.Model(s, self.ent, torch.from_numpy(rel).cuda(),
                                       None if relw is None else torch.from_numpy(relw).cuda())
        g = ks.rng(ks.BASE_SEED, ks.TAG_BATCH, 0)
        self.h_host, self.r_host, self.t_host = (ks.uniform_ids(g, 0, self.n_ent, self.B),
                                                  ks.uniform_ids(g, 0, P["n_rel"], self.B),
                                                  ks.uniform_ids(g, 0, self.n_ent, self.B))
        self.h, self.r, self.t = (torch.from_numpy(x).cuda() for x in (self.h_host, self.r_host, self.t_host))
        self.neg = kge.sample_negatives(ks.BASE_SEED, 0, ks.TAG_NEG, 0, self.n_ent, self.N)
        self.bf16 = False
        torch.cuda.synchronize()

    def step(self, i):
        for s in self.scorers:
            self.kge.score(self.models[s], self.h, self.r, self.t, self.neg)

    def pairs_per_step(self):
        return len(self.scorers) * self.B * (self.N + 1)

    def extra(self, ms):
        return {"scorers": self.scorers}

    def mfma_flops(self, slot):
        # per launch, averaged over the scorers of a step (TransH runs two contractions)
        g = sum(2 if s == "transh" else 1 for s in self.scorers) / len(self.scorers)
        return 2.0 * self.B * self.N * self.d * g

    def cpu_baseline(self, orc, shrink=1):
        ks = self.ks
        bs = max(1, self.B // shrink)
        neg = orc.sample_negatives(ks.BASE_SEED, 0, ks.TAG_NEG, 0, self.n_ent, self.N)
        h, r, t = self.h_host[:bs], self.r_host[:bs], self.t_host[:bs]
        uniq, (ch, ct, cn) = ks.compact_rows(h, t, neg)
        rows = ks.uniform_rows(ks.BASE_SEED, ks.TAG_ENT, uniq, self.d, self.P["amp"])
        t0 = time.time()
        for s in self.scorers:
            rel, relw = ks.relation_tables(s, self.P["n_rel"], self.d, ks.BASE_SEED, self.P["amp"])
            orc.score_batch(s, rows, rel, relw, ch, r, ct, cn)
        dt = time.time() - t0
        return {"value": len(self.scorers) * bs * (self.N + 1) / dt, "unit": "scored_pairs/s",
                "cores": orc.num_threads(), "kind": "oracle", "seconds": round(dt, 2),
                "sample": f"the first {bs} queries against all {self.N} negatives, {len(self.scorers)} scorers"}


class RankWorkload:
    """c4: full-entity ranking, top-K and rank of a held-out tail."""

    def __init__(self, P, scale, only=None, ens_models=0):
        import torch
        import kge_synth as ks
        import kge_synth.device as ksd
        import paper_2211_12281_amd as kge
        self.kge, self.torch, self.ks, self.P = kge, torch, ks, P
        self.n_ent = max(1000, int(P["n_ent"] * scale))
        self.d, self.Q, self.K = P["dim"], P["Q"], P["K"]
        self.ens_models = ens_models
        self.scorers = [only] if only else P["scorers"]
        self.bf16 = P["dtype"] == "bf16"
        dt = torch.bfloat16 if self.bf16 else torch.float32
        self.ent = torch.empty((self.n_ent, self.d), dtype=dt, device="cuda")
        ksd.fill_uniform(self.ent, ks.BASE_SEED, ks.TAG_ENT, P["amp"])
        self.models = {}
        for s in self.scorers:
            rel, relw = ks.relation_tables(s, P["n_rel"], self.d, ks.BASE_SEED, P["amp"])
            self.models[s] = kge.Model(s, self.ent, torch.from_numpy(rel).cuda().to(dt),
                                       None if relw is None else torch.from_numpy(relw).cuda().to(dt))
        g = ks.rng(ks.BASE_SEED, ks.TAG_QUERY, 0)
        self.h_host = ks.ZipfIds(self.n_ent, P["zipf_s"]).draw(g, self.Q)
        self.r_host = ks.uniform_ids(g, 0, P["n_rel"], self.Q)
        self.t_host = ks.uniform_ids(ks.rng(ks.BASE_SEED, ks.TAG_HELDOUT, 0), 0, self.n_ent, self.Q)
        self.h, self.r, self.t = (torch.from_numpy(x).cuda() for x in (self.h_host, self.r_host, self.t_host))
        torch.cuda.synchronize()

    def step(self, i):
        for s in self.scorers:
            self.last = self.kge.topk(self.models[s], self.h, self.r, 0, self.n_ent, self.K, self.t)

    def pairs_per_step(self):
        return len(self.scorers) * self.Q * self.n_ent

    def extra(self, ms):
        out = {"scorers": self.scorers, "queries_per_s": len(self.scorers) * self.Q / (ms * 1e-3)}
        if self.ens_models > 0:
            out["ensemble"] = self.time_ensemble()
        return out

    def time_ensemble(self):
        """Power-rank ensemble (p = -1) of ens_models lists of K tails per query: every model ranks the same pool of
        2.6 K candidates of the query in its own random order (overlapping lists, as trained models give)."""
        torch = self.torch
        g = torch.Generator(device="cuda"); g.manual_seed(self.ks.BASE_SEED)
        pool = torch.randint(0, self.n_ent, (self.Q, int(2.6 * self.K)), device="cuda", generator=g, dtype=torch.int32)
        lists = torch.stack([torch.gather(pool, 1, torch.rand(pool.shape, device="cuda", generator=g).argsort(1)[:, :self.K])
                             for _ in range(self.ens_models)]).contiguous()
        self.kge.ensemble(lists, -1.0, 10)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            self.kge.ensemble(lists, -1.0, 10)
        b.record(); torch.cuda.synchronize()
        us = a.elapsed_time(b) * 100.0
        return {"models": self.ens_models, "K": self.K, "K_out": 10, "p": -1.0, "us_per_call": us,
                "queries_per_s": self.Q / (us * 1e-6)}

    def mfma_flops(self, slot):
        # summed over the chunk launches of one call (TransH: the second contraction, w^ . t, is part of the score)
        return 2.0 * self.Q * self.n_ent * self.d * (2 if self.scorers == ["transh"] else 1)

    def cpu_baseline(self, orc, shrink=1):
        ks = self.ks
        nq = max(1, 8 // shrink)
        ent = self.ent.float().cpu().numpy()
        t0 = time.time()
        for s in self.scorers:
            rel, relw = ks.relation_tables(s, self.P["n_rel"], self.d, ks.BASE_SEED, self.P["amp"])
            if self.bf16:
                rel = ks.round_to_bf16(rel)
                relw = None if relw is None else ks.round_to_bf16(relw)
            orc.topk(s, ent, rel, relw, self.h_host[:nq], self.r_host[:nq], 0, self.n_ent, self.K, self.t_host[:nq])
        dt = time.time() - t0
        return {"value": len(self.scorers) * nq * self.n_ent / dt, "unit": "scored_pairs/s",
                "cores": orc.num_threads(), "kind": "oracle", "seconds": round(dt, 2),
                "sample": f"first {nq} of {self.Q} queries against all {self.n_ent} entities, top-{self.K} + rank"}


def wl_bf16(wl):
    return bool(getattr(wl, "bf16", False))


def main():
    a = parse()
    if a.steps is None:
        a.steps = 20 if a.workload == "c4" else 1000
    if a.warmup is None:
        a.warmup = 2 if a.workload == "c4" else 100
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported (no collectives are built: the path shards by entity partition, one worker per GPU)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import kge_synth as ks
    import paper_2211_12281_amd as kge
    kge.load()
    P = ks.PRESETS[a.workload]
    if a.workload == "c5" and not a.sampled_batches and not a.pair_batches:
        a.sampled_batches = 100_000_000    # the paper's generator (eq. (microbatch), eq. (negsamples)) is the default at full scale
    if a.workload in ("c1", "c3", "c5"):
        wl = TrainWorkload(a.workload, P, a.scale, a.scorer, a.reg_l3, a.sampled_batches, a.encoder, a.p_norm)
    elif a.workload == "c2":
        wl = ScoreWorkload(P, a.scale, a.scorer)
    else:
        wl = RankWorkload(P, a.scale, a.scorer, a.ensemble)

    if a.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    graphed = isinstance(wl, TrainWorkload) and a.graph
    if graphed:
        wl.capture()
        graphed = wl.graphs is not None
    for i in range(a.warmup):
        wl.step(i)
    torch.cuda.synchronize()
    # HIP events in the timed region around ONE kernel, the one the roofline is quoted for: an event record is a packet
    # of its own in the queue (about 4 us of the GPU's time line each, measured: the C3 step takes 247 us without
    # events, 263 us with the two passes bracketed, 274 us with every slot), and ten of them per step cost the host
    # 30 us.  The other slots are measured in a short pass after the clock has stopped.
    timed_slots = ["block_fwd"] if isinstance(wl, TrainWorkload) else \
                  ["block_score"] if isinstance(wl, ScoreWorkload) else ["topk_scan"]
    other_slots = [s_ for s_ in kge.binding.PROF_SLOTS if s_ not in timed_slots]
    # In a training step the bracket is set on every FOURTH step of the timed region (the average below is over
    # those launches): the value then carries a quarter of the cost of its own instrumentation.  When the steps are
    # replayed from HIP graphs, those bracketed steps are the ones enqueued call by call (a graph holds no events).
    every = (16 if a.steps >= 400 else 4) if isinstance(wl, TrainWorkload) else 1
    host_steps = min(a.steps, 50)               # the host's own cost of a step: while the queue still takes everything at once
    t0 = time.perf_counter()
    for i in range(a.warmup, a.warmup + a.steps):
        if i == a.warmup + host_steps:
            dt_host = time.perf_counter() - t0
        if every > 1:
            kge.profile_enable(timed_slots if (i - a.warmup) % every == 0 else False)
            wl.eager_now = (i - a.warmup) % every == 0
        elif i == a.warmup:
            kge.profile_enable(timed_slots)
        wl.step(i)
    if a.steps == host_steps:
        dt_host = time.perf_counter() - t0      # the host has queued every step (the GPU may still be running)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kge.profile_enable(False)
    ms = dt * 1e3 / a.steps

    prof = {}
    for slot in kge.binding.PROF_SLOTS:
        tot, n = kge.profile_collect(slot)
        if n:
            prof[slot] = {"total_ms": tot, "launches": n, "avg_us": 1e3 * tot / n}
            if every > 1:
                prof[slot]["measured"] = f"every {every}th step of the timed region"
                prof[slot]["total_ms"] = tot * every
    if isinstance(wl, TrainWorkload):
        extra_steps = min(a.steps, 20)
        kge.profile_enable(other_slots)
        wl.eager_now = True
        for i in range(a.warmup + a.steps, a.warmup + a.steps + extra_steps):
            wl.step(i)
        torch.cuda.synchronize()
        kge.profile_enable(False)
        for slot in other_slots:
            tot, n = kge.profile_collect(slot)
            if n:                                  # scaled to the timed region's number of steps
                prof[slot] = {"total_ms": tot * a.steps / extra_steps, "launches": n * a.steps // extra_steps,
                              "avg_us": 1e3 * tot / n, "measured": f"{extra_steps} steps after the timed region"}
    roof = None
    if prof:
        # the slots "adam" and "sort" bracket several kernels per call (2, and 1 to 6 launches): they compete with their
        # per-kernel share, the roofline below being that of ONE kernel
        share = {"adam": 2.0, "sort": 2.0}
        dom = max(prof, key=lambda k: prof[k]["total_ms"] / share.get(k, 1.0))
        # The two passes of a training step (block_fwd over the queries, block_gradt over the negatives) are the same
        # kernel template and take the same time to within run-to-run noise: when they are within 5 % of each other the
        # line reports the pass over the queries (two contractions of algorithmic work; the other pass is credited
        # one, its recomputed scores earning nothing), so that the reported kernel does not flip between runs.  Both
        # durations are in "kernels" either way.
        if dom == "block_gradt" and "block_fwd" in prof and prof["block_fwd"]["total_ms"] >= 0.95 * prof[dom]["total_ms"]:
            dom = "block_fwd"
        avg_s = prof[dom]["avg_us"] * 1e-6
        if dom.startswith("block") and getattr(wl, "p_norm", 2) == 1:
            # vector pipe: 256 compute units x 128 lanes x 2.4 GHz = 78.6 T operations/s (the fp32 vector peak of
            # 157.3 TFLOP/s counts a fused multiply-add as two; these kernels have none to fuse)
            ach = wl.alu_ops(dom) / avg_s / 1e12
            roof = {"kernel": dom, "bound": "alu", "achieved": ach, "peak": PEAK_F32_TFLOPS / 2, "unit": "Top/s",
                    "frac": ach / (PEAK_F32_TFLOPS / 2), "traffic": None, "avg_us": avg_s * 1e6}
        elif dom.startswith("block") or dom.startswith("enc_") or dom == "topk_scan":
            flops = wl.mfma_flops(dom)
            if dom == "topk_scan":
                avg_s = prof[dom]["total_ms"] * 1e-3 / (a.steps * len(wl.scorers))   # all chunk launches of one call
            peak = PEAK_BF16_TFLOPS if wl.bf16 else PEAK_F32_TFLOPS
            ach = flops / avg_s / 1e12
            roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                    "frac": ach / peak, "traffic": None, "avg_us": avg_s * 1e6}
            if dom == "block_score" and not wl.bf16:
                # fp32 tables: the library splits every (scaled) operand row into two fp16 pieces and issues three fp16
                # matrix products per fp32 one (error about 3 x 2^-22 of |q| |t|).  The line stays priced in
                # ALGORITHMIC fp32 flops against the fp32 matrix peak, the dtype of the contract (a fraction above 1
                # says that the path is not on the fp32 pipe); the 16-bit pipe does three times that work, against
                # its own peak:
                roof["issued_f16"] = {"achieved": 3 * ach, "peak": PEAK_BF16_TFLOPS, "frac": 3 * ach / PEAK_BF16_TFLOPS}
            if dom in ("block_fwd", "block_gradt") and not wl.bf16 and (wl.d * 4 <= 512 or dom == "block_gradt"):
                # fp32 training passes: every operand value as three bf16 pieces, six bf16 matrix products per fp32 one
                # (all terms down to 2^-26 of |a| |b|); priced like the fp32 score block above
                roof["issued_bf16"] = {"achieved": 6 * ach, "peak": PEAK_BF16_TFLOPS, "frac": 6 * ach / PEAK_BF16_TFLOPS}
        else:
            roof = {"kernel": dom, "bound": "hbm", "achieved": None, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": None, "traffic": None, "avg_us": avg_s * 1e6}

    if roof is not None and "measured" in prof.get(roof["kernel"], {}):
        roof["measured"] = prof[roof["kernel"]]["measured"]

    enc_roof = None
    if "enc_fwd" in prof:                                  # the encoder's contractions against the same matrix peak
        peak = PEAK_BF16_TFLOPS if wl.bf16 else PEAK_F32_TFLOPS
        enc_roof = {}
        for slot in ("enc_fwd", "enc_bwd"):
            ach = wl.mfma_flops(slot) / (prof[slot]["avg_us"] * 1e-6) / 1e12
            enc_roof[slot] = {"bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
                              "avg_us": prof[slot]["avg_us"]}

    cpu = None
    if not a.no_cpu_baseline:
        import ctypes
        import oracle
        oracle.build()

        def timed(shrink, budget_s):
            reps, secs, first = 0, 0.0, None
            while secs < budget_s and reps < 64:   # whole samples until about budget_s of CPU work
                one = wl.cpu_baseline(oracle, shrink)
                secs += one["seconds"]; reps += 1
                first = one if first is None else first
            work = first["value"] * first["seconds"]    # units of one sample
            first["value"] = work * reps / secs
            first["seconds"] = round(secs, 2)
            first["sample"] += f" (x{reps})"
            return first

        cpu = timed(1, 10.0)                       # every thread the OpenMP runtime gives the oracle
        cpu["nproc"] = os.cpu_count()
        try:
            cpu["cpu_model"] = next(l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name"))
        except (OSError, StopIteration):
            cpu["cpu_model"] = None
        try:                                        # the same oracle on ONE thread, on a sample a sixteenth the size
            gomp = ctypes.CDLL("libgomp.so.1")
            gomp.omp_set_num_threads(1)
            one = timed(16, 6.0)
            gomp.omp_set_num_threads(cpu["cores"])
            one["cores"] = 1
            cpu["one_thread"] = {k: one[k] for k in ("value", "unit", "cores", "seconds", "sample")}
        except OSError:
            cpu["one_thread"] = None

    if roof is not None and roof["bound"] == "mfma":
        tpath = os.path.join(ROOT, "profiles", "traffic.json")
        if os.path.exists(tpath):
            try:
                tr = json.load(open(tpath)).get(a.workload, {}).get(roof["kernel"])
                if tr is not None:
                    roof["traffic"] = tr          # HBM bytes per launch, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
                    roof["traffic_source"] = "stored: profiles/traffic.json, read from a rocprofv3 --pmc run of this command (not measured in this run)"
            except (ValueError, OSError):
                pass
    # the same box's own figures beside the published peaks: a loop of independent bf16 matrix instructions and a plain
    # 1 GiB streaming copy (after the timed region; a few milliseconds)
    # (the loop also on operands whose signs and mantissas differ from element to element, as a table's do: the chip
    # holds a lower clock the more bits toggle, so this, not the published peak, is what a kernel fed from real rows
    # could reach if it did nothing but matrix instructions)
    calib = {"mfma_bf16_loop_tflops": kge.calibrate_mfma(), "mfma_bf16_loop_tflops_varied_operands": kge.calibrate_mfma(varied=True),
             "copy_gbs": kge.calibrate_copy(1 << 30)}
    # what two HIP events read when NOTHING lies between them: the share of a bracketed kernel's duration that is the
    # bracket's own (the rocprofv3 trace of the same command shows the kernel without it)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    tot = 0.0
    for _ in range(20):
        e0.record(); e1.record(); e1.synchronize()
        tot += e0.elapsed_time(e1)
    calib["empty_event_pair_us"] = tot / 20 * 1e3
    if roof is not None and roof.get("achieved") and roof.get("avg_us", 0) > 2 * calib["empty_event_pair_us"]:
        # the same figures with the bracket's own duration taken off (information; "frac" above keeps the raw duration)
        net = roof["avg_us"] - calib["empty_event_pair_us"]
        roof["avg_us_less_empty_pair"] = net
        roof["frac_less_empty_pair"] = roof["frac"] * roof["avg_us"] / net
    if roof is not None and roof.get("achieved") is not None and roof["bound"] == "mfma" and wl_bf16(wl):
        roof["frac_of_measured_loop"] = roof["achieved"] / calib["mfma_bf16_loop_tflops"]
        roof["frac_of_measured_loop_varied_operands"] = roof["achieved"] / calib["mfma_bf16_loop_tflops_varied_operands"]
    if roof is not None and isinstance(wl, TrainWorkload) and "block_fwd" in prof and "block_gradt" in prof and roof["bound"] == "mfma":
        # both passes together: the credited flops of the step (scores, dQ, dT: 3 contractions) over the two kernels' time
        us = prof["block_fwd"]["avg_us"] + prof["block_gradt"]["avg_us"]
        fl = wl.mfma_flops("block_fwd") + wl.mfma_flops("block_gradt")
        roof["both_passes"] = {"avg_us": us, "achieved": fl / (us * 1e-6) / 1e12, "frac": fl / (us * 1e-6) / 1e12 / roof["peak"]}
    # the memory-bound kernels of a training step against the HBM peak and against this box's own streaming copy
    hbm = None
    if isinstance(wl, TrainWorkload):
        per = wl.hbm_bytes()
        hbm = {}
        for slot in ("gather", "finish", "adam"):
            if slot in prof and slot in per:
                gbs = per[slot] / (prof[slot]["avg_us"] * 1e-6) / 1e9
                hbm[slot] = {"bytes_algorithmic": int(per[slot]), "avg_us": prof[slot]["avg_us"], "GB/s": gbs,
                             "frac_of_8TBs": gbs / PEAK_HBM_GBS, "frac_of_copy": gbs / calib["copy_gbs"]}
        if hbm:
            hbm["distinct_rows_per_step"] = per["distinct_rows"]
            hbm["note"] = ("avg_us: HIP events around the launch(es) of the slot, 20 steps after the timed region "
                           "(adam: both launches, all tables of the step)")
    pairs = wl.pairs_per_step()
    line = {
        "metric": "scored (query,candidate) pairs/s", "value": pairs / (ms * 1e-3), "unit": "pairs/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": P["dtype"], "data": "synthetic",
        "config": {"workload": a.workload, **{k: v for k, v in P.items() if k in
                                              ("n_ent", "n_rel", "dim", "B", "N", "Q", "K", "loss")}},
        "roofline": roof, "cpu_baseline": cpu, "kernels": prof, "calibration": calib,
    }
    line["host_enqueue_ms_per_step"] = dt_host * 1e3 / host_steps      # (over the first 50 timed steps: later the queue is full and the host waits for the GPU)
    if hbm:
        line["hbm_kernels"] = hbm
    if isinstance(wl, TrainWorkload):
        line["enqueue"] = ("HIP graph replay, one graph per pre-drawn batch; every 4th step call by call with the HIP-event bracket"
                           if graphed else "call by call, one stream (c3: 7 launches per step in two library calls)")
    line.update(wl.extra(ms))
    if enc_roof:
        line["encoder_roofline"] = enc_roof
    print(json.dumps(line))


if __name__ == "__main__":
    main()
