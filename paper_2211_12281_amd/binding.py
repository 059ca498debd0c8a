"""ctypes binding of libkge_mi355x.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch supplies device memory and the
stream.  There is no CPU fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkge_mi355x.so")

SCORERS = {"transe": 0, "transh": 1, "rotate": 2, "distmult": 3, "complex": 4}
LOSSES = {"logsigmoid": 0, "sampled_softmax": 1}
OP_SCORE, OP_LOSS_BWD, OP_SPARSE_ADAM, OP_TOPK, OP_PARTITION, OP_SAMPLER_BUILD, OP_ENCODE, OP_ENCODE_BWD = range(8)
EXPORTS = ["kge_sample_negatives", "kge_score", "kge_loss_bwd", "kge_sparse_adam", "kge_topk",
           "kge_partition_triples", "kge_sampler_build", "kge_sample_triples", "kge_sample_negatives_sharded",
           "kge_encode", "kge_encode_bwd", "kge_encode_workspace_bytes", "kge_ensemble", "kge_sparse_adam_plan",
           "kge_sparse_adam_apply", "kge_sparse_adam_static", "kge_sparse_adam_static_limit", "kge_debug_select",
           "kge_workspace_bytes", "kge_status_string", "kge_profile_enable", "kge_profile_collect",
           "kge_calibrate_mfma", "kge_calibrate_mfma_varied", "kge_calibrate_copy", "kge_step_counter_add", "kge_sample_negatives_dev",
           "kge_sparse_adam_apply_tables", "kge_sparse_adam_plan_tables", "kge_loss_bwd_sampled",
           "kge_loss_bwd_sampled_planned"]
PROF_SLOTS = {"block_score": 0, "block_fwd": 1, "block_gradt": 2, "adam": 3, "sort": 4, "topk_scan": 5,
              "enc_fwd": 6, "enc_bwd": 7, "gather": 8, "finish": 9}


class KgeEncoderT(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("dim", C.c_int32), ("feat_dim", C.c_int32), ("dropout_tag", C.c_uint32),
                ("n_ent", C.c_int64), ("ent_s", C.c_void_p), ("feat", C.c_void_p), ("m_h", C.c_void_p),
                ("m_t", C.c_void_p), ("ent_ld", C.c_int64), ("feat_ld", C.c_int64), ("m_ld", C.c_int64),
                ("dropout", C.c_float), ("reg_t", C.c_float), ("reg_s", C.c_float), ("reg_f", C.c_float)]


class KgeModelT(C.Structure):
    _fields_ = [("scorer", C.c_int32), ("p_norm", C.c_int32), ("dtype", C.c_int32), ("dim", C.c_int32),
                ("rel_dim", C.c_int32), ("reserved", C.c_int32), ("n_ent", C.c_int64), ("n_rel", C.c_int64),
                ("ent", C.c_void_p), ("rel", C.c_void_p), ("relw", C.c_void_p),
                ("ent_ld", C.c_int64), ("rel_ld", C.c_int64), ("relw_ld", C.c_int64)]


class KgeLossCfgT(C.Structure):
    _fields_ = [("loss", C.c_int32), ("gamma", C.c_float), ("adv_temp", C.c_float), ("loss_scale", C.c_float),
                ("n_ent_for_c", C.c_int64), ("reg_l3", C.c_float), ("reserved", C.c_int32)]


class KgeAdamCfgT(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("step", C.c_int64), ("step_counter", C.c_void_p)]


class KgeNegDrawT(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("step", C.c_uint64), ("step_counter", C.c_void_p), ("stream_tag", C.c_uint32),
                ("reserved", C.c_uint32), ("lo", C.c_int64), ("hi", C.c_int64)]


class KgeAdamPlanT(C.Structure):
    _fields_ = [("n_rows", C.c_int64), ("dim", C.c_int32), ("idx", C.c_void_p), ("M", C.c_int64), ("ws", C.c_void_p),
                ("ws_bytes", C.c_size_t)]


class KgeAdamTableT(C.Structure):
    _fields_ = [("param_f32", C.c_void_p), ("param_bf16", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("n_rows", C.c_int64), ("dim", C.c_int32), ("ld", C.c_int64), ("grads", C.c_void_p), ("M", C.c_int64),
                ("ws", C.c_void_p), ("ws_bytes", C.c_size_t)]


class KgeError(RuntimeError):
    pass


_lib = None


def load():
    """Loads the library or raises; never builds it and never falls back to anything else."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise KgeError(f"{LIB_PATH} is missing: build it with `python -m paper_2211_12281_amd.build`")
        lib = C.CDLL(LIB_PATH)
        lib.kge_encode.argtypes = [C.c_void_p] * 3 + [C.c_int64, C.c_void_p, C.c_int64, C.c_uint64, C.c_uint64] + \
            [C.c_void_p] * 4 + [C.c_size_t, C.c_void_p]
        lib.kge_encode_bwd.argtypes = [C.c_void_p] * 3 + [C.c_int64, C.c_void_p, C.c_int64, C.c_uint64, C.c_uint64] + \
            [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
        lib.kge_encode_workspace_bytes.restype = C.c_size_t
        lib.kge_encode_workspace_bytes.argtypes = [C.c_int, C.c_void_p, C.c_int64, C.c_int64]
        lib.kge_sampler_build.argtypes = [C.c_void_p] * 3 + [C.c_int64, C.c_int64, C.c_int32, C.c_int64] + \
            [C.c_void_p] * 4 + [C.c_size_t, C.c_void_p]
        lib.kge_sample_triples.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_int64, C.c_int64, C.c_int64,
                                           C.c_int32, C.c_int64] + [C.c_void_p] * 11
        lib.kge_sample_negatives_sharded.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_int64, C.c_int64,
                                                     C.c_int32, C.c_int64, C.c_void_p, C.c_void_p]
        lib.kge_workspace_bytes.restype = C.c_size_t
        lib.kge_workspace_bytes.argtypes = [C.c_int, C.c_void_p, C.c_int64, C.c_int64, C.c_int64]
        lib.kge_calibrate_mfma.argtypes = [C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        lib.kge_calibrate_mfma_varied.argtypes = [C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        lib.kge_calibrate_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        lib.kge_status_string.restype = C.c_char_p
        lib.kge_status_string.argtypes = [C.c_int]
        lib.kge_sparse_adam_plan_tables.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        lib.kge_sparse_adam_apply_tables.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        lib.kge_step_counter_add.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
        lib.kge_sample_negatives_dev.argtypes = [C.c_uint64, C.c_void_p, C.c_uint64, C.c_uint32, C.c_int64, C.c_int64, C.c_int64,
                                                 C.c_void_p, C.c_void_p]
        lib.kge_sample_negatives.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_int64, C.c_int64, C.c_int64,
                                             C.c_void_p, C.c_void_p]
        lib.kge_score.argtypes = [C.c_void_p] + [C.c_void_p] * 3 + [C.c_int64, C.c_void_p, C.c_int64] + \
            [C.c_void_p] * 3 + [C.c_size_t, C.c_void_p]
        lib.kge_loss_bwd.argtypes = [C.c_void_p, C.c_void_p] + [C.c_void_p] * 3 + [C.c_int64, C.c_void_p, C.c_int64] + \
            [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p]
        lib.kge_loss_bwd_sampled.argtypes = [C.c_void_p, C.c_void_p] + [C.c_void_p] * 3 + [C.c_int64, C.c_void_p, C.c_void_p, C.c_int64] + \
            [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p]
        lib.kge_loss_bwd_sampled_planned.argtypes = [C.c_void_p, C.c_void_p] + [C.c_void_p] * 3 + \
            [C.c_int64, C.c_void_p, C.c_void_p, C.c_int64] + [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p, C.c_int32, C.c_void_p]
        lib.kge_sparse_adam.argtypes = [C.c_void_p] * 4 + [C.c_int64, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p,
                                                           C.c_int64, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.kge_sparse_adam_static.argtypes = [C.c_void_p] * 4 + [C.c_int64, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p,
                                                                  C.c_int64, C.c_void_p, C.c_void_p]
        lib.kge_sparse_adam_static_limit.restype = C.c_size_t
        lib.kge_sparse_adam_static_limit.argtypes = []
        lib.kge_sparse_adam_plan.argtypes = [C.c_int64, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.kge_sparse_adam_apply.argtypes = [C.c_void_p] * 4 + [C.c_int64, C.c_int32, C.c_int64, C.c_void_p, C.c_int64,
                                                                 C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.kge_topk.argtypes = [C.c_void_p] * 3 + [C.c_int64, C.c_int64, C.c_int64, C.c_int32] + [C.c_void_p] * 5 + \
            [C.c_size_t, C.c_void_p]
        lib.kge_ensemble.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_double, C.c_int32, C.c_void_p,
                                     C.c_void_p, C.c_void_p]
        lib.kge_partition_triples.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.kge_sampler_build.argtypes = [C.c_void_p] * 3 + [C.c_int64, C.c_int64, C.c_int32, C.c_int64] + \
            [C.c_void_p] * 4 + [C.c_size_t, C.c_void_p]
        lib.kge_sample_triples.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_int64, C.c_int64, C.c_int64,
                                           C.c_int32, C.c_int64] + [C.c_void_p] * 11
        lib.kge_sample_negatives_sharded.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_int64, C.c_int64,
                                                     C.c_int32, C.c_int64, C.c_void_p, C.c_void_p]
        _lib = lib
    return _lib


def status_string(code: int) -> str:
    return load().kge_status_string(code).decode()


def _check(code: int, what: str):
    if code != 0:
        raise KgeError(f"{what} failed: {status_string(code)} ({code})")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    """The HIP stream of a call: torch's current one, or the given torch.cuda.Stream (saves the lookup and the
    stream context around the call)."""
    return C.c_void_p((stream if stream is not None else torch.cuda.current_stream()).cuda_stream)


def _i32(t):
    assert t.dtype == torch.int32 and t.is_cuda and t.is_contiguous(), "index tensors: contiguous int32 on the GPU"
    return t


class Workspace:
    """A grow-only device buffer handed to the library as its scratch space."""

    def __init__(self):
        self.buf = None

    def get(self, nbytes: int):
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = None
            self.buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        return self.buf


_default_ws = Workspace()


class Model:
    """Scorer + embedding tables (device tensors, fp32 or bf16, row-major 2-D)."""

    def __init__(self, scorer: str, ent, rel, relw=None, p_norm: int = 2):
        self.scorer = scorer
        self.ent, self.rel, self.relw = ent, rel, relw
        assert ent.is_cuda and rel.is_cuda and ent.dim() == 2 and rel.dim() == 2
        assert ent.dtype == rel.dtype and ent.dtype in (torch.float32, torch.bfloat16)
        assert ent.stride(1) == 1 and rel.stride(1) == 1
        self.dim = ent.shape[1]
        s = KgeModelT()
        s.scorer = SCORERS[scorer]
        s.p_norm = p_norm
        s.dtype = 1 if ent.dtype == torch.bfloat16 else 0
        s.dim = self.dim
        s.rel_dim = rel.shape[1]
        s.n_ent, s.n_rel = ent.shape[0], rel.shape[0]
        s.ent, s.rel = ent.data_ptr(), rel.data_ptr()
        s.ent_ld, s.rel_ld = ent.stride(0), rel.stride(0)
        if relw is not None:
            assert relw.is_cuda and relw.dtype == ent.dtype and relw.stride(1) == 1
            s.relw, s.relw_ld = relw.data_ptr(), relw.stride(0)
        self.struct = s

    @property
    def ref(self):
        return C.byref(self.struct)


def workspace_bytes(op: int, model: Model | None, B: int, N: int, K: int = 0) -> int:
    return int(load().kge_workspace_bytes(op, model.ref if model is not None else None, B, N, K))


def _counter(t):
    """Device pointer of a step counter: one int64 (read as uint64) on the GPU, or None."""
    if t is None:
        return None
    assert t.is_cuda and t.dtype == torch.int64 and t.numel() == 1
    return t.data_ptr()


def step_counter_add(counter, inc: int = 1, stream=None):
    """kge_step_counter_add: enqueues counter += inc (for steps replayed from a HIP graph)."""
    _check(load().kge_step_counter_add(_counter(counter), inc, _stream(stream)), "kge_step_counter_add")


def sample_negatives_dev(seed: int, counter, step_offset: int, tag: int, lo: int, hi: int, n: int, out=None, stream=None):
    """kge_sample_negatives_dev: the ids of step step_offset + counter[0], the counter being read on the device."""
    if out is None:
        out = torch.empty(n, dtype=torch.int32, device="cuda")
    _check(load().kge_sample_negatives_dev(seed, _counter(counter), step_offset, tag, lo, hi, n, _ptr(out), _stream(stream)),
           "kge_sample_negatives_dev")
    return out


def sample_negatives(seed: int, step: int, tag: int, lo: int, hi: int, n: int, out=None, stream=None):
    if out is None:
        out = torch.empty(n, dtype=torch.int32, device="cuda")
    _check(load().kge_sample_negatives(seed, step, tag, lo, hi, n, _ptr(out), _stream(stream)), "kge_sample_negatives")
    return out


def score(model: Model, h, r, t, neg, want_neg: bool = True, ws: Workspace | None = None):
    B, N = h.numel(), neg.numel()
    pos = torch.empty(B, dtype=torch.float32, device="cuda")
    blk = torch.empty((B, N), dtype=torch.float32, device="cuda") if want_neg else None
    ws = ws or _default_ws
    nbytes = workspace_bytes(OP_SCORE, model, B, N)
    buf = ws.get(nbytes)
    _check(load().kge_score(model.ref, _ptr(_i32(h)), _ptr(_i32(r)), _ptr(_i32(t)), B, _ptr(_i32(neg)), N,
                            _ptr(pos), _ptr(blk), _ptr(buf), buf.numel(), _stream()), "kge_score")
    return pos, blk


def loss_bwd(model: Model, loss: str, h, r, t, neg, gamma: float = 0.0, adv_temp: float = 0.0,
             loss_scale: float = 0.0, n_ent_for_c: int = 0, ws: Workspace | None = None, out=None,
             reg_l3: float = 0.0, stream=None, draw=None, plans=None):
    """kge_loss_bwd; with draw = (seed, step, stream_tag, lo, hi[, step_counter]) kge_loss_bwd_sampled, which draws the
    negatives itself and writes their ids to `neg` (an int32 tensor of N entries); with plans = [(n_rows, dim, idx, ws),
    ...] as well kge_loss_bwd_sampled_planned, which also plans the sparse update of those tables."""
    B, N, d = h.numel(), neg.numel(), model.dim
    k = model.rel.shape[1]
    if out is None:
        out = {
            "loss": torch.empty(1, dtype=torch.float32, device="cuda"),
            "g_ent": torch.empty((2 * B + N, d), dtype=torch.float32, device="cuda"),
            "g_ent_idx": torch.empty(2 * B + N, dtype=torch.int32, device="cuda"),
            "g_rel": torch.empty((B, k), dtype=torch.float32, device="cuda"),
            "g_relw": torch.empty((B, d), dtype=torch.float32, device="cuda") if model.relw is not None else None,
            "g_rel_idx": torch.empty(B, dtype=torch.int32, device="cuda"),
        }
    cfg = KgeLossCfgT(LOSSES[loss], gamma, adv_temp, loss_scale, n_ent_for_c, reg_l3, 0)
    ws = ws or _default_ws
    buf = ws.get(workspace_bytes(OP_LOSS_BWD, model, B, N))
    if draw is not None:
        assert neg.is_cuda and neg.dtype == torch.int32 and neg.is_contiguous()
        dr = KgeNegDrawT(draw[0], draw[1], _counter(draw[5]) if len(draw) > 5 else None, draw[2], 0, draw[3], draw[4])
        if plans is not None:
            arr = _plan_array(plans)
            _check(load().kge_loss_bwd_sampled_planned(model.ref, C.byref(cfg), _ptr(_i32(h)), _ptr(_i32(r)), _ptr(_i32(t)), B,
                                                       C.byref(dr), _ptr(neg), N, _ptr(out["loss"]), _ptr(out["g_ent"]),
                                                       _ptr(out["g_ent_idx"]), _ptr(out["g_rel"]), _ptr(out["g_relw"]),
                                                       _ptr(out["g_rel_idx"]), _ptr(buf), buf.numel(), arr, len(plans),
                                                       _stream(stream)), "kge_loss_bwd_sampled_planned")
            return out
        _check(load().kge_loss_bwd_sampled(model.ref, C.byref(cfg), _ptr(_i32(h)), _ptr(_i32(r)), _ptr(_i32(t)), B,
                                           C.byref(dr), _ptr(neg), N, _ptr(out["loss"]), _ptr(out["g_ent"]),
                                           _ptr(out["g_ent_idx"]), _ptr(out["g_rel"]), _ptr(out["g_relw"]),
                                           _ptr(out["g_rel_idx"]), _ptr(buf), buf.numel(), _stream(stream)),
               "kge_loss_bwd_sampled")
        return out
    _check(load().kge_loss_bwd(model.ref, C.byref(cfg), _ptr(_i32(h)), _ptr(_i32(r)), _ptr(_i32(t)), B,
                               _ptr(_i32(neg)), N, _ptr(out["loss"]), _ptr(out["g_ent"]), _ptr(out["g_ent_idx"]),
                               _ptr(out["g_rel"]), _ptr(out["g_relw"]), _ptr(out["g_rel_idx"]), _ptr(buf),
                               buf.numel(), _stream(stream)), "kge_loss_bwd")
    return out


def sparse_adam(param, shadow, m, v, idx, grads, lr: float, beta1: float = 0.9, beta2: float = 0.999,
                eps: float = 1e-8, step: int = 1, ws: Workspace | None = None, step_counter=None):
    assert param.dtype == torch.float32 and m.dtype == torch.float32 and v.dtype == torch.float32
    assert grads.dtype == torch.float32 and grads.is_contiguous() and param.stride(1) == 1
    assert m.stride() == param.stride() and v.stride() == param.stride()
    if shadow is not None:
        assert shadow.dtype == torch.bfloat16 and shadow.stride() == param.stride()
    M, d = idx.numel(), param.shape[1]
    cfg = KgeAdamCfgT(lr, beta1, beta2, eps, step, _counter(step_counter))
    ws = ws or _default_ws
    buf = ws.get(workspace_bytes(OP_SPARSE_ADAM, None, M, d))
    _check(load().kge_sparse_adam(_ptr(param), _ptr(shadow), _ptr(m), _ptr(v), param.shape[0], d, param.stride(0),
                                  _ptr(_i32(idx)), _ptr(grads), M, C.byref(cfg), _ptr(buf), buf.numel(), _stream()),
           "kge_sparse_adam")


def sparse_adam_static_limit() -> int:
    return int(load().kge_sparse_adam_static_limit())


def sparse_adam_static(param, shadow, m, v, idx, grads, lr: float, beta1: float = 0.9, beta2: float = 0.999,
                       eps: float = 1e-8, step: int = 1, stream=None, step_counter=None):
    """kge_sparse_adam_static: the update with the library's built-in scratch buffer (no workspace, no allocation)."""
    assert param.dtype == torch.float32 and m.dtype == torch.float32 and v.dtype == torch.float32
    assert grads.dtype == torch.float32 and grads.is_contiguous() and param.stride(1) == 1
    assert m.stride() == param.stride() and v.stride() == param.stride()
    if shadow is not None:
        assert shadow.dtype == torch.bfloat16 and shadow.stride() == param.stride()
    cfg = KgeAdamCfgT(lr, beta1, beta2, eps, step, _counter(step_counter))
    _check(load().kge_sparse_adam_static(_ptr(param), _ptr(shadow), _ptr(m), _ptr(v), param.shape[0], param.shape[1],
                                         param.stride(0), _ptr(_i32(idx)), _ptr(grads), idx.numel(), C.byref(cfg),
                                         _stream(stream)), "kge_sparse_adam_static")


def sparse_adam_plan(n_rows: int, dim: int, idx, ws: Workspace, stream=None):
    """Sorts the row ids of a later sparse_adam_apply into `ws` (which must be kept for that call alone)."""
    M = idx.numel()
    buf = ws.get(workspace_bytes(OP_SPARSE_ADAM, None, M, dim))
    _check(load().kge_sparse_adam_plan(n_rows, dim, _ptr(_i32(idx)), M, _ptr(buf), buf.numel(), _stream(stream)),
           "kge_sparse_adam_plan")


def sparse_adam_apply(param, shadow, m, v, grads, ws: Workspace, lr: float, beta1: float = 0.9, beta2: float = 0.999,
                      eps: float = 1e-8, step: int = 1, stream=None, step_counter=None):
    assert param.dtype == torch.float32 and m.dtype == torch.float32 and v.dtype == torch.float32
    assert grads.dtype == torch.float32 and grads.is_contiguous() and param.stride(1) == 1
    assert m.stride() == param.stride() and v.stride() == param.stride()
    if shadow is not None:
        assert shadow.dtype == torch.bfloat16 and shadow.stride() == param.stride()
    M, d = grads.shape[0], param.shape[1]
    cfg = KgeAdamCfgT(lr, beta1, beta2, eps, step, _counter(step_counter))
    buf = ws.get(workspace_bytes(OP_SPARSE_ADAM, None, M, d))
    _check(load().kge_sparse_adam_apply(_ptr(param), _ptr(shadow), _ptr(m), _ptr(v), param.shape[0], d, param.stride(0),
                                        _ptr(grads), M, C.byref(cfg), _ptr(buf), buf.numel(), _stream(stream)),
           "kge_sparse_adam_apply")


def sparse_adam_plan_tables(plans, stream=None):
    """kge_sparse_adam_plan_tables: plans = [(n_rows, dim, idx, ws), ...]; the sorts of up to 32,768 ids share one launch."""
    _check(load().kge_sparse_adam_plan_tables(_plan_array(plans), len(plans), _stream(stream)), "kge_sparse_adam_plan_tables")


def _plan_array(plans):
    arr = (KgeAdamPlanT * len(plans))()
    for a, (n_rows, dim, idx, ws) in zip(arr, plans):
        M = idx.numel()
        buf = ws.get(workspace_bytes(OP_SPARSE_ADAM, None, M, dim))
        a.n_rows, a.dim, a.idx, a.M, a.ws, a.ws_bytes = n_rows, dim, _ptr(_i32(idx)), M, _ptr(buf), buf.numel()
    return arr


def sparse_adam_apply_tables(tables, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, step: int = 1,
                             stream=None, step_counter=None):
    """kge_sparse_adam_apply_tables: tables = [(param, shadow, m, v, grads, ws), ...], each planned into its own ws."""
    arr = (KgeAdamTableT * len(tables))()
    for a, (param, shadow, m, v, grads, ws) in zip(arr, tables):
        assert param.dtype == torch.float32 and m.dtype == torch.float32 and v.dtype == torch.float32
        assert grads.dtype == torch.float32 and grads.is_contiguous() and param.stride(1) == 1
        assert m.stride() == param.stride() and v.stride() == param.stride()
        if shadow is not None:
            assert shadow.dtype == torch.bfloat16 and shadow.stride() == param.stride()
        M, d = grads.shape[0], param.shape[1]
        buf = ws.get(workspace_bytes(OP_SPARSE_ADAM, None, M, d))
        a.param_f32, a.param_bf16, a.m, a.v = _ptr(param), _ptr(shadow), _ptr(m), _ptr(v)
        a.n_rows, a.dim, a.ld, a.grads, a.M, a.ws, a.ws_bytes = param.shape[0], d, param.stride(0), _ptr(grads), M, _ptr(buf), buf.numel()
    cfg = KgeAdamCfgT(lr, beta1, beta2, eps, step, _counter(step_counter))
    _check(load().kge_sparse_adam_apply_tables(arr, len(tables), C.byref(cfg), _stream(stream)), "kge_sparse_adam_apply_tables")


def topk(model: Model, h, r, cand_lo: int, cand_hi: int, K: int, true_t=None, ws: Workspace | None = None):
    Q = h.numel()
    out_idx = torch.empty((Q, K), dtype=torch.int32, device="cuda")
    out_score = torch.empty((Q, K), dtype=torch.float32, device="cuda")
    rank = torch.empty(Q, dtype=torch.int64, device="cuda") if true_t is not None else None
    ws = ws or _default_ws
    buf = ws.get(workspace_bytes(OP_TOPK, model, Q, cand_hi - cand_lo, K))
    _check(load().kge_topk(model.ref, _ptr(_i32(h)), _ptr(_i32(r)), Q, cand_lo, cand_hi, K, _ptr(out_idx),
                           _ptr(out_score), _ptr(true_t), _ptr(rank), _ptr(buf), buf.numel(), _stream()), "kge_topk")
    return out_idx, out_score, rank


def ensemble(lists, p: float, K_out: int = 10):
    """Power-rank ensemble of M top-K lists: lists int32 [M, Q, K] -> (idx int32 [Q, K_out], score fp32 [Q, K_out])."""
    assert lists.dtype == torch.int32 and lists.dim() == 3 and lists.is_contiguous()
    M, Q, K = lists.shape
    out_idx = torch.empty((Q, K_out), dtype=torch.int32, device="cuda")
    out_score = torch.empty((Q, K_out), dtype=torch.float32, device="cuda")
    _check(load().kge_ensemble(_ptr(lists), M, Q, K, float(p), K_out, _ptr(out_idx), _ptr(out_score), _stream()),
           "kge_ensemble")
    return out_idx, out_score


DEBUG_KNOBS = {"fwd_one_role": 0, "gradt_one_role": 1, "score_f32_mfma": 2, "two_role": 3, "gradt_recompute": 4}


def debug_select(knob: str, value: bool):
    """kge_debug_select: tests and benchmarks only - take the alternative kernel of a job (process-wide)."""
    _check(load().kge_debug_select(DEBUG_KNOBS[knob], 1 if value else 0), "kge_debug_select")


def profile_enable(on):
    """True / False: every instrumented kernel / none; a list of slot names: those only."""
    if isinstance(on, (list, tuple, set)):
        mask = 0
        for s in on:
            mask |= 1 << PROF_SLOTS[s]
    else:
        mask = -1 if on else 0
    _check(load().kge_profile_enable(mask), "kge_profile_enable")


def profile_collect(slot: str):
    """(total milliseconds, launches) of the instrumented kernel `slot` since the last collect."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    _check(load().kge_profile_collect(PROF_SLOTS[slot], C.byref(ms), C.byref(n)), "kge_profile_collect")
    return ms.value, n.value


def calibrate_mfma(iters: int = 4096, varied: bool = False) -> float:
    """TFLOP/s of a loop of independent bf16 matrix instructions on this GPU (synchronises the stream); varied: on
    operands whose signs and mantissas differ from element to element instead of constant ones."""
    sink = torch.empty(2048 * 512, dtype=torch.float32, device="cuda")
    out = C.c_double(0.0)
    fn = load().kge_calibrate_mfma_varied if varied else load().kge_calibrate_mfma
    _check(fn(iters, _ptr(sink), sink.numel(), C.byref(out), _stream()), "kge_calibrate_mfma")
    return out.value


def calibrate_copy(nbytes: int = 1 << 30) -> float:
    """GB/s (read + written) of a plain streaming copy of nbytes on this GPU (synchronises the stream)."""
    src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").zero_()
    dst = torch.empty_like(src)
    out = C.c_double(0.0)
    _check(load().kge_calibrate_copy(_ptr(src), _ptr(dst), C.c_size_t(src.numel() * 4), C.byref(out), _stream()),
           "kge_calibrate_copy")
    return out.value


def partition_triples(h, t, part_size: int, D: int, ws: Workspace | None = None):
    n = h.numel()
    offsets = torch.empty(D * D + 1, dtype=torch.int64, device="cuda")
    order = torch.empty(n, dtype=torch.int64, device="cuda")
    ws = ws or _default_ws
    buf = ws.get(workspace_bytes(OP_PARTITION, None, n, D))
    _check(load().kge_partition_triples(_ptr(_i32(h)), _ptr(_i32(t)), n, part_size, D, _ptr(offsets), _ptr(order),
                                        _ptr(buf), buf.numel(), _stream()), "kge_partition_triples")
    return offsets, order


class TripleSampler:
    """Index of kge_sampler_build over device triple arrays (h, r, t: int32), and draws from it."""

    def __init__(self, h, r, t, part_size: int, D: int, n_rel: int, ws: Workspace | None = None):
        self.h, self.r, self.t = _i32(h), _i32(r), _i32(t)
        self.part_size, self.D, self.n_rel = part_size, D, n_rel
        n, groups = self.h.numel(), D * D * n_rel
        self.order = torch.empty(max(n, 1), dtype=torch.int64, device="cuda")[:n]
        self.rel_offsets = torch.empty(groups + 1, dtype=torch.int64, device="cuda")
        self.cdf = torch.empty(groups, dtype=torch.int64, device="cuda")       # bit pattern of uint64
        ws = ws or _default_ws
        buf = ws.get(workspace_bytes(OP_SAMPLER_BUILD, None, n, D))
        _check(load().kge_sampler_build(_ptr(self.h), _ptr(self.r), _ptr(self.t), n, part_size, D, n_rel,
                                        _ptr(self.order), _ptr(self.rel_offsets), _ptr(self.cdf), _ptr(buf),
                                        buf.numel(), _stream()), "kge_sampler_build")

    def sample(self, seed: int, step: int, stream_tag: int, bucket_lo: int, n_buckets: int, per_bucket: int,
               want_pos: bool = False):
        n = n_buckets * per_bucket
        oh, orr, ot = (torch.empty(n, dtype=torch.int32, device="cuda") for _ in range(3))
        pos = torch.empty(n, dtype=torch.int64, device="cuda") if want_pos else None
        # (an index over zero triples still hands over valid pointers: its storage has one spare element)
        order = self.order if self.order.numel() else self.order.new_zeros(1)
        h, r, t = ((x if x.numel() else x.new_zeros(1)) for x in (self.h, self.r, self.t))
        _check(load().kge_sample_triples(seed, step, stream_tag, bucket_lo, n_buckets, per_bucket, self.D, self.n_rel,
                                         _ptr(self.rel_offsets), _ptr(self.cdf), _ptr(order), _ptr(h),
                                         _ptr(r), _ptr(t), _ptr(pos), _ptr(oh), _ptr(orr), _ptr(ot),
                                         _stream()), "kge_sample_triples")
        return (oh, orr, ot, pos) if want_pos else (oh, orr, ot)


def sample_negatives_sharded(seed: int, step: int, stream_tag: int, part_size: int, n_ent: int, D: int,
                             per_shard: int, out=None):
    if out is None:
        out = torch.empty(D * per_shard, dtype=torch.int32, device="cuda")
    _check(load().kge_sample_negatives_sharded(seed, step, stream_tag, part_size, n_ent, D, per_shard, _ptr(out),
                                               _stream()), "kge_sample_negatives_sharded")
    return out


class Encoder:
    """kge_encoder_t over device tensors: shallow table, feature table, projections M_H, M_T (may be the same)."""

    def __init__(self, ent_s, feat, m_h, m_t, dropout: float = 0.0, reg_t: float = 0.0, reg_s: float = 0.0,
                 reg_f: float = 0.0, dropout_tag: int = 12):
        assert ent_s.dtype == feat.dtype == m_h.dtype == m_t.dtype and ent_s.dtype in (torch.float32, torch.bfloat16)
        self.ent_s, self.feat, self.m_h, self.m_t = ent_s, feat, m_h, m_t
        self.dim, self.feat_dim = ent_s.shape[1], feat.shape[1]
        self.ref = KgeEncoderT(1 if ent_s.dtype == torch.bfloat16 else 0, self.dim, self.feat_dim, dropout_tag, ent_s.shape[0], ent_s.data_ptr(),
                               feat.data_ptr(), m_h.data_ptr(), m_t.data_ptr(), ent_s.stride(0), feat.stride(0),
                               m_h.stride(0), dropout, reg_t, reg_s, reg_f)

    def _ws(self, op, B, N, ws):
        ws = ws or _default_ws
        n = load().kge_encode_workspace_bytes(op, C.byref(self.ref), B, N)
        if n == 0:
            raise KgeError("kge_encode_workspace_bytes: invalid arguments")
        return ws.get(n)

    def encode(self, h, t, neg, seed: int = 0, step: int = 0, ws: Workspace | None = None):
        """(e [(2B+N), dim] in the table dtype, proj fp32 [(2B+N), dim], reg fp32 [1])."""
        B, N = h.numel(), neg.numel()
        n = 2 * B + N
        e = torch.empty((n, self.dim), dtype=self.ent_s.dtype, device="cuda")
        proj = torch.empty((n, self.dim), dtype=torch.float32, device="cuda")
        reg = torch.empty(1, dtype=torch.float32, device="cuda")
        buf = self._ws(OP_ENCODE, B, N, ws)
        _check(load().kge_encode(C.byref(self.ref), _ptr(_i32(h)), _ptr(_i32(t)), B, _ptr(_i32(neg)), N, seed, step,
                                 _ptr(e), _ptr(proj), _ptr(reg), _ptr(buf), buf.numel(), _stream()), "kge_encode")
        return e, proj, reg

    def encode_bwd(self, h, t, neg, proj, de, seed: int = 0, step: int = 0, ws: Workspace | None = None):
        """(g_es fp32 [(2B+N), dim], g_mh, g_mt fp32 [dim, feat_dim])."""
        B, N = h.numel(), neg.numel()
        g_es = torch.empty((2 * B + N, self.dim), dtype=torch.float32, device="cuda")
        g_mh = torch.empty((self.dim, self.feat_dim), dtype=torch.float32, device="cuda")
        g_mt = torch.empty_like(g_mh)
        buf = self._ws(OP_ENCODE_BWD, B, N, ws)
        _check(load().kge_encode_bwd(C.byref(self.ref), _ptr(_i32(h)), _ptr(_i32(t)), B, _ptr(_i32(neg)), N, seed, step,
                                     _ptr(proj), _ptr(de), _ptr(g_es), _ptr(g_mh), _ptr(g_mt), _ptr(buf), buf.numel(),
                                     _stream()), "kge_encode_bwd")
        return g_es, g_mh, g_mt
