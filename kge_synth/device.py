"""Device-side table fill (same function as kge_synth.uniform_rows) for tables too large to
generate on the host.  Input generation only."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fill.hip")
LIB_PATH = os.path.join(_HERE, "libkge_synth.so")
_lib = None


def build() -> str:
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-fPIC", "-shared", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-o", LIB_PATH, _SRC]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(r.stderr)
    return LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run kge_synth.device.build()")
        _lib = C.CDLL(LIB_PATH)
        _lib.synth_fill_uniform.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int64, C.c_uint64, C.c_uint32,
                                            C.c_float, C.c_int, C.c_int64, C.c_void_p]
    return _lib


def fill_uniform(t, seed: int, tag: int, amp: float, row0: int = 0):
    """Fills the 2-D device tensor t (fp32 or bf16) in place; row i gets table row row0 + i."""
    import torch
    assert t.is_cuda and t.dim() == 2 and t.stride(1) == 1 and t.dtype in (torch.float32, torch.bfloat16)
    rc = _load().synth_fill_uniform(C.c_void_p(t.data_ptr()), t.shape[0], t.shape[1], t.stride(0), seed, tag,
                                    float(amp), 1 if t.dtype == torch.bfloat16 else 0, row0,
                                    C.c_void_p(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise RuntimeError("synth_fill_uniform failed")
    return t
