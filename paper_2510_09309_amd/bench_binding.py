"""ctypes binding of libmaskkv_bench.so (``include/maskkv_bench.h``): measurement probes and maskkv_score with stage
marks.  For benchmark harnesses and their tests only; nothing of the method's path goes through this module."""
from __future__ import annotations

import ctypes as ct
import os
from typing import Optional, Sequence

import torch

from . import binding as _b

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MASKKV_BENCH_LIB_PATH", os.path.join(_HERE, "libmaskkv_bench.so"))
SYMBOLS = ["maskkv_bench_last_error", "maskkv_bench_probe", "maskkv_bench_score_marked"]


def _load() -> ct.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2510_09309_amd.build)")
    lib = ct.CDLL(LIB_PATH)
    lib.maskkv_bench_last_error.restype = ct.c_char_p
    for name in SYMBOLS:
        getattr(lib, name)
    return lib


_lib = _load()


def maskkv_bench_probe(which: int, iters: int, src: Optional[torch.Tensor], dst: torch.Tensor, groups: int,
                       stream=None) -> float:
    """Enqueue a probe (0 matrix pipe on constants, 1 v_exp_f32, 2 copy src -> dst, 3 read of src, 4 the scoring
    instruction mix, 5 matrix pipe on the data in src, 6 the form-and-reduce pipeline on the data in src, 7 / 8 / 9 eight-
    wave workgroups whose waves 0-3 issue MFMAs on the data in src and whose waves 4-7 issue the vector work: both
    halves, the matrix half alone, the vector half alone); returns the work it does (flops, exponentials or bytes)."""
    work = ct.c_double(0.0)
    nbytes = src.numel() * src.element_size() if src is not None else 0
    status = _lib.maskkv_bench_probe(ct.c_int(which), ct.c_int32(iters), _b._ptr(src) if src is not None else None,
                                     _b._ptr(dst), ct.c_int64(nbytes), ct.c_int64(dst.numel() * dst.element_size()),
                                     ct.c_int32(groups), _b._stream(stream), ct.byref(work))
    if status != 0:
        raise _b.MaskKVError(status, "maskkv_bench_probe", _lib.maskkv_bench_last_error().decode())
    return float(work.value)


def maskkv_bench_score_marked(desc: "_b.Desc", Q_mask, K_full, scale: float, scores: torch.Tensor, score_stride: int,
                              prompt_mass: Optional[torch.Tensor], workspace: Optional[torch.Tensor],
                              events: Sequence[int], stream=None) -> None:
    """``events``: four raw hipEvent_t handles (0 to skip one), recorded at the stage boundaries of the call."""
    q, k = _b._as_view(Q_mask), _b._as_view(K_full)
    wp, wn = _b._ws(workspace)
    ev = (ct.c_void_p * 4)(*[ct.c_void_p(int(e)) for e in events])
    _b._check(_lib.maskkv_bench_score_marked(ct.byref(desc.c()), ct.byref(q), ct.byref(k), ct.c_float(scale),
                                             _b._ptr(scores), ct.c_int64(score_stride), _b._ptr(prompt_mass), wp, wn,
                                             _b._stream(stream), ev), "maskkv_bench_score_marked")


def raw_library() -> ct.CDLL:
    return _lib
