"""ctypes binding of libmaskkv.so: argument marshalling only.

Every function mirrors the C entry point of the same name in ``include/maskkv.h`` and takes
torch device tensors; torch is used for device memory and streams, nothing is computed here.
If the shared library has not been built the import of this module fails loudly: there is no
CPU or PyTorch fallback.
"""
from __future__ import annotations

import ctypes as ct
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# MASKKV_LIB_PATH selects another build of the same library (e.g. an instrumented one)
LIB_PATH = os.environ.get("MASKKV_LIB_PATH", os.path.join(_HERE, "libmaskkv.so"))

MASKKV_F32, MASKKV_BF16 = 0, 1
POOL_MEAN, POOL_MAX = 0, 1
MAX_BATCH = 64

SYMBOLS = [
    "maskkv_version", "maskkv_strerror", "maskkv_last_error",
    "maskkv_score_workspace_bytes", "maskkv_score", "maskkv_score_given_lse", "maskkv_score_static",
    "maskkv_select_workspace_bytes", "maskkv_select",
    "maskkv_compact",
    "maskkv_attend_workspace_bytes", "maskkv_attend", "maskkv_attend_full",
    "maskkv_head_budgets",
    "maskkv_layer_importance_workspace_bytes", "maskkv_layer_importance", "maskkv_layer_budgets",
    "maskkv_value_shift",
]


class MaskKVError(RuntimeError):
    def __init__(self, status: int, what: str, detail: str):
        super().__init__(f"{what} failed: status {status} ({detail})")
        self.status = status


class _CTensor(ct.Structure):
    _fields_ = [("ptr", ct.c_void_p), ("stride_b", ct.c_int64), ("stride_h", ct.c_int64),
                ("stride_t", ct.c_int64), ("seq_start", ct.POINTER(ct.c_int32))]


class _CDesc(ct.Structure):
    _fields_ = [("B", ct.c_int32), ("H", ct.c_int32), ("d", ct.c_int32), ("dtype", ct.c_int32),
                ("n_resp", ct.c_int32), ("n_query", ct.c_int32), ("P_max", ct.c_int32), ("q_per_kv", ct.c_int32),
                ("prompt_len", ct.POINTER(ct.c_int32))]


def _load() -> ct.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2510_09309_amd.build); "
            "this package has no fallback path")
    lib = ct.CDLL(LIB_PATH)
    lib.maskkv_strerror.restype = ct.c_char_p
    lib.maskkv_last_error.restype = ct.c_char_p
    for name in SYMBOLS:
        getattr(lib, name)  # raises AttributeError if a declared entry point is not exported
    return lib


_lib = _load()


@dataclass
class Desc:
    """Python mirror of maskkv_desc."""
    B: int
    H: int
    d: int
    dtype: int
    n_resp: int
    P_max: int
    n_query: Optional[int] = None
    prompt_len: Optional[Sequence[int]] = None
    q_per_kv: int = 0   # query heads per key/value head (0 or 1: multi-head attention); H counts KV heads

    def c(self) -> _CDesc:
        nq = self.n_resp if self.n_query is None else self.n_query
        c = _CDesc(self.B, self.H, self.d, self.dtype, self.n_resp, nq, self.P_max, int(self.q_per_kv), None)
        if self.prompt_len is not None:
            arr = (ct.c_int32 * len(self.prompt_len))(*[int(x) for x in self.prompt_len])
            c._keep = arr
            c.prompt_len = ct.cast(arr, ct.POINTER(ct.c_int32))
        return c


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return MASKKV_BF16
    if t.dtype == torch.float32:
        return MASKKV_F32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def tensor_view(t: torch.Tensor, seq_start: Optional[Sequence[int]] = None) -> _CTensor:
    """Describe a [B, H, T, d] device tensor (any strides with a contiguous last axis)."""
    assert t.is_cuda and t.dim() == 4 and t.stride(3) == 1, "need a [B,H,T,d] device tensor with contiguous d"
    v = _CTensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2), None)
    if seq_start is not None:
        arr = (ct.c_int32 * len(seq_start))(*[int(x) for x in seq_start])
        v._keep = arr
        v.seq_start = ct.cast(arr, ct.POINTER(ct.c_int32))
    v._tensor = t
    return v


def _as_view(t) -> _CTensor:
    return t if isinstance(t, _CTensor) else tensor_view(t)


def _stream(stream) -> ct.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ct.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status: int, what: str) -> None:
    if status != 0:
        detail = _lib.maskkv_last_error().decode() or _lib.maskkv_strerror(status).decode()
        raise MaskKVError(status, what, detail)


def _ptr(t: Optional[torch.Tensor]) -> ct.c_void_p:
    return ct.c_void_p(0 if t is None else t.data_ptr())


def _ws(t: Optional[torch.Tensor]):
    return _ptr(t), ct.c_size_t(0 if t is None else t.numel() * t.element_size())


def maskkv_version() -> int:
    return int(_lib.maskkv_version())


def maskkv_score_workspace_bytes(desc: Desc) -> int:
    n = ct.c_size_t(0)
    _check(_lib.maskkv_score_workspace_bytes(ct.byref(desc.c()), ct.byref(n)), "maskkv_score_workspace_bytes")
    return int(n.value)


def maskkv_select_workspace_bytes(desc: Desc) -> int:
    n = ct.c_size_t(0)
    _check(_lib.maskkv_select_workspace_bytes(ct.byref(desc.c()), ct.byref(n)), "maskkv_select_workspace_bytes")
    return int(n.value)


def maskkv_attend_workspace_bytes(desc: Desc, full: bool) -> int:
    n = ct.c_size_t(0)
    _check(_lib.maskkv_attend_workspace_bytes(ct.byref(desc.c()), ct.c_int(1 if full else 0), ct.byref(n)),
           "maskkv_attend_workspace_bytes")
    return int(n.value)


def maskkv_score(desc: Desc, Q_mask, K_full, scale: float, scores: torch.Tensor, score_stride: int,
                 prompt_mass: Optional[torch.Tensor], workspace: Optional[torch.Tensor], stream=None) -> None:
    q, k = _as_view(Q_mask), _as_view(K_full)
    wp, wn = _ws(workspace)
    _check(_lib.maskkv_score(ct.byref(desc.c()), ct.byref(q), ct.byref(k), ct.c_float(scale), _ptr(scores),
                             ct.c_int64(score_stride), _ptr(prompt_mass), wp, wn, _stream(stream)), "maskkv_score")


def maskkv_score_given_lse(desc: Desc, Q_mask, K_full, scale: float, row_lse: torch.Tensor, scores: torch.Tensor,
                           score_stride: int, prompt_mass: Optional[torch.Tensor], workspace: Optional[torch.Tensor],
                           stream=None) -> None:
    """maskkv_score from the rows' natural-log softmax normalisers (as maskkv_attend_full returns them)."""
    q, k = _as_view(Q_mask), _as_view(K_full)
    wp, wn = _ws(workspace)
    _check(_lib.maskkv_score_given_lse(ct.byref(desc.c()), ct.byref(q), ct.byref(k), ct.c_float(scale), _ptr(row_lse),
                                       _ptr(scores), ct.c_int64(score_stride), _ptr(prompt_mass), wp, wn,
                                       _stream(stream)), "maskkv_score_given_lse")


def maskkv_score_static(desc: Desc, Q_mask, K_full, scale: float, scores: torch.Tensor, score_stride: int,
                        prompt_mass: Optional[torch.Tensor], stream=None) -> None:
    """maskkv_score with the library's own static scratch array instead of a caller workspace."""
    q, k = _as_view(Q_mask), _as_view(K_full)
    _check(_lib.maskkv_score_static(ct.byref(desc.c()), ct.byref(q), ct.byref(k), ct.c_float(scale), _ptr(scores),
                                    ct.c_int64(score_stride), _ptr(prompt_mass), _stream(stream)),
           "maskkv_score_static")


def _host_i32(values: Optional[Sequence[int]]):
    if values is None:
        return None
    return (ct.c_int32 * len(values))(*[int(x) for x in values])


def maskkv_select(desc: Desc, scores: torch.Tensor, score_stride: int, pool_window: int, pool_mode: int,
                  budgets: torch.Tensor, idx: torch.Tensor, cu_budget: torch.Tensor, capacity: int,
                  workspace: Optional[torch.Tensor], stream=None, budgets_host: Optional[Sequence[int]] = None) -> None:
    wp, wn = _ws(workspace)
    _check(_lib.maskkv_select(ct.byref(desc.c()), _ptr(scores), ct.c_int64(score_stride), ct.c_int(pool_window),
                              ct.c_int(pool_mode), _ptr(budgets), _host_i32(budgets_host), _ptr(idx), _ptr(cu_budget),
                              ct.c_int64(capacity), wp, wn, _stream(stream)), "maskkv_select")


def maskkv_compact(desc: Desc, K, V, idx: torch.Tensor, cu_budget: torch.Tensor, capacity: int,
                   Kc: torch.Tensor, Vc: torch.Tensor, stream=None) -> None:
    k, v = _as_view(K), _as_view(V)
    _check(_lib.maskkv_compact(ct.byref(desc.c()), ct.byref(k), ct.byref(v), _ptr(idx), _ptr(cu_budget),
                               ct.c_int64(capacity), _ptr(Kc), _ptr(Vc), _stream(stream)), "maskkv_compact")


def maskkv_attend(desc: Desc, Q_resp, Kc: torch.Tensor, Vc: torch.Tensor, cu_budget: torch.Tensor, capacity: int,
                  K_resp, V_resp, scale: float, O, lse: Optional[torch.Tensor],
                  workspace: Optional[torch.Tensor], stream=None) -> None:
    q, k2, v2, o = _as_view(Q_resp), _as_view(K_resp), _as_view(V_resp), _as_view(O)
    wp, wn = _ws(workspace)
    _check(_lib.maskkv_attend(ct.byref(desc.c()), ct.byref(q), _ptr(Kc), _ptr(Vc), _ptr(cu_budget),
                              ct.c_int64(capacity), ct.byref(k2), ct.byref(v2), ct.c_float(scale), ct.byref(o),
                              _ptr(lse), wp, wn, _stream(stream)), "maskkv_attend")


def maskkv_attend_full(desc: Desc, Q_resp, K_full, V_full, scale: float, O, lse: Optional[torch.Tensor],
                       workspace: Optional[torch.Tensor], stream=None) -> None:
    q, k2, v2, o = _as_view(Q_resp), _as_view(K_full), _as_view(V_full), _as_view(O)
    wp, wn = _ws(workspace)
    _check(_lib.maskkv_attend_full(ct.byref(desc.c()), ct.byref(q), ct.byref(k2), ct.byref(v2), ct.c_float(scale),
                                   ct.byref(o), _ptr(lse), wp, wn, _stream(stream)), "maskkv_attend_full")


def maskkv_head_budgets(desc: Desc, prompt_mass: torch.Tensor, k_l: int, alpha: float, budgets: torch.Tensor,
                        stream=None) -> None:
    _check(_lib.maskkv_head_budgets(ct.byref(desc.c()), _ptr(prompt_mass), ct.c_int32(k_l), ct.c_float(alpha),
                                    _ptr(budgets), _stream(stream)), "maskkv_head_budgets")


def maskkv_layer_importance_workspace_bytes() -> int:
    n = ct.c_size_t(0)
    _check(_lib.maskkv_layer_importance_workspace_bytes(ct.byref(n)), "maskkv_layer_importance_workspace_bytes")
    return int(n.value)


def maskkv_layer_importance(h_in: torch.Tensor, h_out: torch.Tensor, importance: torch.Tensor,
                            workspace: Optional[torch.Tensor], stream=None) -> None:
    """h_in, h_out: [n_tokens, hidden] device tensors of the same dtype and row stride; importance: float32 [1]."""
    assert h_in.is_cuda and h_in.dim() == 2 and h_in.stride(1) == 1 and h_out.shape == h_in.shape
    assert h_out.stride() == h_in.stride() and h_out.dtype == h_in.dtype
    wp, wn = _ws(workspace)
    _check(_lib.maskkv_layer_importance(_ptr(h_in), _ptr(h_out), ct.c_int64(h_in.shape[0]), ct.c_int32(h_in.shape[1]),
                                        ct.c_int32(_dtype_code(h_in)), ct.c_int64(h_in.stride(0)), _ptr(importance),
                                        wp, wn, _stream(stream)), "maskkv_layer_importance")


def maskkv_layer_budgets(importance: Sequence[float], k_p: int, beta: float,
                         boundary: Optional[Sequence[int]] = None) -> list:
    """Host arithmetic: per-layer budgets k_l from the layer importances."""
    n = len(importance)
    imp = (ct.c_float * n)(*[float(x) for x in importance])
    out = (ct.c_int64 * n)()
    if boundary is None:
        bptr, nb = None, 0
    else:
        barr = (ct.c_int32 * len(boundary))(*[int(x) for x in boundary])
        bptr, nb = barr, len(boundary)
    _check(_lib.maskkv_layer_budgets(imp, ct.c_int32(n), ct.c_int64(int(k_p)), ct.c_float(beta), bptr, ct.c_int32(nb),
                                     out), "maskkv_layer_budgets")
    return [int(x) for x in out]


def maskkv_value_shift(V_now: torch.Tensor, V_prev: torch.Tensor, delta: float, cos: torch.Tensor,
                       refresh: torch.Tensor, count: torch.Tensor, stream=None) -> None:
    """V_now, V_prev: [n_tokens, width] device tensors; cos: float32 [n]; refresh: int32 [n]; count: int32 [1]."""
    assert V_now.is_cuda and V_now.dim() == 2 and V_now.stride(1) == 1 and V_prev.shape == V_now.shape
    assert V_prev.stride() == V_now.stride() and V_prev.dtype == V_now.dtype
    assert cos.dtype == torch.float32 and cos.numel() >= V_now.shape[0]
    assert refresh.dtype == torch.int32 and refresh.numel() >= V_now.shape[0] and count.dtype == torch.int32
    _check(_lib.maskkv_value_shift(_ptr(V_now), _ptr(V_prev), ct.c_int64(V_now.shape[0]), ct.c_int32(V_now.shape[1]),
                                   ct.c_int32(_dtype_code(V_now)), ct.c_int64(V_now.stride(0)), ct.c_float(delta),
                                   _ptr(cos), _ptr(refresh), _ptr(count), _stream(stream)), "maskkv_value_shift")


def raw_library() -> ct.CDLL:
    """The loaded CDLL (for tests that exercise error paths with hand-built arguments)."""
    return _lib
