"""Shared plumbing of the GPU parity tests: upload seeded inputs, call the C ABI, run the oracle."""
from __future__ import annotations

import math
from typing import List, Sequence

import numpy as np
import torch

from oracle import maskkv_oracle as orc
from paper_2510_09309_amd import synth

SCORE_RTOL = 1e-3        # spec tolerance for fp32 scores
BAND_RTOL = 1e-4         # index sets may differ only where the pooled score is this close to the k-th largest
ATTEND_ATOL_BF16 = 2e-2  # bf16 inputs, fp32 accumulation
ATTEND_ATOL_F32 = 2e-5   # fp32 inputs: fp32 accumulation of d<=128 products, probabilities in fp32


def mk():
    from paper_2510_09309_amd import binding
    return binding


def torch_dtype(name: str):
    return torch.bfloat16 if name == "bf16" else torch.float32


def upload(x: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 array of dtype-exact values -> device tensor of that dtype (conversion is exact)."""
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda").to(torch_dtype(dtype))


class Batch:
    """A batch of sequences (one LayerInputs per sequence), padded to [B, H, N_max, d] on the device."""

    def __init__(self, layers: Sequence[synth.LayerInputs]):
        self.layers = list(layers)
        L0 = self.layers[0]
        self.B, self.H, self.d, self.n_m, self.dtype = len(self.layers), L0.H, L0.d, L0.n_m, L0.dtype
        self.P = [L.P for L in self.layers]
        self.P_max = max(self.P)
        N_max = self.P_max + self.n_m
        K = np.zeros((self.B, self.H, N_max, self.d), dtype=np.float32)
        V = np.zeros_like(K)
        Q = np.zeros((self.B, self.H, self.n_m, self.d), dtype=np.float32)
        for b, L in enumerate(self.layers):
            K[b, :, :L.N] = L.K
            V[b, :, :L.N] = L.V
            Q[b] = L.Q
        self.K, self.V, self.Q = upload(K, self.dtype), upload(V, self.dtype), upload(Q, self.dtype)
        m = mk()
        self.desc = m.Desc(B=self.B, H=self.H, d=self.d,
                           dtype=m.MASKKV_BF16 if self.dtype == "bf16" else m.MASKKV_F32,
                           n_resp=self.n_m, P_max=self.P_max,
                           prompt_len=None if all(p == self.P_max for p in self.P) else self.P)

    def resp_views(self):
        """Response-span K and V of every sequence as [B, H, n_m, d] views with per-sequence offsets."""
        m = mk()
        return (m.tensor_view(self.K, seq_start=self.P), m.tensor_view(self.V, seq_start=self.P))


def workspace(nbytes: int):
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")


def gpu_score(batch: Batch, scale: float = 0.0):
    m = mk()
    stride = (batch.P_max + 63) // 64 * 64
    scores = torch.full((batch.B * batch.H, max(stride, 1)), float("nan"), dtype=torch.float32, device="cuda")
    mass = torch.full((batch.B * batch.H,), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(m.maskkv_score_workspace_bytes(batch.desc))
    m.maskkv_score(batch.desc, batch.Q, batch.K, scale, scores, scores.stride(0), mass, ws)
    torch.cuda.synchronize()
    return scores, mass


def gpu_score_given_lse(batch: Batch, row_lse: torch.Tensor, scale: float = 0.0):
    """Scores and prompt mass from given natural-log row normalisers [B*H*n_m]; padding stays NaN."""
    m = mk()
    scores = torch.full((batch.B * batch.H, batch.P_max), float("nan"), dtype=torch.float32, device="cuda")
    mass = torch.full((batch.B * batch.H,), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(m.maskkv_score_workspace_bytes(batch.desc))
    m.maskkv_score_given_lse(batch.desc, batch.Q, batch.K, scale, row_lse, scores, batch.P_max, mass, ws)
    torch.cuda.synchronize()
    return scores, mass


def gpu_select(batch: Batch, scores: torch.Tensor, budgets: np.ndarray, window: int, mode: int = 0, capacity=None):
    m = mk()
    BH = batch.B * batch.H
    bud = torch.from_numpy(np.asarray(budgets, dtype=np.int32)).to("cuda")
    clamped = [min(max(int(budgets[i]), 0), batch.P[i // batch.H]) for i in range(BH)]
    cap = int(sum(clamped)) if capacity is None else capacity
    idx = torch.full((max(cap, 1),), -1, dtype=torch.int32, device="cuda")
    cu = torch.full((BH + 1,), -1, dtype=torch.int32, device="cuda")
    ws = workspace(m.maskkv_select_workspace_bytes(batch.desc))
    m.maskkv_select(batch.desc, scores, scores.stride(0), window, mode, bud, idx, cu, cap, ws)
    torch.cuda.synchronize()
    return idx, cu, cap


def gpu_compact(batch: Batch, idx, cu, cap):
    m = mk()
    Kc = torch.zeros((max(cap, 1), batch.d), dtype=torch_dtype(batch.dtype), device="cuda")
    Vc = torch.zeros_like(Kc)
    m.maskkv_compact(batch.desc, batch.K, batch.V, idx, cu, cap, Kc, Vc)
    torch.cuda.synchronize()
    return Kc, Vc


def gpu_attend(batch: Batch, Kc, Vc, cu, cap, Q=None, Kr=None, Vr=None, scale: float = 0.0):
    m = mk()
    Q = batch.Q if Q is None else Q
    if Kr is None:
        Kr, Vr = batch.resp_views()
    O = torch.full((batch.B, batch.H, batch.n_m, batch.d), float("nan"), dtype=torch_dtype(batch.dtype), device="cuda")
    lse = torch.full((batch.B * batch.H * batch.n_m,), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(m.maskkv_attend_workspace_bytes(batch.desc, False))
    m.maskkv_attend(batch.desc, Q, Kc, Vc, cu, cap, Kr, Vr, scale, O, lse, ws)
    torch.cuda.synchronize()
    return O, lse


def gpu_attend_full(batch: Batch, scale: float = 0.0):
    m = mk()
    O = torch.full((batch.B, batch.H, batch.n_m, batch.d), float("nan"), dtype=torch_dtype(batch.dtype), device="cuda")
    lse = torch.full((batch.B * batch.H * batch.n_m,), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(m.maskkv_attend_workspace_bytes(batch.desc, True))
    m.maskkv_attend_full(batch.desc, batch.Q, batch.K, batch.V, scale, O, lse, ws)
    torch.cuda.synchronize()
    return O, lse


# ------------------------------------------------------------------------------------------ checks
def check_scores(batch: Batch, scores: torch.Tensor, mass: torch.Tensor, heads=None, rtol=SCORE_RTOL, scale=None):
    """Element-wise comparison of GPU scores with the oracle; returns the worst relative error seen."""
    sc = scores.cpu().numpy()
    ms = mass.cpu().numpy()
    worst = 0.0
    for b, L in enumerate(batch.layers):
        for h in (range(batch.H) if heads is None else heads):
            I, m_or = orc.score(L.Q[h], L.K[h], L.P, scale)
            got = sc[b * batch.H + h, :L.P].astype(np.float64)
            assert np.isfinite(got).all(), f"non-finite scores b={b} h={h}"
            rel = np.abs(got - I) / np.abs(I)
            worst = max(worst, float(rel.max()) if L.P else 0.0)
            assert rel.max() <= rtol if L.P else True, f"b={b} h={h}: score rel err {rel.max():.3e} > {rtol}"
            assert abs(ms[b * batch.H + h] - m_or) <= rtol * max(abs(m_or), 1e-30) + 1e-30, \
                f"b={b} h={h}: prompt mass {ms[b * batch.H + h]} vs {m_or}"
            # untouched padding
            assert np.isnan(sc[b * batch.H + h, L.P:]).all()
    return worst


def check_keep_against_oracle(pooled64: np.ndarray, k: int, keep_gpu: np.ndarray, tag: str = ""):
    """Index set parity with the near-tie band: differences only where the pooled score is within
    BAND_RTOL (relative) of the oracle's k-th largest value; what is unique is compared exactly."""
    P = pooled64.shape[0]
    k = min(max(k, 0), P)
    assert keep_gpu.shape[0] == k, f"{tag}: kept {keep_gpu.shape[0]} != k {k}"
    if k == 0:
        return 0
    assert np.all(np.diff(keep_gpu) > 0), f"{tag}: indices not strictly ascending"
    assert keep_gpu[0] >= 0 and keep_gpu[-1] < P, f"{tag}: index out of range"
    ref = orc.select(pooled64, k)
    tau = np.sort(pooled64)[::-1][k - 1]
    diff = np.setxor1d(ref, keep_gpu)
    if diff.size:
        gap = np.abs(pooled64[diff] - tau)
        assert np.all(gap < BAND_RTOL * abs(tau)), \
            f"{tag}: {diff.size} indices differ outside the near-tie band (worst gap {gap.max() / abs(tau):.3e})"
    return int(diff.size)


def split_idx(idx: torch.Tensor, cu: torch.Tensor):
    idx_h = idx.cpu().numpy()
    cu_h = cu.cpu().numpy()
    return [idx_h[cu_h[i]:cu_h[i + 1]] for i in range(cu_h.shape[0] - 1)], cu_h
