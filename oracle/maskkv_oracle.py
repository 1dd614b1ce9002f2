"""Float64 CPU oracle for the MaskKV eviction hot path.  TEST INFRASTRUCTURE ONLY.

This module is the plain definition of what the GPU library must compute, written
from the MaskKV paper (arXiv 2510.09309), Section 3.3 "The MaskKV Framework":

  * Stage 1, "Mask-Voting": the attention matrix of the mask queries against all
    keys and its column sums over the prompt (the two unnumbered equations that
    define ``A`` and ``I_j``).
  * The top-k eviction rule ``S_keep = argtopk(I, k_{l,h})`` that closes Stage 2.
  * Appendix "Prompt-state Exclusion": only the prompt's key/value rows are cached,
    so the evicted cache is a row gather of K and V.
  * The layer forward equation of Section 3.1 and the appendix proof's
    ``AttnOut_m = sum_j alpha_mj V_j``: bidirectional softmax attention of the
    response span over [kept prompt KV ; response KV].
  * Stage 2, head level: prompt preference ``P_h`` and the head budget formula
    ``k_{l,h}``; layer level: ``k_base``, ``k_imp``, group budgets and ``k_l``.
  * Variants: grouped-query heads (Dream-7B, Section 4.1, shares one KV head between
    several query heads; the paper does not say how votes map to a shared KV head, and
    this oracle lets every mask query of every query head in the group vote), and the
    response-token refresh criterion of the dLLM-Cache background (Section 3.1,
    ``S_shift``: cosine similarity of a token's value vector between two steps below
    a threshold).

Everything is float64 numpy on one head at a time, with no blocking, fusion or
reordering; a reader can check each function against the paper by eye.  It is only
ever imported by tests, by the smoke check and by the benchmark's CPU-baseline leg.
It shares no code with the HIP path and never imports it.

Score pooling (``pool``) is not part of the paper; it is the benchmark
specification's "pool window" and is defined here as a centred, edge-clipped
window over the prompt axis.

Parity pins: every function below is pinned in the CPU test-suite by closed forms,
invariants and pure-Python brute force.  The paper prints no worked numeric
example of ``I``, ``S_keep`` or an attention output, so there is no published
value to pin against: in that respect the oracle is "parity unpinned" (no golden
numbers from the paper exist); all pins are mathematical.
"""
from __future__ import annotations

import math

import numpy as np

__all__ = [
    "softmax_rows",
    "attention_matrix",
    "score",
    "pool",
    "select",
    "compact",
    "attend",
    "attend_full",
    "prompt_preference",
    "head_budgets",
    "layer_importance",
    "layer_budgets",
    "kv_cache_bytes",
    "score_grouped",
    "attend_grouped",
    "value_shift",
]


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def softmax_rows(S: np.ndarray) -> np.ndarray:
    """Row-wise softmax of a 2-D float64 matrix (the ``softmax_row`` of Stage 1).

    Subtracting the row maximum first is the standard overflow-safe evaluation of
    exp(s_ij) / sum_j exp(s_ij); it does not change the value.
    """
    S = _f64(S)
    m = S.max(axis=1, keepdims=True)
    E = np.exp(S - m)
    return E / E.sum(axis=1, keepdims=True)


def attention_matrix(Q: np.ndarray, K: np.ndarray, scale: float | None = None) -> np.ndarray:
    """A = softmax_row(Q K^T * scale), scale = 1/sqrt(d_k) by default (Stage 1, first equation).

    Q: [n_q, d], K: [N, d]; returns [n_q, N].  No causal or other mask: the model is
    bidirectional (Section 3.1).
    """
    Q = _f64(Q)
    K = _f64(K)
    assert Q.ndim == 2 and K.ndim == 2 and Q.shape[1] == K.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(Q.shape[1])
    return softmax_rows((Q @ K.T) * scale)


def score(Q_mask: np.ndarray, K_full: np.ndarray, n_prompt: int, scale: float | None = None):
    """Mask-Voting importance of the prompt tokens for ONE (layer, head).

    Q_mask: [n_m, d] queries of the mask (response-span) positions.
    K_full: [N, d] keys of the whole sequence, prompt rows first (N = n_prompt + n_resp).
    Returns (I, mass):
      I[j]  = sum_i A_ij for the prompt columns j < n_prompt      (Stage 1, second equation)
      mass  = sum_{j < n_prompt} I[j], the mask-to-prompt attention sum S_{m->p} used by
              the prompt-preference metric (Stage 2, head level).
    The softmax is normalised over all N keys (the paper's "all keys (K_full)"); only
    the prompt columns are kept afterwards.
    """
    A = attention_matrix(Q_mask, K_full, scale)
    assert 0 <= n_prompt <= A.shape[1]
    I = A[:, :n_prompt].sum(axis=0)
    return I, float(I.sum())


def pool(I: np.ndarray, window: int = 7, mode: str = "mean", dtype=np.float64) -> np.ndarray:
    """Smooth importance scores along the prompt axis (benchmark spec, not the paper).

    Centred window of odd width ``window`` and stride 1, clipped at the prompt ends:
    position j sees indices max(0, j-r) .. min(P-1, j+r) with r = (window-1)/2.
    ``mode='mean'`` divides by the number of in-range positions; ``mode='max'`` takes
    their maximum.  window == 1 is the identity.

    ``dtype=np.float32`` evaluates the mean in single precision, adding the in-range
    terms from the lowest index to the highest and then dividing by the count; this is
    the precision in which the GPU library decides the selection, so that index-exact
    comparisons use one and the same decision precision on both sides.
    """
    assert window >= 1 and window % 2 == 1
    assert mode in ("mean", "max")
    x = np.asarray(I, dtype=dtype)
    P = x.shape[0]
    r = (window - 1) // 2
    j = np.arange(P)
    if mode == "max":
        out = x.copy()
    else:
        out = np.zeros(P, dtype=dtype)
    count = np.zeros(P, dtype=dtype)
    # one window offset at a time, lowest index first: out[j] (+)= x[j+t] where j+t is in range
    for t in range(-r, r + 1):
        ok = (j + t >= 0) & (j + t < P)
        src = j[ok] + t
        if mode == "max":
            out[ok] = np.maximum(out[ok], x[src])
        else:
            out[ok] = out[ok] + x[src]
            count[ok] = count[ok] + dtype(1)
    if mode == "mean":
        out = out / count
    return out.astype(dtype, copy=False)


def select(I_pooled: np.ndarray, k: int) -> np.ndarray:
    """S_keep = argtopk(I, k) for one head (Stage 2, last equation).

    Returns the k = min(k, P) positions with the largest score as int32, sorted
    ascending.  Ties are broken towards the lower position (the paper is silent; the
    library fixes this choice).  k = 0 gives an empty set.
    """
    x = np.asarray(I_pooled)
    P = x.shape[0]
    assert k >= 0
    k = min(int(k), P)
    assert not np.isnan(x).any()
    # sort by (-score, index): lexsort's last key is the primary one
    order = np.lexsort((np.arange(P), -x.astype(np.float64)))
    return np.sort(order[:k]).astype(np.int32)


def compact(K_prompt: np.ndarray, V_prompt: np.ndarray, keep: np.ndarray):
    """Evict: keep only rows ``keep`` of the prompt's K and V (Prompt-state Exclusion).

    A pure row gather; dtype and bits are preserved.
    """
    keep = np.asarray(keep, dtype=np.int64)
    return K_prompt[keep].copy(), V_prompt[keep].copy()


def attend(Q_resp, Kc, Vc, K_resp, V_resp, scale: float | None = None, return_lse: bool = False):
    """Bidirectional attention of the response span over the evicted cache, ONE head.

    O_i = sum_j softmax_j(q_i . k_j * scale) v_j with j running over the kept prompt
    rows (Kc, Vc) followed by all response rows (K_resp, V_resp); no mask (layer
    forward equation, Section 3.1; appendix: AttnOut_m = sum_j alpha_mj V_j).
    Q_resp: [n_r, d]; Kc, Vc: [k, d] (k may be 0); K_resp, V_resp: [n_r, d].
    Returns O [n_r, d] float64 (and the natural-log row normaliser if asked).
    """
    Q = _f64(Q_resp)
    d = Q.shape[1]
    K = np.concatenate([_f64(Kc).reshape(-1, d), _f64(K_resp)], axis=0)
    V = np.concatenate([_f64(Vc).reshape(-1, d), _f64(V_resp)], axis=0)
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    S = (Q @ K.T) * scale
    A = softmax_rows(S)
    O = A @ V
    if return_lse:
        m = S.max(axis=1)
        lse = m + np.log(np.exp(S - m[:, None]).sum(axis=1))
        return O, lse
    return O


def attend_full(Q_resp, K_full, V_full, scale: float | None = None, return_lse: bool = False):
    """Attention of the response span over the whole un-evicted sequence, ONE head.

    K_full, V_full: [N, d], prompt rows then response rows.  This is ``attend`` with
    nothing evicted; it is the cost the eviction removes.
    """
    Q = _f64(Q_resp)
    d = Q.shape[1]
    empty = np.zeros((0, d))
    return attend(Q, empty, empty, K_full, V_full, scale, return_lse)


def prompt_preference(mass: np.ndarray, n_mask: int) -> np.ndarray:
    """P_h = S_{m->p} / (S_{m->p} + S_{m->m}) per head (Stage 2, head level).

    The two sums together are the whole attention mass of the n_mask mask rows, i.e.
    exactly n_mask, so P_h = mass_h / n_mask.
    """
    return _f64(mass) / float(n_mask)


def head_budgets(P_h: np.ndarray, k_l: int, alpha: float = 0.1) -> np.ndarray:
    """k_{l,h} = floor(alpha*k_l + (1-alpha) * N_h * k_l * P_h / sum_j P_j)  (head budget formula).

    k_l is the layer's per-head average budget, N_h the number of heads.  The paper does not say what a
    layer gets whose heads all have zero prompt preference (no prompt at all: the normalised preference
    is 0/0).  Reading: with nothing to tell the heads apart the normalised preferences are equal, 1/N_h
    each, which gives every head the average k_l.
    """
    P_h = _f64(P_h)
    n_h = P_h.shape[0]
    total = P_h.sum()
    p_hat = P_h / total if total > 0.0 else np.full(n_h, 1.0 / n_h)
    return np.floor(alpha * k_l + (1.0 - alpha) * n_h * k_l * p_hat).astype(np.int64)


def layer_importance(h_in: np.ndarray, h_out: np.ndarray) -> float:
    """I^(l) = 1 - mean_i cos_sim(h_in_i, h_out_i) over the n tokens (layer importance metric)."""
    a = _f64(h_in)
    b = _f64(h_out)
    cos = (a * b).sum(axis=1) / (np.linalg.norm(a, axis=1) * np.linalg.norm(b, axis=1))
    return float(1.0 - cos.mean())


def layer_budgets(importance: np.ndarray, k_p: int, beta: float = 0.4, boundary=None) -> np.ndarray:
    """Boundary-aware layer budgets k_l (Stage 2, layer level).

    k_base = floor(beta*k_p/L); k_imp = k_p - L*k_base; k_imp is split between the
    boundary group (first and last layer unless given) and the middle group in
    proportion to their summed importance; every layer gets k_base plus the floor of
    an equal share of its group's part.
    """
    imp = _f64(importance)
    L = imp.shape[0]
    if boundary is None:
        boundary = [0, L - 1] if L > 1 else [0]
    bset = sorted(set(int(i) for i in boundary))
    mset = [i for i in range(L) if i not in bset]
    k_base = math.floor(beta * k_p / L)
    k_imp = k_p - L * k_base
    I_B = imp[bset].sum()
    I_M = imp[mset].sum() if mset else 0.0
    kg_B = k_imp * I_B / (I_B + I_M)
    kg_M = k_imp - kg_B
    out = np.full(L, k_base, dtype=np.int64)
    for i in bset:
        out[i] += math.floor(kg_B / len(bset))
    for i in mset:
        out[i] += math.floor(kg_M / len(mset))
    return out


def kv_cache_bytes(seq_len: int, n_heads: int, d_head: int, elem_bytes: int = 2) -> int:
    """Mem_KV = 2 * L * H * d_head * s_bf16 bytes per layer (appendix, evaluation metrics)."""
    return 2 * seq_len * n_heads * d_head * elem_bytes


def score_grouped(Q_heads: np.ndarray, K_full: np.ndarray, n_prompt: int, scale: float | None = None):
    """Mask-Voting for ONE key/value head shared by g query heads (grouped-query attention).

    Q_heads: [g, n_m, d] mask queries of the g query heads that read this KV head;
    K_full: [N, d].  Every mask query of every head in the group votes:
      I[j] = sum_{h in group} sum_i A^(h)_ij,   mass = sum_{j < n_prompt} I[j].
    The paper evaluates a grouped-query model (Dream-7B) without stating this mapping;
    the plain sum is the reading taken here (it is Stage 1's sum over "all mask
    queries", with the queries of one KV head's group being all of its queries).
    """
    Q_heads = _f64(Q_heads)
    assert Q_heads.ndim == 3
    I = np.zeros(n_prompt, dtype=np.float64)
    for g in range(Q_heads.shape[0]):
        I_g, _ = score(Q_heads[g], K_full, n_prompt, scale)
        I = I + I_g
    return I, float(I.sum())


def attend_grouped(Q_heads, Kc, Vc, K_resp, V_resp, scale: float | None = None):
    """Attention of the g query heads of one group over their shared evicted cache.

    Q_heads: [g, n_r, d]; the cache and the response rows belong to the group's single KV
    head.  Returns O [g, n_r, d]: every query head attends on its own (Section 3.1's layer
    forward equation per head), only the keys and values are shared.
    """
    Q_heads = _f64(Q_heads)
    return np.stack([attend(Q_heads[g], Kc, Vc, K_resp, V_resp, scale) for g in range(Q_heads.shape[0])])


def value_shift(V_now: np.ndarray, V_prev: np.ndarray, delta: float):
    """Response tokens whose value vector moved between two denoising steps (Section 3.1, S_shift).

    V_now, V_prev: [n, width] value features of the n response tokens at steps t and t-1.
    Returns (cos, refresh): cos[i] = cos_sim(V_now[i], V_prev[i]); refresh = ascending int32
    positions i with cos[i] < delta (the tokens dLLM-Cache recomputes at this step in
    addition to the periodic refresh).
    """
    a = _f64(V_now)
    b = _f64(V_prev)
    assert a.shape == b.shape and a.ndim == 2
    cos = (a * b).sum(axis=1) / (np.linalg.norm(a, axis=1) * np.linalg.norm(b, axis=1))
    refresh = np.nonzero(cos < delta)[0].astype(np.int32)
    return cos, refresh
