"""Variants of the hot path against the float64 oracle (needs an MI355X): grouped-query heads and the
value-shift refresh criterion."""
import numpy as np
import pytest
import torch

from oracle import maskkv_oracle as orc
from paper_2510_09309_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu

COS_ATOL = 5e-6       # fp32 accumulation of `width` products against float64, values <= 1
SHIFT_BAND = 2e-5     # refresh sets may differ only where the cosine is this close to the threshold


# ------------------------------------------------------------------------------------------ grouped queries
def run_grouped(seed, H, g, d, P, n_m, dtype, budgets, window=7, sigma=1.0):
    """Whole path with g query heads per KV head; every step is compared with the oracle."""
    m = hp.mk()
    L = synth.make_layer(seed, H, d, P, n_m, dtype, n_planted=max(P // 50, 1), amplitude=2.5, sigma=sigma)
    Qg = synth.make_grouped_queries(seed + 1, L, g, sigma=sigma)            # [H*g, n_m, d]
    K, V = hp.upload(L.K[None], dtype), hp.upload(L.V[None], dtype)          # [1, H, N, d]
    Q = hp.upload(Qg[None], dtype)                                          # [1, H*g, n_m, d]
    desc = m.Desc(B=1, H=H, d=d, dtype=m.MASKKV_BF16 if dtype == "bf16" else m.MASKKV_F32, n_resp=n_m, P_max=P,
                  q_per_kv=g)
    # --- score
    stride = (P + 63) // 64 * 64
    scores = torch.full((H, stride), float("nan"), dtype=torch.float32, device="cuda")
    mass = torch.full((H,), float("nan"), dtype=torch.float32, device="cuda")
    m.maskkv_score(desc, Q, K, 0.0, scores, stride, mass, hp.workspace(m.maskkv_score_workspace_bytes(desc)))
    torch.cuda.synchronize()
    sc, ms = scores.cpu().numpy(), mass.cpu().numpy()
    ref_scores = []
    for h in range(H):
        I, mass_ref = orc.score_grouped(Qg[h * g:(h + 1) * g], L.K[h], P)
        ref_scores.append(I)
        rel = np.abs(sc[h, :P] - I) / np.abs(I)
        assert rel.max() <= hp.SCORE_RTOL, f"kv head {h}: score rel err {rel.max():.3e}"
        assert abs(ms[h] - mass_ref) <= hp.SCORE_RTOL * mass_ref
        assert np.isnan(sc[h, P:]).all()
    # --- select (the oracle pools its own scores; the near-tie band covers the fp32 differences)
    bud = torch.from_numpy(np.asarray(budgets, dtype=np.int32)).to("cuda")
    cap = int(sum(min(int(b), P) for b in budgets))
    idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    cu = torch.full((H + 1,), -1, dtype=torch.int32, device="cuda")
    m.maskkv_select(desc, scores, stride, window, 0, bud, idx, cu, cap,
                    hp.workspace(m.maskkv_select_workspace_bytes(desc)))
    torch.cuda.synchronize()
    keeps, cu_h = hp.split_idx(idx, cu)
    for h in range(H):
        hp.check_keep_against_oracle(orc.pool(ref_scores[h], window), int(budgets[h]), keeps[h], f"kv head {h}")
    # --- compact: bit-exact gather of the KV head's rows
    Kc = torch.zeros((cap, d), dtype=hp.torch_dtype(dtype), device="cuda")
    Vc = torch.zeros_like(Kc)
    m.maskkv_compact(desc, K, V, idx, cu, cap, Kc, Vc)
    torch.cuda.synchronize()
    Kc_h, Vc_h = Kc.float().cpu().numpy(), Vc.float().cpu().numpy()
    for h in range(H):
        k_ref, v_ref = orc.compact(L.K[h, :P], L.V[h, :P], keeps[h])
        assert np.array_equal(Kc_h[cu_h[h]:cu_h[h + 1]], k_ref) and np.array_equal(Vc_h[cu_h[h]:cu_h[h + 1]], v_ref)
    # --- attend over the shared cache, every query head on its own
    atol = hp.ATTEND_ATOL_BF16 if dtype == "bf16" else hp.ATTEND_ATOL_F32
    O = torch.full((1, H * g, n_m, d), float("nan"), dtype=hp.torch_dtype(dtype), device="cuda")
    lse = torch.full((H * g * n_m,), float("nan"), dtype=torch.float32, device="cuda")
    Kr, Vr = m.tensor_view(K, seq_start=[P]), m.tensor_view(V, seq_start=[P])
    m.maskkv_attend(desc, Q, Kc, Vc, cu, cap, Kr, Vr, 0.0, O, lse,
                    hp.workspace(m.maskkv_attend_workspace_bytes(desc, False)))
    torch.cuda.synchronize()
    O_h, lse_h = O.float().cpu().numpy()[0], lse.cpu().numpy().reshape(H * g, n_m)
    for h in range(H):
        k_ref, v_ref = orc.compact(L.K[h, :P], L.V[h, :P], keeps[h])
        want = orc.attend_grouped(Qg[h * g:(h + 1) * g], k_ref, v_ref, L.K[h, P:], L.V[h, P:])
        got = O_h[h * g:(h + 1) * g]
        assert np.isfinite(got).all()
        assert np.abs(got - want).max() <= atol, f"kv head {h}: attend err {np.abs(got - want).max():.3e}"
        for gi in range(g):
            _, lse_ref = orc.attend(Qg[h * g + gi], k_ref, v_ref, L.K[h, P:], L.V[h, P:], return_lse=True)
            assert np.abs(lse_h[h * g + gi] - lse_ref).max() <= 1e-3
    # --- the un-evicted attention with the same grouping
    O2 = torch.full_like(O, float("nan"))
    m.maskkv_attend_full(desc, Q, K, V, 0.0, O2, None, hp.workspace(m.maskkv_attend_workspace_bytes(desc, True)))
    torch.cuda.synchronize()
    O2_h = O2.float().cpu().numpy()[0]
    for hq in range(H * g):
        want = orc.attend_full(Qg[hq], L.K[hq // g], L.V[hq // g])
        assert np.abs(O2_h[hq] - want).max() <= atol, f"query head {hq}: full attention err"


def test_grouped_queries_dream_shape():
    """Seven query heads per KV head at head_dim 128 (the grouped-query model the paper evaluates), a response
    span that is not a multiple of the query tiles, ragged budgets.  Few workgroups: the narrow attention kernel."""
    run_grouped(seed=4100, H=4, g=7, d=128, P=1500, n_m=72, dtype="bf16", budgets=[64, 200, 0, 1500])


def test_grouped_queries_fp32_small_heads():
    run_grouped(seed=4200, H=2, g=3, d=64, P=333, n_m=50, dtype="f32", budgets=[17, 90], window=1)


def test_grouped_queries_wide_launch():
    """Enough query tiles for the tiled attention kernel (256 workgroups or more)."""
    run_grouped(seed=4300, H=8, g=4, d=128, P=520, n_m=1000, dtype="bf16", budgets=[100] * 4 + [37] * 4)


def test_grouped_queries_ragged_batch_token_major_layout():
    """Two sequences of different prompt length, g = 3, tensors stored [B, T, heads, d]: the query-head stride is
    then not a multiple of the token stride, and query tiles straddle query heads (n_resp = 40)."""
    m = hp.mk()
    B, H, g, d, n_m, dtype = 2, 2, 3, 128, 40, "bf16"
    Ps = [700, 413]
    P_max, N_max = max(Ps), max(Ps) + n_m
    Ls = [synth.make_layer(4500 + b, H, d, Ps[b], n_m, dtype, n_planted=9, amplitude=2.5) for b in range(B)]
    Qg = [synth.make_grouped_queries(4510 + b, Ls[b], g) for b in range(B)]
    Kh = np.zeros((B, H, N_max, d), dtype=np.float32)
    Vh = np.zeros_like(Kh)
    for b, L in enumerate(Ls):
        Kh[b, :, :L.N], Vh[b, :, :L.N] = L.K, L.V
    token_major = lambda x: hp.upload(x, dtype).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    K, V, Q = token_major(Kh), token_major(Vh), token_major(np.stack(Qg))
    assert Q.stride(1) == d and Q.stride(2) == H * g * d
    desc = m.Desc(B=B, H=H, d=d, dtype=m.MASKKV_BF16, n_resp=n_m, P_max=P_max, prompt_len=Ps, q_per_kv=g)
    stride = (P_max + 63) // 64 * 64
    scores = torch.full((B * H, stride), float("nan"), dtype=torch.float32, device="cuda")
    m.maskkv_score(desc, Q, K, 0.0, scores, stride, None, hp.workspace(m.maskkv_score_workspace_bytes(desc)))
    budgets = np.array([50, 0, 413, 77], dtype=np.int32)
    cap = int(budgets.sum())
    idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    cu = torch.full((B * H + 1,), -1, dtype=torch.int32, device="cuda")
    m.maskkv_select(desc, scores, stride, 7, 0, torch.from_numpy(budgets).cuda(), idx, cu, cap,
                    hp.workspace(m.maskkv_select_workspace_bytes(desc)))
    Kc = torch.zeros((cap, d), dtype=torch.bfloat16, device="cuda")
    Vc = torch.zeros_like(Kc)
    m.maskkv_compact(desc, K, V, idx, cu, cap, Kc, Vc)
    O = torch.full((B, n_m, H * g, d), float("nan"), dtype=torch.bfloat16, device="cuda").permute(0, 2, 1, 3)
    lse = torch.full((B * H * g * n_m,), float("nan"), dtype=torch.float32, device="cuda")
    Kr, Vr = m.tensor_view(K, seq_start=Ps), m.tensor_view(V, seq_start=Ps)
    m.maskkv_attend(desc, Q, Kc, Vc, cu, cap, Kr, Vr, 0.0, O, lse, hp.workspace(m.maskkv_attend_workspace_bytes(desc, False)))
    torch.cuda.synchronize()
    sc = scores.cpu().numpy()
    keeps, _ = hp.split_idx(idx, cu)
    O_h, lse_h = O.float().cpu().numpy(), lse.cpu().numpy().reshape(B, H * g, n_m)
    for b, L in enumerate(Ls):
        for h in range(H):
            I, _ = orc.score_grouped(Qg[b][h * g:(h + 1) * g], L.K[h], L.P)
            assert (np.abs(sc[b * H + h, :L.P] - I) / I).max() <= hp.SCORE_RTOL
            keep = keeps[b * H + h]
            hp.check_keep_against_oracle(orc.pool(I, 7), int(budgets[b * H + h]), keep, f"b={b} h={h}")
            want = orc.attend_grouped(Qg[b][h * g:(h + 1) * g], L.K[h, keep], L.V[h, keep], L.K[h, L.P:], L.V[h, L.P:])
            assert np.abs(O_h[b, h * g:(h + 1) * g] - want).max() <= hp.ATTEND_ATOL_BF16
            for gi in range(g):
                _, rl = orc.attend(Qg[b][h * g + gi], L.K[h, keep], L.V[h, keep], L.K[h, L.P:], L.V[h, L.P:],
                                   return_lse=True)
                assert np.abs(lse_h[b, h * g + gi] - rl).max() <= 1e-3


def test_group_of_one_is_multi_head_attention():
    """q_per_kv = 1 and q_per_kv = 0 give the same bits as each other."""
    m = hp.mk()
    L = synth.make_layer(4400, 3, 64, 200, 40, "bf16", n_planted=4, amplitude=2.5)
    K, Q = hp.upload(L.K[None], "bf16"), hp.upload(L.Q[None], "bf16")
    outs = []
    for g in (0, 1):
        desc = m.Desc(B=1, H=3, d=64, dtype=m.MASKKV_BF16, n_resp=40, P_max=200, q_per_kv=g)
        scores = torch.zeros((3, 256), dtype=torch.float32, device="cuda")
        m.maskkv_score(desc, Q, K, 0.0, scores, 256, None, hp.workspace(m.maskkv_score_workspace_bytes(desc)))
        torch.cuda.synchronize()
        outs.append(scores.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


# ------------------------------------------------------------------------------------------ value shift
def gpu_value_shift(v_now, v_prev, dtype, delta, row_stride=None):
    m = hp.mk()
    n, width = v_now.shape
    stride = width if row_stride is None else row_stride
    tdt = hp.torch_dtype(dtype)
    a = torch.full((n, stride), 3.0, dtype=tdt, device="cuda")      # padding columns must never be read
    b = torch.full((n, stride), -5.0, dtype=tdt, device="cuda")
    a[:, :width] = torch.from_numpy(v_now).to("cuda").to(tdt)
    b[:, :width] = torch.from_numpy(v_prev).to("cuda").to(tdt)
    cos = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    refresh = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    count = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    m.maskkv_value_shift(a[:, :width], b[:, :width], delta, cos, refresh, count)
    torch.cuda.synchronize()
    c = int(count.item())
    r = refresh.cpu().numpy()
    assert 0 <= c <= n and np.all(r[c:] == -7), "entries past the count must stay untouched"
    return cos.cpu().numpy(), r[:c]


@pytest.mark.parametrize("n,width,dtype,delta,stride", [
    (256, 4096, "bf16", 0.9, None),     # one sequence's response span at the model's value width
    (4096, 4096, "bf16", 0.95, None),   # batch 8 x 512 response tokens: several rounds of the collecting workgroup
    (1500, 512, "f32", 0.8, 520),       # ragged last round, padded rows
    (1, 1024, "bf16", 0.9, None),
    (70, 8, "f32", 0.5, None),          # shortest legal row
])
def test_value_shift_matches_oracle(n, width, dtype, delta, stride):
    v_now, v_prev = synth.make_value_steps(900 + n, n, width, dtype, 0.05, 1.0)
    cos_ref, refresh_ref = orc.value_shift(v_now, v_prev, delta)
    cos, refresh = gpu_value_shift(v_now, v_prev, dtype, delta, stride)
    assert np.abs(cos - cos_ref).max() <= COS_ATOL
    assert np.all(np.diff(refresh) > 0)
    diff = np.setxor1d(refresh, refresh_ref)
    assert np.all(np.abs(cos_ref[diff] - delta) < SHIFT_BAND), "sets differ away from the threshold"
    if n > 1:
        assert 0 < refresh_ref.size < n                      # the case exercises both outcomes
    # the decision itself is exact on the device's own cosines
    assert np.array_equal(refresh, np.nonzero(cos < np.float32(delta))[0])


def test_value_shift_special_cases():
    v, _ = synth.make_value_steps(5, 300, 256, "f32", 0.0, 0.0)
    cos, refresh = gpu_value_shift(v, v, "f32", 0.99)
    assert np.abs(cos - 1.0).max() <= COS_ATOL and refresh.size == 0          # nothing moved
    cos, refresh = gpu_value_shift(-v, v, "f32", 0.0)
    assert np.abs(cos + 1.0).max() <= COS_ATOL and np.array_equal(refresh, np.arange(300))   # everything flipped
    cos, refresh = gpu_value_shift(2.5 * v, v, "f32", 0.99)
    assert refresh.size == 0                                                  # scale invariance
