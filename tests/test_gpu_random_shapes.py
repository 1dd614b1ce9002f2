"""Seeded random problem shapes through the whole path against the oracle (needs an MI355X): ragged batches with
empty and tiny prompts, odd response lengths, every dtype / head_dim, budgets from 0 to beyond the prompt, several
smoothing windows, grouped-query heads."""
import numpy as np
import pytest

from paper_2510_09309_amd import synth
from tests import helpers as hp
from tests.test_gpu_parity import pipeline_parity
from tests.test_gpu_variants import run_grouped

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(10_000 + seed)
    dtype = ["bf16", "f32"][int(rng.integers(2))]
    d = [64, 128][int(rng.integers(2))]
    B = int(rng.integers(1, 5))
    H = int(rng.integers(1, 7))
    n_m = int(rng.choice([1, 7, 31, 32, 33, 64, 100, 129, 200, 257]))
    P = [int(rng.choice([0, 1, 5, 63, 64, 65, 300, 1000, 2049, 4097, 5000])) for _ in range(B)]
    if max(P) == 0:
        P[0] = 77
    window = int(rng.choice([1, 3, 7, 15]))
    sigma = float(rng.choice([1.0, 3.0, 9.5]))
    budgets = np.array([int(rng.choice([0, 1, 2, 31, 64, 200, 1000, 10 ** 6])) for _ in range(B * H)], dtype=np.int32)
    return dict(dtype=dtype, d=d, B=B, H=H, n_m=n_m, P=P, window=window, sigma=sigma, budgets=budgets)


@pytest.mark.parametrize("seed", range(16))
def test_random_ragged_batches(seed):
    c = draw_case(seed)
    layers = [synth.make_layer(20_000 + 10 * seed + b, H=c["H"], d=c["d"], P=c["P"][b], n_m=c["n_m"], dtype=c["dtype"],
                               n_planted=min(5, c["P"][b]), amplitude=2.5, sigma=c["sigma"]) for b in range(c["B"])]
    batch = hp.Batch(layers)
    worst, _ = pipeline_parity(batch, c["budgets"], c["window"])
    assert worst <= hp.SCORE_RTOL, (seed, c, worst)


@pytest.mark.parametrize("seed", range(6))
def test_random_grouped_query_shapes(seed):
    rng = np.random.default_rng(30_000 + seed)
    dtype = ["bf16", "f32"][int(rng.integers(2))]
    H = int(rng.integers(1, 5))
    g = int(rng.integers(2, 6))
    P = int(rng.choice([65, 300, 1000, 2049]))
    n_m = int(rng.choice([5, 32, 50, 96, 130]))
    budgets = [int(rng.choice([0, 3, 64, 200, 10 ** 6])) for _ in range(H)]
    run_grouped(seed=31_000 + seed, H=H, g=g, d=[64, 128][int(rng.integers(2))], P=P, n_m=n_m, dtype=dtype,
                budgets=budgets, window=int(rng.choice([1, 7])))


def score_family(kind, rng, P):
    if kind == "few_values":
        return rng.choice(np.array([0.0, 1e-7, 0.5, 0.5000001], dtype=np.float32), size=P)
    if kind == "ascending":
        return np.sort(rng.random(P).astype(np.float32))
    if kind == "descending":
        return np.sort(rng.random(P).astype(np.float32))[::-1].copy()
    if kind == "negative_and_zero":
        x = rng.standard_normal(P).astype(np.float32)
        x[rng.random(P) < 0.3] = 0.0
        x[rng.random(P) < 0.05] = -0.0
        return x
    if kind == "denormal":
        return (rng.random(P) * 1e-41).astype(np.float32)
    if kind == "huge_range":
        return (10.0 ** rng.uniform(-30, 30, size=P)).astype(np.float32) * rng.choice([-1.0, 1.0], size=P).astype(np.float32)
    if kind == "flat_with_spikes":
        x = np.full(P, 7.6e-3, dtype=np.float32) * (1 + 1e-6 * rng.standard_normal(P)).astype(np.float32)
        x[rng.choice(P, size=max(P // 100, 1), replace=False)] *= np.float32(40.0)
        return x
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["few_values", "ascending", "descending", "negative_and_zero", "denormal",
                                  "huge_range", "flat_with_spikes"])
def test_select_on_adversarial_score_distributions(kind):
    """select alone on given fp32 scores: every decision is made in fp32 on both sides, so the index lists are
    identical - for ties, signed zeros, denormals, 60 decades of range, sorted inputs, and budgets on both sides of
    the 4096-candidate list."""
    import torch
    from oracle import maskkv_oracle as orc
    m = hp.mk()
    rng = np.random.default_rng(sum(kind.encode()))
    Ps = [4095, 4097, 8191, 12289, 33001]
    budgets_per = [1, 300, 4096, 4097]
    for window in (1, 7):
        for P in Ps:
            H = len(budgets_per)
            desc = m.Desc(B=1, H=H, d=128, dtype=m.MASKKV_BF16, n_resp=8, P_max=P)
            sc = np.stack([score_family(kind, rng, P) for _ in range(H)])
            budgets = np.array([min(b, P) for b in budgets_per], dtype=np.int32)
            budgets[-1] = min(P - 1, budgets[-1] + (P // 2 if P > 20000 else 0))      # a budget of half a long prompt
            cap = int(budgets.sum())
            idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
            cu = torch.zeros(H + 1, dtype=torch.int32, device="cuda")
            m.maskkv_select(desc, torch.from_numpy(sc).to("cuda"), P, window, 0, torch.from_numpy(budgets).to("cuda"),
                            idx, cu, cap, hp.workspace(m.maskkv_select_workspace_bytes(desc)))
            torch.cuda.synchronize()
            keeps, _ = hp.split_idx(idx, cu)
            for h in range(H):
                ref = orc.select(orc.pool(sc[h], window, "mean", dtype=np.float32), int(budgets[h]))
                assert np.array_equal(keeps[h], ref), f"{kind} window {window} P {P} k {budgets[h]}"


@pytest.mark.parametrize("sigma,dtype", [(40.0, "bf16"), (80.0, "bf16"), (80.0, "f32")])
def test_very_large_logits_stay_finite_and_accurate(sigma, dtype):
    """Logits of magnitude 50-230 (exp would overflow fp32 without the running reference): scores stay finite and
    within the score tolerance wherever fp32 can represent them (the float64 oracle goes down to 1e-200, fp32 output
    underflows to zero there); the un-evicted attention stays within bf16 rounding of its value range."""
    from oracle import maskkv_oracle as orc
    L = synth.make_layer(77, H=2, d=128, P=1500, n_m=70, dtype=dtype, n_planted=10, amplitude=2.5, sigma=sigma)
    batch = hp.Batch([L])
    scores, mass = hp.gpu_score(batch)
    sc = scores.cpu().numpy()
    O, _ = hp.gpu_attend_full(batch)
    for h in range(L.H):
        I, m_ref = orc.score(L.Q[h], L.K[h], L.P)
        got = sc[h, :L.P].astype(np.float64)
        assert np.isfinite(got).all() and (got >= 0).all()
        big = I > 1e-30
        assert big.sum() > 1000
        assert (np.abs(got[big] - I[big]) / I[big]).max() <= hp.SCORE_RTOL
        assert (got[~big] <= 2e-30).all()
        assert abs(mass[h].item() - m_ref) <= hp.SCORE_RTOL * m_ref
        ref = orc.attend_full(L.Q[h], L.K[h], L.V[h])
        atol = (hp.ATTEND_ATOL_BF16 if dtype == "bf16" else 1e-4) * max(1.0, float(np.abs(L.V[h]).max()))
        assert np.abs(O[0, h].float().cpu().numpy() - ref).max() <= atol


def test_packed_variable_length_layout():
    """Sequences packed back to back on the token axis ([T_total, heads, d], batch stride 0, per-sequence token
    offsets): the layout of variable-length attention libraries.  Every call of the path reads and writes it."""
    import torch
    from oracle import maskkv_oracle as orc
    m = hp.mk()
    H, d, n_m = 3, 128, 48
    Ps = [700, 0, 1300]
    B = len(Ps)
    layers = [synth.make_layer(5000 + b, H=H, d=d, P=Ps[b], n_m=n_m, dtype="bf16", n_planted=min(8, Ps[b]),
                               amplitude=2.5) for b in range(B)]
    starts = np.concatenate([[0], np.cumsum([P + n_m for P in Ps])]).astype(int)
    T = int(starts[-1])
    Kp = np.zeros((T, H, d), dtype=np.float32)
    Vp = np.zeros_like(Kp)
    Qp = np.zeros((B * n_m, H, d), dtype=np.float32)
    for b, L in enumerate(layers):
        Kp[starts[b]:starts[b + 1]] = L.K.transpose(1, 0, 2)
        Vp[starts[b]:starts[b + 1]] = L.V.transpose(1, 0, 2)
        Qp[b * n_m:(b + 1) * n_m] = L.Q.transpose(1, 0, 2)
    packed = lambda x: hp.upload(x, "bf16").permute(1, 0, 2)[None].expand(B, -1, -1, -1)   # [B, H, T, d], stride_b = 0
    K, V, Q = packed(Kp), packed(Vp), packed(Qp)
    assert K.stride(0) == 0 and K.stride(1) == d and K.stride(2) == H * d
    kv_start = [int(s) for s in starts[:-1]]
    q_start = [b * n_m for b in range(B)]
    Kv, Vv, Qv = m.tensor_view(K, kv_start), m.tensor_view(V, kv_start), m.tensor_view(Q, q_start)
    desc = m.Desc(B=B, H=H, d=d, dtype=m.MASKKV_BF16, n_resp=n_m, P_max=max(Ps), prompt_len=Ps)
    stride = (max(Ps) + 63) // 64 * 64
    scores = torch.full((B * H, stride), float("nan"), dtype=torch.float32, device="cuda")
    mass = torch.zeros(B * H, dtype=torch.float32, device="cuda")
    m.maskkv_score(desc, Qv, Kv, 0.0, scores, stride, mass, hp.workspace(m.maskkv_score_workspace_bytes(desc)))
    budgets = np.array([100, 7, 700, 5, 5, 5, 64, 1300, 0], dtype=np.int32)
    clamped = [min(int(budgets[i]), Ps[i // H]) for i in range(B * H)]
    cap = sum(clamped)
    idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    cu = torch.zeros(B * H + 1, dtype=torch.int32, device="cuda")
    m.maskkv_select(desc, scores, stride, 7, 0, torch.from_numpy(budgets).cuda(), idx, cu, cap,
                    hp.workspace(m.maskkv_select_workspace_bytes(desc)))
    Kc = torch.zeros((cap, d), dtype=torch.bfloat16, device="cuda")
    Vc = torch.zeros_like(Kc)
    m.maskkv_compact(desc, Kv, Vv, idx, cu, cap, Kc, Vc)
    Op = torch.full((B * n_m, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    Ov = m.tensor_view(Op.permute(1, 0, 2)[None].expand(B, -1, -1, -1), q_start)
    resp_start = [int(starts[b] + Ps[b]) for b in range(B)]
    m.maskkv_attend(desc, Qv, Kc, Vc, cu, cap, m.tensor_view(K, resp_start), m.tensor_view(V, resp_start), 0.0, Ov,
                    None, hp.workspace(m.maskkv_attend_workspace_bytes(desc, False)))
    torch.cuda.synchronize()
    keeps, cu_h = hp.split_idx(idx, cu)
    sc = scores.cpu().numpy()
    O_h = Op.float().cpu().numpy()
    assert np.isfinite(O_h).all()
    for b, L in enumerate(layers):
        for h in range(H):
            bh = b * H + h
            keep = keeps[bh]
            if L.P:
                I, _ = orc.score(L.Q[h], L.K[h], L.P)
                assert (np.abs(sc[bh, :L.P] - I) / I).max() <= hp.SCORE_RTOL
                hp.check_keep_against_oracle(orc.pool(I, 7), clamped[bh], keep, f"b{b} h{h}")
            assert np.array_equal(Kc.float().cpu().numpy()[cu_h[bh]:cu_h[bh + 1]], L.K[h, keep])
            ref = orc.attend(L.Q[h], L.K[h, keep], L.V[h, keep], L.K[h, L.P:], L.V[h, L.P:])
            assert np.abs(O_h[b * n_m:(b + 1) * n_m, h] - ref).max() <= hp.ATTEND_ATOL_BF16


def test_maximum_batch_of_64_ragged_sequences():
    """MASKKV_MAX_BATCH sequences in one call, prompts from empty to a few hundred tokens."""
    rng = np.random.default_rng(64)
    B, H = 64, 2
    Ps = [int(p) for p in rng.integers(0, 400, size=B)]
    Ps[0], Ps[63] = 399, 0
    layers = [synth.make_layer(7000 + b, H=H, d=64, P=Ps[b], n_m=33, dtype="bf16", n_planted=min(3, Ps[b]),
                               amplitude=2.5) for b in range(B)]
    batch = hp.Batch(layers)
    budgets = rng.integers(0, 120, size=B * H).astype(np.int32)
    worst, _ = pipeline_parity(batch, budgets, 7, heads=[0, 1])
    assert worst <= hp.SCORE_RTOL


def test_largest_supported_token_stride():
    """Rows 16 MiB apart (the documented limit): one head, 40 prompt + 24 response tokens spread over 1 GiB."""
    import torch
    from oracle import maskkv_oracle as orc
    m = hp.mk()
    d, P, n_m = 128, 40, 24
    N = P + n_m
    stride_t = (16 << 20) // 2                      # elements of bf16
    L = synth.make_layer(7100, H=1, d=d, P=P, n_m=n_m, dtype="bf16", n_planted=4, amplitude=2.5)
    big = [torch.zeros((N - 1) * stride_t + d, dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    views = []
    for buf, src in zip(big, (L.K[0], L.V[0])):
        v = torch.as_strided(buf, (1, 1, N, d), (0, 0, stride_t, 1))
        v.copy_(hp.upload(src, "bf16")[None, None])
        views.append(v)
    K, V = views
    Q = hp.upload(L.Q[None], "bf16")
    desc = m.Desc(B=1, H=1, d=d, dtype=m.MASKKV_BF16, n_resp=n_m, P_max=P)
    scores = torch.zeros((1, 64), dtype=torch.float32, device="cuda")
    m.maskkv_score(desc, Q, K, 0.0, scores, 64, None, hp.workspace(m.maskkv_score_workspace_bytes(desc)))
    idx = torch.zeros(10, dtype=torch.int32, device="cuda")
    cu = torch.zeros(2, dtype=torch.int32, device="cuda")
    m.maskkv_select(desc, scores, 64, 1, 0, torch.tensor([10], dtype=torch.int32, device="cuda"), idx, cu, 10,
                    hp.workspace(m.maskkv_select_workspace_bytes(desc)))
    Kc = torch.zeros((10, d), dtype=torch.bfloat16, device="cuda")
    Vc = torch.zeros_like(Kc)
    m.maskkv_compact(desc, K, V, idx, cu, 10, Kc, Vc)
    O = torch.zeros((1, 1, n_m, d), dtype=torch.bfloat16, device="cuda")
    m.maskkv_attend(desc, Q, Kc, Vc, cu, 10, m.tensor_view(K, [P]), m.tensor_view(V, [P]), 0.0, O, None, None)
    O2 = torch.zeros_like(O)
    m.maskkv_attend_full(desc, Q, K, V, 0.0, O2, None, hp.workspace(m.maskkv_attend_workspace_bytes(desc, True)))
    torch.cuda.synchronize()
    I, _ = orc.score(L.Q[0], L.K[0], P)
    assert (np.abs(scores[0, :P].cpu().numpy() - I) / I).max() <= hp.SCORE_RTOL
    keep = idx.cpu().numpy()
    hp.check_keep_against_oracle(I, 10, keep, "16 MiB stride")
    assert np.array_equal(Kc.float().cpu().numpy(), L.K[0, keep])
    ref = orc.attend(L.Q[0], L.K[0, keep], L.V[0, keep], L.K[0, P:], L.V[0, P:])
    assert np.abs(O[0, 0].float().cpu().numpy() - ref).max() <= hp.ATTEND_ATOL_BF16
    assert np.abs(O2[0, 0].float().cpu().numpy() - orc.attend_full(L.Q[0], L.K[0], L.V[0])).max() <= hp.ATTEND_ATOL_BF16


def test_very_long_prompt():
    """A 200k-token prompt: thousands of key tiles per head, 49 select chunks read in place, one budget far beyond
    the candidate list."""
    L = synth.make_layer(7200, H=2, d=128, P=200_003, n_m=40, dtype="bf16", n_planted=500, amplitude=2.5)
    batch = hp.Batch([L])
    worst, _ = pipeline_parity(batch, np.array([5000, 100_000], dtype=np.int32), 7)
    assert worst <= hp.SCORE_RTOL
