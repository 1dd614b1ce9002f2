"""GPU-vs-oracle parity of the whole hot path, called through the C ABI (needs an MI355X).

Tolerances (stated once in tests/helpers.py): scores within 1e-3 relative of the float64 oracle;
kept index sets identical except inside the 1e-4 near-tie band at the k-th largest pooled score;
compaction bit-exact; attention within 2e-2 max-abs for bf16 inputs (2e-5 for fp32 inputs).
"""
import math

import numpy as np
import pytest
import torch

from oracle import maskkv_oracle as orc
from paper_2510_09309_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def pipeline_parity(batch: hp.Batch, budgets: np.ndarray, window: int, check_full: bool = True, heads=None,
                    score_rtol: float = hp.SCORE_RTOL):
    atol = hp.ATTEND_ATOL_BF16 if batch.dtype == "bf16" else hp.ATTEND_ATOL_F32
    H = batch.H
    heads = list(range(H)) if heads is None else heads
    scores, mass = hp.gpu_score(batch)
    worst = hp.check_scores(batch, scores, mass, heads=heads, rtol=score_rtol)
    idx, cu, cap = hp.gpu_select(batch, scores, budgets, window)
    keeps, cu_h = hp.split_idx(idx, cu)
    clamped = [min(max(int(budgets[i]), 0), batch.P[i // H]) for i in range(batch.B * H)]
    assert cu_h.tolist() == np.concatenate([[0], np.cumsum(clamped)]).tolist()
    Kc, Vc = hp.gpu_compact(batch, idx, cu, cap)
    O, lse = hp.gpu_attend(batch, Kc, Vc, cu, cap)
    if check_full:
        Of, lsef = hp.gpu_attend_full(batch)
    Kc_h, Vc_h = Kc.float().cpu().numpy(), Vc.float().cpu().numpy()
    O_h, lse_h = O.float().cpu().numpy(), lse.cpu().numpy().reshape(batch.B, H, batch.n_m)
    n_band = 0
    for b, L in enumerate(batch.layers):
        for h in heads:
            bh = b * H + h
            I, _ = orc.score(L.Q[h], L.K[h], L.P)
            n_band += hp.check_keep_against_oracle(orc.pool(I, window), clamped[bh], keeps[bh], f"b{b} h{h}")
            keep = keeps[bh]
            # compaction is a bit-exact gather of the rows the GPU selected
            assert np.array_equal(Kc_h[cu_h[bh]:cu_h[bh + 1]], L.K[h, keep])
            assert np.array_equal(Vc_h[cu_h[bh]:cu_h[bh + 1]], L.V[h, keep])
            ref, ref_lse = orc.attend(L.Q[h], L.K[h, keep], L.V[h, keep], L.K[h, L.P:], L.V[h, L.P:], return_lse=True)
            err = np.abs(O_h[b, h] - ref).max()
            assert err <= atol, f"attend b{b} h{h}: max abs err {err:.3e}"
            assert np.abs(lse_h[b, h] - ref_lse).max() <= 1e-3
            if check_full:
                ref_f = orc.attend_full(L.Q[h], L.K[h], L.V[h])
                errf = np.abs(Of[b, h].float().cpu().numpy() - ref_f).max()
                assert errf <= atol, f"attend_full b{b} h{h}: max abs err {errf:.3e}"
    return worst, n_band


def test_config_c1_end_to_end():
    """Benchmark config 1 (fp32, d=64, P=512, 64 mask queries, window 7, budget 32): every output, every head."""
    cfg = synth.CONFIGS["C1"]
    batch = hp.Batch([synth.config_layer("C1")])
    worst, n_band = pipeline_parity(batch, synth.config_budgets("C1"), cfg["window"])
    assert worst < 2e-5, f"fp32 path should be far inside the tolerance, got {worst:.2e}"
    # planted positions dominate what is kept
    scores, _ = hp.gpu_score(batch)
    idx, cu, cap = hp.gpu_select(batch, scores, synth.config_budgets("C1"), cfg["window"])
    keeps, _ = hp.split_idx(idx, cu)
    L = batch.layers[0]
    for h in range(cfg["H"]):
        near = {p + t for p in L.planted[h].tolist() for t in range(-3, 4)}
        assert set(keeps[h].tolist()) <= near


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 128), ("f32", 64)])
def test_ragged_shapes_all_dtypes(dtype, d):
    """Sizes that are no multiple of any tile (keys, queries, chunks), budgets from 0 to beyond P."""
    L = synth.make_layer(77, H=3, d=d, P=777, n_m=100, dtype=dtype, n_planted=15, amplitude=2.5)
    batch = hp.Batch([L])
    budgets = np.array([0, 50, 5000], dtype=np.int32)
    pipeline_parity(batch, budgets, window=7)


def test_ragged_batch_with_empty_and_short_prompts():
    layers = [synth.make_layer(200 + i, H=2, d=128, P=P, n_m=96, dtype="bf16", n_planted=min(5, P), amplitude=2.5)
              for i, P in enumerate([1300, 0, 7, 2049])]
    batch = hp.Batch(layers)
    budgets = np.array([64, 200, 3, 3, 7, 2, 1024, 1], dtype=np.int32)
    pipeline_parity(batch, budgets, window=7)


def test_many_query_groups_and_subspan():
    """More than 256 queries (several sweeps per chunk) and a voting sub-span of the mask queries."""
    L = synth.make_layer(78, H=2, d=128, P=1500, n_m=520, dtype="bf16", n_planted=30, amplitude=2.5)
    batch = hp.Batch([L])
    pipeline_parity(batch, np.array([300, 77], dtype=np.int32), window=7)
    # position-aware voting: only the middle third of the mask queries vote
    m = hp.mk()
    lo, n = 173, 174
    desc = m.Desc(B=1, H=2, d=128, dtype=m.MASKKV_BF16, n_resp=L.n_m, P_max=L.P, n_query=n)
    scores = torch.full((2, 1536), float("nan"), dtype=torch.float32, device="cuda")
    ws = hp.workspace(m.maskkv_score_workspace_bytes(desc))
    m.maskkv_score(desc, batch.Q[:, :, lo:lo + n], batch.K, 0.0, scores, 1536, None, ws)
    torch.cuda.synchronize()
    for h in range(2):
        I, _ = orc.score(L.Q[h, lo:lo + n], L.K[h], L.P)
        got = scores[h, :L.P].cpu().numpy()
        assert np.max(np.abs(got - I) / I) < hp.SCORE_RTOL


@pytest.mark.parametrize("sigma", [3.0, 9.5])
def test_peaky_logits(sigma):
    """Wide logit spread: exercises the running-max rescaling and large top-k gaps."""
    L = synth.make_layer(79, H=4, d=128, P=3000, n_m=256, dtype="bf16", n_planted=40, amplitude=2.0 * sigma,
                         sigma=sigma, query_shift=sigma)
    batch = hp.Batch([L])
    # scores now span many orders of magnitude; tiny ones (< 1e-30 of the mass) are compared absolutely
    scores, mass = hp.gpu_score(batch)
    sc = scores.cpu().numpy()
    for h in range(L.H):
        I, m_or = orc.score(L.Q[h], L.K[h], L.P)
        got = sc[h, :L.P]
        big = I > 1e-20
        assert np.max(np.abs(got[big] - I[big]) / I[big]) < hp.SCORE_RTOL
        assert np.all(got[~big] < 1e-19)
        assert abs(mass[h].item() - m_or) < 1e-3 * m_or
    idx, cu, cap = hp.gpu_select(batch, scores, np.full(4, 128, dtype=np.int32), 1)
    keeps, _ = hp.split_idx(idx, cu)
    for h in range(L.H):
        I, _ = orc.score(L.Q[h], L.K[h], L.P)
        hp.check_keep_against_oracle(I, 128, keeps[h], f"h{h}")
    Kc, Vc = hp.gpu_compact(batch, idx, cu, cap)
    O, _ = hp.gpu_attend(batch, Kc, Vc, cu, cap)
    for h in range(L.H):
        ref = orc.attend(L.Q[h], L.K[h, keeps[h]], L.V[h, keeps[h]], L.K[h, L.P:], L.V[h, L.P:])
        assert np.abs(O[0, h].float().cpu().numpy() - ref).max() <= hp.ATTEND_ATOL_BF16 * max(1.0, sigma)


def test_explicit_scale_and_strided_layout():
    """[B, T, H, d] memory layout through the stride fields, and a caller-given softmax scale."""
    m = hp.mk()
    L = synth.make_layer(80, H=4, d=64, P=600, n_m=64, dtype="bf16", n_planted=8, amplitude=2.5)
    to_bthd = lambda x: hp.upload(x, "bf16")[None].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    K, V, Q = to_bthd(L.K), to_bthd(L.V), to_bthd(L.Q)
    assert K.stride(1) == 64 and K.stride(2) == 4 * 64
    desc = m.Desc(B=1, H=4, d=64, dtype=m.MASKKV_BF16, n_resp=64, P_max=600)
    scores = torch.zeros((4, 640), dtype=torch.float32, device="cuda")
    mass = torch.zeros(4, dtype=torch.float32, device="cuda")
    scale = 0.2
    m.maskkv_score(desc, Q, K, scale, scores, 640, mass, hp.workspace(m.maskkv_score_workspace_bytes(desc)))
    torch.cuda.synchronize()
    for h in range(4):
        I, _ = orc.score(L.Q[h], L.K[h], L.P, scale=scale)
        assert np.max(np.abs(scores[h, :600].cpu().numpy() - I) / I) < hp.SCORE_RTOL
    O = torch.zeros((1, 64, 4, 64), dtype=torch.bfloat16, device="cuda").permute(0, 2, 1, 3)
    m.maskkv_attend_full(desc, Q, K, V, scale, O, None, hp.workspace(m.maskkv_attend_workspace_bytes(desc, True)))
    torch.cuda.synchronize()
    for h in range(4):
        ref = orc.attend_full(L.Q[h], L.K[h], L.V[h], scale=scale)
        assert np.abs(O[0, h].float().cpu().numpy() - ref).max() <= hp.ATTEND_ATOL_BF16


def test_config_c2_full_parity():
    """Benchmark config 2 (32 heads x 128, bf16, P=4096, 256 mask queries, budgets 341/171): all heads."""
    cfg = synth.CONFIGS["C2"]
    batch = hp.Batch([synth.config_layer("C2")])
    budgets = synth.config_budgets("C2")
    assert budgets.sum() == 32 * 256 and sorted(set(budgets.tolist())) == [171, 341]
    worst, n_band = pipeline_parity(batch, budgets, cfg["window"])
    assert worst < 1e-4, f"bf16 inputs with fp32 accumulation should reach ~1e-6, got {worst:.2e}"


def test_select_standalone_is_bit_exact():
    """select on given fp32 scores: same decision precision on both sides -> identical index lists."""
    m = hp.mk()
    rng = np.random.default_rng(5)
    B, H = 2, 5
    P = [4099, 1000]
    desc = m.Desc(B=B, H=H, d=128, dtype=m.MASKKV_BF16, n_resp=8, P_max=max(P), prompt_len=P)
    stride = 4160
    sc = rng.random((B * H, stride)).astype(np.float32) * 0.01
    sc[3, :] = 0.25                      # all ties: lowest positions win
    sc[4, ::2] = sc[4, 1::2]             # pairwise ties
    sc[7, :] = np.float32(1e-3)
    budgets = np.array([0, 1, 4099, 5000, 777, 64, 999, 1000, 1, 333], dtype=np.int32)
    for window, mode, name in [(7, 0, "mean"), (1, 0, "mean"), (5, 1, "max"), (63, 0, "mean")]:
        scores = torch.from_numpy(sc).to("cuda")
        bud = torch.from_numpy(budgets).to("cuda")
        clamped = [min(int(budgets[i]), P[i // H]) for i in range(B * H)]
        cap = sum(clamped)
        idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
        cu = torch.zeros(B * H + 1, dtype=torch.int32, device="cuda")
        m.maskkv_select(desc, scores, stride, window, mode, bud, idx, cu, cap,
                        hp.workspace(m.maskkv_select_workspace_bytes(desc)))
        torch.cuda.synchronize()
        keeps, cu_h = hp.split_idx(idx, cu)
        assert cu_h.tolist() == np.concatenate([[0], np.cumsum(clamped)]).tolist()
        for bh in range(B * H):
            pooled = orc.pool(sc[bh, :P[bh // H]], window, name, dtype=np.float32)
            ref = orc.select(pooled, clamped[bh])
            assert np.array_equal(keeps[bh], ref), f"window {window} mode {name} bh {bh}"


def test_select_long_prompt_reads_candidates_in_place():
    """Prompts longer than the LDS key buffer: the final stage reads the chunk candidates in place; still bit-exact."""
    m = hp.mk()
    rng = np.random.default_rng(6)
    P = 50000
    desc = m.Desc(B=1, H=2, d=128, dtype=m.MASKKV_BF16, n_resp=8, P_max=P)
    assert m.maskkv_select_workspace_bytes(desc) == 2 * 13 * 4096 * 8 + 256   # candidates + their counts per chunk
    sc = (rng.random((2, P)) ** 4).astype(np.float32)
    budgets = np.array([1234, 40000], dtype=np.int32)
    idx = torch.full((int(budgets.sum()),), -1, dtype=torch.int32, device="cuda")
    cu = torch.zeros(3, dtype=torch.int32, device="cuda")
    m.maskkv_select(desc, torch.from_numpy(sc).to("cuda"), P, 7, 0, torch.from_numpy(budgets).to("cuda"), idx, cu,
                    int(budgets.sum()), hp.workspace(m.maskkv_select_workspace_bytes(desc)))
    torch.cuda.synchronize()
    keeps, _ = hp.split_idx(idx, cu)
    for h in range(2):
        ref = orc.select(orc.pool(sc[h], 7, dtype=np.float32), int(budgets[h]))
        assert np.array_equal(keeps[h], ref)


def test_select_capacity_is_never_overrun():
    m = hp.mk()
    desc = m.Desc(B=1, H=4, d=128, dtype=m.MASKKV_BF16, n_resp=8, P_max=500)
    sc = torch.rand((4, 512), device="cuda")
    bud = torch.full((4,), 100, dtype=torch.int32, device="cuda")
    cap = 250
    idx = torch.full((cap + 64,), -7, dtype=torch.int32, device="cuda")
    cu = torch.zeros(5, dtype=torch.int32, device="cuda")
    m.maskkv_select(desc, sc, 512, 1, 0, bud, idx, cu, cap, hp.workspace(m.maskkv_select_workspace_bytes(desc)))
    torch.cuda.synchronize()
    assert cu.cpu().tolist() == [0, 100, 200, 300, 400]
    assert (idx[cap:] == -7).all() and (idx[:cap] >= 0).all()


def test_head_budgets_on_device():
    """Stage 2 head-level budgets from the scoring kernel's prompt mass, no host round trip."""
    m = hp.mk()
    L = synth.make_layer(81, H=8, d=128, P=2000, n_m=128, dtype="bf16", n_planted=40, amplitude=2.5)
    # make the heads differ in prompt preference: scale some heads' prompt keys
    for h in range(8):
        L.K[h, :L.P] = synth.round_to_bf16(L.K[h, :L.P] * np.float32(0.5 + 0.25 * h))
    batch = hp.Batch([L])
    scores, mass = hp.gpu_score(batch)
    bud = torch.zeros(8, dtype=torch.int32, device="cuda")
    m.maskkv_head_budgets(batch.desc, mass, 256, 0.1, bud)
    torch.cuda.synchronize()
    masses = np.array([orc.score(L.Q[h], L.K[h], L.P)[1] for h in range(8)])
    pref = orc.prompt_preference(masses, L.n_m)
    exact = 0.1 * 256 + 0.9 * 8 * 256 * pref / pref.sum()
    ref = orc.head_budgets(pref, 256, 0.1)
    got = bud.cpu().numpy()
    # identical except where the real-valued budget sits within 1e-3 of an integer (fp32 vs fp64 floor)
    near_int = np.abs(exact - np.rint(exact)) < 1e-3
    assert np.all((got == ref) | near_int)
    assert np.all(np.abs(got - exact) < 1.0 + 1e-3)
    assert got.sum() <= 8 * 256
    # and the budgets feed select directly
    idx = torch.zeros(8 * 256, dtype=torch.int32, device="cuda")
    cu = torch.zeros(9, dtype=torch.int32, device="cuda")
    m.maskkv_select(batch.desc, scores, scores.stride(0), 7, 0, bud, idx, cu, 8 * 256,
                    hp.workspace(m.maskkv_select_workspace_bytes(batch.desc)))
    torch.cuda.synchronize()
    assert cu.cpu().numpy().tolist() == np.concatenate([[0], np.cumsum(got)]).tolist()


def test_head_budgets_batch_with_an_empty_prompt_and_many_heads():
    """Per-sequence normalisation over more heads than one pass of the workgroup covers; a sequence without a prompt
    (all masses zero) gets the uniform budget."""
    m = hp.mk()
    B, H, k_l, alpha = 3, 300, 100, 0.25
    rng = np.random.default_rng(12)
    mass_h = rng.random((B, H)).astype(np.float32) * 50
    mass_h[1] = 0.0
    desc = m.Desc(B=B, H=H, d=64, dtype=m.MASKKV_BF16, n_resp=64, P_max=128, prompt_len=[128, 0, 77])
    bud = torch.full((B * H,), -1, dtype=torch.int32, device="cuda")
    m.maskkv_head_budgets(desc, torch.from_numpy(mass_h.reshape(-1)).cuda(), k_l, alpha, bud)
    torch.cuda.synchronize()
    got = bud.cpu().numpy().reshape(B, H)
    assert got[1].tolist() == orc.head_budgets(orc.prompt_preference(np.zeros(H), 64), k_l, alpha).tolist() == [k_l] * H
    for b in (0, 2):
        pref = orc.prompt_preference(mass_h[b].astype(np.float64), 64)
        exact = alpha * k_l + (1 - alpha) * H * k_l * pref / pref.sum()
        near_int = np.abs(exact - np.rint(exact)) < 1e-2
        assert np.all((got[b] == orc.head_budgets(pref, k_l, alpha)) | near_int)
        assert got[b].sum() <= H * k_l


def test_full_budget_compressed_equals_full_attention_on_gpu():
    """Nothing evicted: attend over the compacted cache must agree with attend_full (same kernel family)."""
    L = synth.make_layer(82, H=2, d=128, P=900, n_m=130, dtype="bf16", n_planted=10, amplitude=2.5)
    batch = hp.Batch([L])
    scores, _ = hp.gpu_score(batch)
    idx, cu, cap = hp.gpu_select(batch, scores, np.array([900, 2000], dtype=np.int32), 7)
    assert idx.cpu().numpy().tolist() == list(range(900)) * 2
    Kc, Vc = hp.gpu_compact(batch, idx, cu, cap)
    O1, lse1 = hp.gpu_attend(batch, Kc, Vc, cu, cap)
    O2, lse2 = hp.gpu_attend_full(batch)
    assert (O1.float() - O2.float()).abs().max().item() <= 2 ** -7  # bf16 rounding of nearly equal fp32 results
    assert (lse1 - lse2).abs().max().item() < 1e-4


def test_attend_wide_launch_takes_the_tiled_kernel():
    """B*H*ceil(n_resp/128) >= 256 workgroups: the compressed call runs the tiled kernel (narrower launches
    run the kernel whose waves split the key axis); both are checked against the oracle elsewhere and here."""
    B, H = 4, 64
    layers = [synth.make_layer(900 + b, H=H, d=64, P=200 + 37 * b, n_m=129, dtype="bf16", n_planted=6, amplitude=2.5)
              for b in range(B)]
    batch = hp.Batch(layers)
    assert B * H * 2 >= 256
    budgets = synth.budgets_log_uniform(B * H, 8, 150, seed=77)
    scores, _ = hp.gpu_score(batch)
    idx, cu, cap = hp.gpu_select(batch, scores, budgets, 7)
    keeps, _ = hp.split_idx(idx, cu)
    Kc, Vc = hp.gpu_compact(batch, idx, cu, cap)
    O, lse = hp.gpu_attend(batch, Kc, Vc, cu, cap)
    O_h, lse_h = O.float().cpu().numpy(), lse.cpu().numpy().reshape(B, H, 129)
    for b, L in enumerate(layers):
        for h in (0, 17, 63):
            keep = keeps[b * H + h]
            ref, rl = orc.attend(L.Q[h], L.K[h, keep], L.V[h, keep], L.K[h, L.P:], L.V[h, L.P:], return_lse=True)
            assert np.abs(O_h[b, h] - ref).max() <= hp.ATTEND_ATOL_BF16
            assert np.abs(lse_h[b, h] - rl).max() <= 1e-3


@pytest.mark.parametrize("d,n_m,sigma", [(128, 512, 1.0), (64, 250, 1.0), (128, 256, 9.5)])
def test_attend_many_heads_long_response_span(d, n_m, sigma):
    """128 heads with response spans of several query tiles: ragged budgets from an empty cache to the whole
    prompt, a key axis that ends inside a 32-key block, peaky logits, compressed and un-evicted calls."""
    B, H = 2, 64
    layers = [synth.make_layer(1300 + b, H=H, d=d, P=333 + 120 * b, n_m=n_m, dtype="bf16", n_planted=6, amplitude=2.5,
                               sigma=sigma) for b in range(B)]
    batch = hp.Batch(layers)
    assert B * H * ((n_m + 255) // 256) >= 128
    budgets = synth.budgets_log_uniform(B * H, 8, 300, seed=78)
    budgets[0], budgets[1], budgets[H] = 0, 10 ** 6, 453
    scores, _ = hp.gpu_score(batch)
    idx, cu, cap = hp.gpu_select(batch, scores, budgets, 7)
    keeps, _ = hp.split_idx(idx, cu)
    Kc, Vc = hp.gpu_compact(batch, idx, cu, cap)
    O, lse = hp.gpu_attend(batch, Kc, Vc, cu, cap)
    O2, lse2 = hp.gpu_attend_full(batch)
    O_h, lse_h = O.float().cpu().numpy(), lse.cpu().numpy().reshape(B, H, n_m)
    O2_h, lse2_h = O2.float().cpu().numpy(), lse2.cpu().numpy().reshape(B, H, n_m)
    assert np.isfinite(O_h).all() and np.isfinite(O2_h).all()
    for b, L in enumerate(layers):
        for h in (0, 1, 17, 63):
            keep = keeps[b * H + h]
            ref, rl = orc.attend(L.Q[h], L.K[h, keep], L.V[h, keep], L.K[h, L.P:], L.V[h, L.P:], return_lse=True)
            assert np.abs(O_h[b, h] - ref).max() <= hp.ATTEND_ATOL_BF16, (b, h)
            assert np.abs(lse_h[b, h] - rl).max() <= 1e-3
            ref2, rl2 = orc.attend_full(L.Q[h], L.K[h], L.V[h], return_lse=True)
            assert np.abs(O2_h[b, h] - ref2).max() <= hp.ATTEND_ATOL_BF16, (b, h)
            assert np.abs(lse2_h[b, h] - rl2).max() <= 1e-3


def test_repeated_calls_are_deterministic():
    L = synth.make_layer(83, H=4, d=128, P=5000, n_m=256, dtype="bf16", n_planted=50, amplitude=2.5)
    batch = hp.Batch([L])
    s1, m1 = hp.gpu_score(batch)
    s2, m2 = hp.gpu_score(batch)
    assert torch.equal(s1[:, :5000], s2[:, :5000]) and torch.equal(m1, m2)
