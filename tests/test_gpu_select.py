"""The chunked selection on long prompts, ties across chunks, capacity clipping and the host copy of the budgets,
through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

from oracle import maskkv_oracle as orc
from paper_2510_09309_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,d,Ps", [("bf16", 128, [9000, 300, 0, 4097]), ("f32", 64, [5000, 4096]),
                                        ("bf16", 64, [700]), ("f32", 128, [12289])])
def test_select_then_compact_on_chunked_and_single_chunk_prompts(dtype, d, Ps):
    H = 3
    layers = [synth.make_layer(600 + i, H=H, d=d, P=P, n_m=40, dtype=dtype, n_planted=min(20, P), amplitude=2.5)
              for i, P in enumerate(Ps)]
    batch = hp.Batch(layers)
    rng = np.random.default_rng(5)
    budgets = rng.choice([0, 1, 17, 200, 1000, 10 ** 6], size=len(Ps) * H).astype(np.int32)
    scores, _ = hp.gpu_score(batch)
    idx, cu, cap = hp.gpu_select(batch, scores, budgets, 7)
    Kc, Vc = hp.gpu_compact(batch, idx, cu, cap)
    keeps, cu_h = hp.split_idx(idx, cu)
    Kc_h, Vc_h = Kc.float().cpu().numpy(), Vc.float().cpu().numpy()
    for b, L in enumerate(batch.layers):
        for h in range(H):
            bh = b * H + h
            I, _ = orc.score(L.Q[h], L.K[h], L.P)
            hp.check_keep_against_oracle(orc.pool(I, 7), int(budgets[bh]), keeps[bh], f"b{b} h{h}")
            Kr, Vr = orc.compact(L.K[h, :L.P], L.V[h, :L.P], keeps[bh])
            assert np.array_equal(Kc_h[cu_h[bh]:cu_h[bh + 1]], Kr) and np.array_equal(Vc_h[cu_h[bh]:cu_h[bh + 1]], Vr)


def test_rows_beyond_the_capacity_are_not_written():
    """Budgets that only exist on the device may exceed the capacity: rows beyond it are not written, the prefix
    sums stay unclipped, and what is written is what an ample capacity would have received."""
    L = synth.make_layer(77, H=4, d=128, P=5000, n_m=16, dtype="bf16", n_planted=10, amplitude=2.5)
    batch = hp.Batch([L])
    budgets = np.array([100, 200, 300, 400], dtype=np.int32)
    scores, _ = hp.gpu_score(batch)
    cap = 450
    idx, cu, _ = hp.gpu_select(batch, scores, budgets, 7, capacity=cap)
    Kc, Vc = hp.gpu_compact(batch, idx, cu, cap)
    assert cu.cpu().tolist() == [0, 100, 300, 600, 1000]
    idx_h = idx.cpu().numpy()
    assert (idx_h[:cap] >= 0).all()
    full_idx, _, _ = hp.gpu_select(batch, scores, budgets, 7)
    assert np.array_equal(idx_h[:cap], full_idx.cpu().numpy()[:cap])
    Kc_h = Kc.float().cpu().numpy()
    for r in (0, 99, 100, 299, 300, 449):
        h = int(np.searchsorted([100, 300, 600, 1000], r, side="right"))
        assert np.array_equal(Kc_h[r], L.K[h, idx_h[r]])


def test_host_copy_of_the_budgets_is_checked_on_real_buffers():
    m = hp.mk()
    L = synth.make_layer(78, H=2, d=128, P=600, n_m=16, dtype="bf16")
    batch = hp.Batch([L])
    scores, _ = hp.gpu_score(batch)
    bud = torch.tensor([500, 700], dtype=torch.int32, device="cuda")
    idx = torch.empty(2000, dtype=torch.int32, device="cuda")
    cu = torch.empty(3, dtype=torch.int32, device="cuda")
    with pytest.raises(m.MaskKVError) as e:
        m.maskkv_select(batch.desc, scores, scores.stride(0), 7, 0, bud, idx, cu, 1000, None, budgets_host=[500, 700])
    assert e.value.status == 6      # 500 + min(700, 600) = 1100 > 1000
    m.maskkv_select(batch.desc, scores, scores.stride(0), 7, 0, bud, idx, cu, 1100, None, budgets_host=[500, 700])
    torch.cuda.synchronize()
    assert cu.cpu().tolist() == [0, 500, 1100]


@pytest.mark.parametrize("kind", ["all_equal", "two_values", "one_spike_per_chunk"])
def test_chunk_candidates_cover_ties_across_chunks(kind):
    """Many chunks whose keys tie with the head's k-th largest: every tie must reach the final stage, which then
    keeps the lowest positions (bit-exact against the fp32 oracle on given scores)."""
    m = hp.mk()
    rng = np.random.default_rng(3)
    P, H = 20000, 3
    if kind == "all_equal":
        sc = np.full((H, P), 0.25, dtype=np.float32)
    elif kind == "two_values":
        sc = rng.choice(np.array([0.25, 0.5], dtype=np.float32), size=(H, P))
    else:
        sc = np.full((H, P), 0.125, dtype=np.float32)
        sc[:, ::4096] = 7.0
    desc = m.Desc(B=1, H=H, d=128, dtype=m.MASKKV_BF16, n_resp=8, P_max=P)
    budgets = np.array([3, 5000, 19999], dtype=np.int32)
    for window in (1, 7):
        cap = int(budgets.sum())
        idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
        cu = torch.zeros(H + 1, dtype=torch.int32, device="cuda")
        m.maskkv_select(desc, torch.from_numpy(sc).to("cuda"), P, window, 0, torch.from_numpy(budgets).to("cuda"),
                        idx, cu, cap, hp.workspace(m.maskkv_select_workspace_bytes(desc)))
        torch.cuda.synchronize()
        keeps, _ = hp.split_idx(idx, cu)
        for h in range(H):
            ref = orc.select(orc.pool(sc[h], window, "mean", dtype=np.float32), int(budgets[h]))
            assert np.array_equal(keeps[h], ref), f"{kind} window {window} head {h}"
