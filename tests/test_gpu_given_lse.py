"""Mask-Voting from given row normalisers (maskkv_score_given_lse: the second scoring pass alone) against the
float64 oracle and against the two-pass call (needs an MI355X).  The normalisers come from where a caller would
take them - the library's own un-evicted attention call on the same queries - or from the oracle."""
import numpy as np
import pytest
import torch

from oracle import maskkv_oracle as orc
from paper_2510_09309_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,d,Ps,n_m,sigma", [
    ("bf16", 128, [3000, 0, 700, 4097], 96, 1.0),     # ragged batch with an empty prompt
    ("bf16", 64, [1500], 250, 1.0),
    ("f32", 64, [900, 333], 40, 1.0),
    ("bf16", 128, [2000], 128, 9.5),                  # peaky rows: normalisers span many orders of magnitude
])
def test_scores_from_the_normalisers_of_the_full_attention_call(dtype, d, Ps, n_m, sigma):
    H = 3
    layers = [synth.make_layer(5200 + i, H=H, d=d, P=P, n_m=n_m, dtype=dtype, n_planted=min(20, P), amplitude=2.5,
                               sigma=sigma) for i, P in enumerate(Ps)]
    batch = hp.Batch(layers)
    _, lse = hp.gpu_attend_full(batch)                     # natural-log normaliser of every response row
    scores, mass = hp.gpu_score_given_lse(batch, lse)
    hp.check_scores(batch, scores, mass)                   # against the oracle, every head, NaN padding untouched
    two_pass, mass2 = hp.gpu_score(batch)
    for b, L in enumerate(layers):
        for h in range(H):
            a = scores[b * H + h, :L.P].double().cpu().numpy()
            c = two_pass[b * H + h, :L.P].double().cpu().numpy()
            assert np.all(np.abs(a - c) <= 1e-4 * np.abs(c) + 1e-30), f"b{b} h{h}: given-normaliser vs two-pass scores"
    assert torch.allclose(mass, mass2, rtol=1e-4, atol=0)


def test_oracle_normalisers_and_several_query_groups():
    """600 voting rows per head are three groups of 256 rows whose column sums a last kernel adds; the normalisers
    are the oracle's (float64 rounded to fp32), so the call is checked on its own."""
    H, d, P, n_m = 2, 128, 2500, 600
    L = synth.make_layer(5300, H=H, d=d, P=P, n_m=n_m, dtype="bf16", n_planted=30, amplitude=2.5)
    batch = hp.Batch([L])
    lse = np.stack([orc.attend_full(L.Q[h], L.K[h], L.V[h], return_lse=True)[1] for h in range(H)])
    scores, mass = hp.gpu_score_given_lse(batch, torch.from_numpy(lse.astype(np.float32).reshape(-1)).cuda())
    worst = hp.check_scores(batch, scores, mass)
    assert worst < 1e-5


def test_grouped_query_heads_use_the_layout_of_the_attention_calls_lse():
    """Two query heads per key/value head: row r of a key/value head is (query head r // n_m, token r % n_m), the
    order in which maskkv_attend_full writes its normalisers."""
    m = hp.mk()
    H, g, d, P, n_m = 2, 2, 128, 1800, 64
    L = synth.make_layer(5400, H, d, P, n_m, "bf16", n_planted=20, amplitude=2.5)
    Qg = synth.make_grouped_queries(5401, L, g)                              # [H*g, n_m, d]
    K, V, Q = hp.upload(L.K[None], "bf16"), hp.upload(L.V[None], "bf16"), hp.upload(Qg[None], "bf16")
    desc = m.Desc(B=1, H=H, d=d, dtype=m.MASKKV_BF16, n_resp=n_m, P_max=P, q_per_kv=g)
    O = torch.empty((1, H * g, n_m, d), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((H * g * n_m,), float("nan"), dtype=torch.float32, device="cuda")
    m.maskkv_attend_full(desc, Q, K, V, 0.0, O, lse, hp.workspace(m.maskkv_attend_workspace_bytes(desc, True)))
    scores = torch.full((H, P), float("nan"), dtype=torch.float32, device="cuda")
    mass = torch.full((H,), float("nan"), dtype=torch.float32, device="cuda")
    m.maskkv_score_given_lse(desc, Q, K, 0.0, lse, scores, P, mass, hp.workspace(m.maskkv_score_workspace_bytes(desc)))
    torch.cuda.synchronize()
    sc, ms = scores.cpu().numpy(), mass.cpu().numpy()
    for h in range(H):
        I, mass_ref = orc.score_grouped(Qg[h * g:(h + 1) * g], L.K[h], P)
        assert (np.abs(sc[h] - I) / I).max() <= hp.SCORE_RTOL
        assert abs(ms[h] - mass_ref) <= hp.SCORE_RTOL * mass_ref
