"""maskkv_score_static (the entry point for callers that cannot allocate) against maskkv_score, through the C ABI.

Two calls in a row on the same GPU, the second on a smaller problem, so that whatever the first call left in the
library's static scratch array is still there when the second one runs.  Both entry points run the same kernels,
so the scores and the prompt mass must agree bit for bit; the static call is also held to the oracle at the
score tolerance.
"""
import numpy as np
import pytest
import torch

from paper_2510_09309_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def run_both(batch: hp.Batch):
    m = hp.mk()
    stride = (batch.P_max + 63) // 64 * 64
    shape = (batch.B * batch.H, stride)
    want = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    want_mass = torch.full((shape[0],), float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    got_mass = torch.full((shape[0],), float("nan"), dtype=torch.float32, device="cuda")
    ws = hp.workspace(m.maskkv_score_workspace_bytes(batch.desc))
    m.maskkv_score(batch.desc, batch.Q, batch.K, 0.0, want, stride, want_mass, ws)
    m.maskkv_score_static(batch.desc, batch.Q, batch.K, 0.0, got, stride, got_mass)
    torch.cuda.synchronize()
    return want, want_mass, got, got_mass


def test_static_scratch_score_matches_workspace_score_twice():
    m = hp.mk()
    big = hp.Batch([synth.make_layer(41, H=6, d=128, P=5000, n_m=200, dtype="bf16", n_planted=60, amplitude=2.5),
                    synth.make_layer(42, H=6, d=128, P=3333, n_m=200, dtype="bf16", n_planted=40, amplitude=2.5)])
    small = hp.Batch([synth.make_layer(43, H=3, d=128, P=700, n_m=72, dtype="bf16", n_planted=10, amplitude=2.5)])
    for batch in (big, small):      # the second call is the smaller one
        assert m.maskkv_score_workspace_bytes(batch.desc) <= 16 << 20
        want, want_mass, got, got_mass = run_both(batch)
        assert torch.equal(got.view(torch.int32), want.view(torch.int32)), "scores differ (NaN padding included)"
        assert torch.equal(got_mass, want_mass)
        worst = hp.check_scores(batch, got, got_mass)
        assert worst <= hp.SCORE_RTOL


def test_static_scratch_rejects_oversized_descriptions():
    m = hp.mk()
    desc = m.Desc(B=8, H=32, d=128, dtype=m.MASKKV_BF16, n_resp=512, P_max=16384)
    assert m.maskkv_score_workspace_bytes(desc) > 16 << 20
    fake = m._CTensor(0x1000, 32 * (16384 + 512) * 128, (16384 + 512) * 128, 128, None)
    scores = torch.empty(16, dtype=torch.float32, device="cuda")
    with pytest.raises(m.MaskKVError) as e:
        m.maskkv_score_static(desc, fake, fake, 0.0, scores, 16384, None)
    assert e.value.status == 4 and "static" in str(e.value)
