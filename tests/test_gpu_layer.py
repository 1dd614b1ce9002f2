"""Layer importance kernel against the float64 oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

from oracle import maskkv_oracle as orc
from paper_2510_09309_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu

# fp32 accumulation of `hidden` products and of n cosines against float64: a few ulp of fp32 on values <= 1
IMPORTANCE_ATOL = 5e-6


def gpu_importance(h_in: np.ndarray, h_out: np.ndarray, dtype: str, row_stride=None) -> float:
    m = hp.mk()
    n, hidden = h_in.shape
    stride = hidden if row_stride is None else row_stride
    tdt = hp.torch_dtype(dtype)
    a = torch.zeros((n, stride), dtype=tdt, device="cuda")
    b = torch.full((n, stride), 7.0, dtype=tdt, device="cuda")   # padding columns must never be read
    a[:, :hidden] = torch.from_numpy(h_in).to("cuda").to(tdt)
    b[:, :hidden] = torch.from_numpy(h_out).to("cuda").to(tdt)
    out = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    ws = hp.workspace(m.maskkv_layer_importance_workspace_bytes())
    m.maskkv_layer_importance(a[:, :hidden], b[:, :hidden], out, ws)
    torch.cuda.synchronize()
    return float(out.item())


@pytest.mark.parametrize("n,hidden,dtype,drift,stride", [
    (1000, 4096, "bf16", 0.5, None),    # the model's hidden size, several rows per wave
    (37, 512, "f32", 2.0, 520),         # ragged rows per wave, padded row stride
    (1, 4096, "bf16", 1.0, None),       # a single token
    (9001, 1024, "bf16", 0.1, 1032),    # more rows than waves in the grid
    (300, 8, "f32", 1.0, None),         # shortest legal row: most lanes idle
])
def test_layer_importance_matches_oracle(n, hidden, dtype, drift, stride):
    h_in, h_out = synth.make_hidden_states(500 + n, n, hidden, dtype, drift)
    want = orc.layer_importance(h_in, h_out)
    got = gpu_importance(h_in, h_out, dtype, stride)
    assert abs(got - want) <= IMPORTANCE_ATOL, (got, want)


def test_layer_importance_special_cases():
    h_in, _ = synth.make_hidden_states(1, 64, 256, "f32", 0.0)
    assert abs(gpu_importance(h_in, h_in, "f32")) <= IMPORTANCE_ATOL               # identical states: 0
    assert abs(gpu_importance(h_in, -h_in, "f32") - 2.0) <= IMPORTANCE_ATOL        # opposite states: 2
    assert abs(gpu_importance(h_in, 3.0 * h_in, "f32")) <= IMPORTANCE_ATOL         # scale invariance


def test_importance_feeds_layer_budgets():
    """Importances measured on the device, budgets from the host formula, both against the oracle."""
    m = hp.mk()
    drifts = [1.5, 0.2, 0.3, 0.25, 0.4, 1.0]
    imps, refs = [], []
    for l, dr in enumerate(drifts):
        h_in, h_out = synth.make_hidden_states(700 + l, 257, 1024, "bf16", dr)
        imps.append(gpu_importance(h_in, h_out, "bf16"))
        refs.append(orc.layer_importance(h_in, h_out))
    assert np.abs(np.array(imps) - np.array(refs)).max() <= IMPORTANCE_ATOL
    k_p = 6 * 256
    got = m.maskkv_layer_budgets(imps, k_p, 0.4)
    want = orc.layer_budgets(np.array(imps, dtype=np.float32).astype(np.float64), k_p, np.float64(np.float32(0.4)))
    assert got == want.tolist() and sum(got) <= k_p
    assert got[0] > got[1] and got[-1] > got[2]   # the drifting boundary layers receive more


def test_measurement_probes_run_and_the_copy_is_exact():
    from paper_2510_09309_amd import bench_binding as bb
    out = torch.full((8 * 256,), float("nan"), dtype=torch.float32, device="cuda")
    flops = bb.maskkv_bench_probe(0, 10, None, out, 8)
    torch.cuda.synchronize()
    assert flops == 8 * 4 * 4 * 10 * 32768.0 and bool(torch.isfinite(out).all())
    out.fill_(float("nan"))
    n_exp = bb.maskkv_bench_probe(1, 10, None, out, 8)
    torch.cuda.synchronize()
    assert n_exp == 8 * 256 * 8 * 10 and bool(((out > 0) & (out <= 8)).all())      # eight values in (0, 1] per lane
    out.fill_(float("nan"))
    assert bb.maskkv_bench_probe(4, 10, None, out, 8) == 8 * 4 * 16 * 10 * 32768.0
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    operands = (torch.randn(64 * 24 * 8, device="cuda") / 11.3).to(torch.bfloat16)   # 24 KiB of Gaussian bf16
    out.fill_(float("nan"))
    assert bb.maskkv_bench_probe(5, 10, operands, out, 8) == 8 * 4 * 16 * 10 * 32768.0
    assert bb.maskkv_bench_probe(6, 9, operands, out, 8) == 8 * 4 * 16 * 10 * 32768.0      # iterations run in pairs
    assert bb.maskkv_bench_probe(7, 10, operands, out, 4) == 4 * 4 * 16 * 10 * 32768.0     # matrix and vector halves
    assert bb.maskkv_bench_probe(8, 10, operands, out, 4) == 4 * 4 * 16 * 10 * 32768.0     # the matrix half alone
    assert bb.maskkv_bench_probe(9, 10, operands, out, 4) == 4 * 256 * 32 * 10             # the vector half alone
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    src = torch.arange(100003 * 4, dtype=torch.int32, device="cuda")               # a ragged number of 16-byte pieces
    dst = torch.zeros_like(src)
    moved = bb.maskkv_bench_probe(2, 0, src, dst, 7)
    torch.cuda.synchronize()
    assert moved == 2.0 * src.numel() * 4 and torch.equal(src, dst)
    words = torch.zeros(7 * 256, dtype=torch.int32, device="cuda")
    assert bb.maskkv_bench_probe(3, 0, src, words, 7) == src.numel() * 4
    torch.cuda.synchronize()
    fold = int(np.bitwise_xor.reduce(src.cpu().numpy()))
    assert int(np.bitwise_xor.reduce(words.cpu().numpy())) == fold


def test_stage_marks_leave_the_scores_unchanged():
    """maskkv_bench_score_marked runs the body of maskkv_score: same bits, four ordered events."""
    from paper_2510_09309_amd import bench_binding as bb
    from paper_2510_09309_amd import synth
    m = hp.mk()
    batch = hp.Batch([synth.make_layer(5, H=2, d=128, P=3000, n_m=64, dtype="bf16", n_planted=10, amplitude=2.5)])
    want, want_mass = hp.gpu_score(batch)
    got = torch.full_like(want, float("nan"))
    mass = torch.full_like(want_mass, float("nan"))
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for e in ev:
        e.record()                       # creates the underlying HIP events
    torch.cuda.synchronize()
    ws = hp.workspace(m.maskkv_score_workspace_bytes(batch.desc))
    bb.maskkv_bench_score_marked(batch.desc, batch.Q, batch.K, 0.0, got, got.stride(0), mass, ws,
                                 [e.cuda_event for e in ev])
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int32), want.view(torch.int32)) and torch.equal(mass, want_mass)
    assert ev[0].elapsed_time(ev[1]) > 0 and ev[1].elapsed_time(ev[2]) > 0 and ev[2].elapsed_time(ev[3]) > 0
