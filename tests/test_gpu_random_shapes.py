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
