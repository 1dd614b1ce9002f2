"""The whole path (score -> on-device head budgets -> select -> compact -> attend) captured as one HIP graph
must give, on every replay, exactly what the eager calls give (needs an MI355X).

The library enqueues kernels only (no memsets, no allocation, no synchronisation), so a caller may capture
it; the replays here are separated by eager work and synchronisation and each one is compared.
"""
import numpy as np
import pytest
import torch

from paper_2510_09309_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager_calls():
    m = hp.mk()
    layers = [synth.make_layer(4000 + l, H=4, d=128, P=3000 + 123 * l, n_m=96, dtype="bf16", n_planted=30, amplitude=2.5)
              for l in range(2)]
    batches = [hp.Batch([L]) for L in layers]
    k_l, alpha = 48, 0.1
    bufs = []
    for bt in batches:
        H, P, n_m, d = bt.H, bt.P[0], bt.n_m, bt.d
        cap = H * k_l
        dev = dict(device="cuda")
        bufs.append(dict(
            scores=torch.zeros((H, P), dtype=torch.float32, **dev), mass=torch.zeros(H, dtype=torch.float32, **dev),
            budgets=torch.zeros(H, dtype=torch.int32, **dev), idx=torch.zeros(cap, dtype=torch.int32, **dev),
            cu=torch.zeros(H + 1, dtype=torch.int32, **dev), Kc=torch.zeros((cap, d), dtype=torch.bfloat16, **dev),
            Vc=torch.zeros((cap, d), dtype=torch.bfloat16, **dev), cap=cap,
            O=torch.zeros((1, H, n_m, d), dtype=torch.bfloat16, **dev),
            ws_score=hp.workspace(m.maskkv_score_workspace_bytes(bt.desc)),
            ws_sel=hp.workspace(m.maskkv_select_workspace_bytes(bt.desc)),
            ws_att=hp.workspace(m.maskkv_attend_workspace_bytes(bt.desc, False)), resp=bt.resp_views()))

    def run(stream):
        for bt, x in zip(batches, bufs):
            P = bt.P[0]
            m.maskkv_score(bt.desc, bt.Q, bt.K, 0.0, x["scores"], P, x["mass"], x["ws_score"], stream)
            m.maskkv_head_budgets(bt.desc, x["mass"], k_l, alpha, x["budgets"], stream)
            m.maskkv_select(bt.desc, x["scores"], P, 7, m.POOL_MEAN, x["budgets"], x["idx"], x["cu"], x["cap"],
                            x["ws_sel"], stream)
            m.maskkv_compact(bt.desc, bt.K, bt.V, x["idx"], x["cu"], x["cap"], x["Kc"], x["Vc"], stream)
            m.maskkv_attend(bt.desc, bt.Q, x["Kc"], x["Vc"], x["cu"], x["cap"], x["resp"][0], x["resp"][1], 0.0,
                            x["O"], None, x["ws_att"], stream)

    outputs = ("scores", "budgets", "idx", "cu", "Kc", "Vc", "O")
    run(torch.cuda.current_stream())
    torch.cuda.synchronize()
    want = [{k: x[k].clone() for k in outputs} for x in bufs]
    assert all(int(w["cu"][-1]) > 0 for w in want)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        run(torch.cuda.current_stream())
    for replay in range(3):
        for x in bufs:                       # eager work between the replays: wipe every output
            for k in outputs:
                x[k].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for x, w in zip(bufs, want):
            for k in outputs:
                assert torch.equal(x[k], w[k]), f"replay {replay}: {k} differs from the eager result"
