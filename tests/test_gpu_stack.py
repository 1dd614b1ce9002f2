"""The path with budgets that never leave the device (score -> head budgets -> select -> compact -> attend),
layer after layer, against the oracle's own chain prompt_preference -> head_budgets -> select -> attend, eagerly
and on a replay of the captured HIP graph (needs an MI355X)."""
import numpy as np
import pytest
import torch

from oracle import maskkv_oracle as orc
from paper_2510_09309_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def test_device_budget_stack_matches_the_oracle_eagerly_and_on_a_graph_replay():
    m = hp.mk()
    H, d, n_m, k_l, alpha, window = 8, 128, 96, 160, 0.1, 7
    layers = []
    for l, P in enumerate((5000, 3333)):     # one prompt longer than a selection chunk, one shorter
        L = synth.make_layer(4100 + l, H=H, d=d, P=P, n_m=n_m, dtype="bf16", n_planted=60, amplitude=2.5)
        for h in range(H):                   # heads that differ in how much the mask queries prefer the prompt:
            pull = np.float32(9.0 * ((h + 3 * l) % H))   # response keys pulled towards the queries' shared direction
            L.K[h, P:] = synth.round_to_bf16(L.K[h, P:] + pull * L.u[h])
        layers.append(L)
    batches = [hp.Batch([L]) for L in layers]
    cap = H * k_l
    dev = dict(device="cuda")
    bufs = []
    for bt in batches:
        P = bt.P[0]
        bufs.append(dict(
            scores=torch.zeros((H, P), dtype=torch.float32, **dev), mass=torch.zeros(H, dtype=torch.float32, **dev),
            budgets=torch.zeros(H, dtype=torch.int32, **dev), idx=torch.zeros(cap, dtype=torch.int32, **dev),
            cu=torch.zeros(H + 1, dtype=torch.int32, **dev), Kc=torch.zeros((cap, d), dtype=torch.bfloat16, **dev),
            Vc=torch.zeros((cap, d), dtype=torch.bfloat16, **dev),
            O=torch.zeros((1, H, n_m, d), dtype=torch.bfloat16, **dev),
            ws_score=hp.workspace(m.maskkv_score_workspace_bytes(bt.desc)),
            ws_sel=hp.workspace(m.maskkv_select_workspace_bytes(bt.desc)),
            ws_att=hp.workspace(m.maskkv_attend_workspace_bytes(bt.desc, False)), resp=bt.resp_views()))
    outputs = ("scores", "mass", "budgets", "idx", "cu", "Kc", "Vc", "O")

    def run(stream):
        for bt, x in zip(batches, bufs):
            P = bt.P[0]
            m.maskkv_score(bt.desc, bt.Q, bt.K, 0.0, x["scores"], P, x["mass"], x["ws_score"], stream)
            m.maskkv_head_budgets(bt.desc, x["mass"], k_l, alpha, x["budgets"], stream)
            m.maskkv_select(bt.desc, x["scores"], P, window, m.POOL_MEAN, x["budgets"], x["idx"], x["cu"], cap,
                            x["ws_sel"], stream)
            m.maskkv_compact(bt.desc, bt.K, bt.V, x["idx"], x["cu"], cap, x["Kc"], x["Vc"], stream)
            m.maskkv_attend(bt.desc, bt.Q, x["Kc"], x["Vc"], x["cu"], cap, x["resp"][0], x["resp"][1], 0.0, x["O"],
                            None, x["ws_att"], stream)

    # the oracle's chain, once
    refs = []
    for L in layers:
        I = [orc.score(L.Q[h], L.K[h], L.P) for h in range(H)]
        pref = orc.prompt_preference(np.array([i[1] for i in I]), n_m)
        exact = alpha * k_l + (1 - alpha) * H * k_l * pref / pref.sum()
        refs.append(dict(I=[i[0] for i in I], budgets=orc.head_budgets(pref, k_l, alpha), exact=exact))
        assert len(set(refs[-1]["budgets"].tolist())) > H // 2, "the heads' budgets should differ"

    def check(tag):
        n_band = 0
        for L, x, ref in zip(layers, bufs, refs):
            got = x["budgets"].cpu().numpy()
            # the floor is taken in single precision on the device: a head whose real-valued budget lies within
            # 1e-3 of an integer may land on either side; every other head must match the oracle's integer
            near_int = np.abs(ref["exact"] - np.rint(ref["exact"])) < 1e-3
            assert np.all((got == ref["budgets"]) | near_int), f"{tag}: budgets {got} vs {ref['budgets']}"
            assert np.all(np.abs(got - ref["budgets"]) <= 1) and got.sum() <= cap
            keeps, cu_h = hp.split_idx(x["idx"], x["cu"])
            assert cu_h.tolist() == np.concatenate([[0], np.cumsum(got)]).tolist()
            sc = x["scores"].cpu().numpy()
            Kc_h, Vc_h = x["Kc"].float().cpu().numpy(), x["Vc"].float().cpu().numpy()
            O_h = x["O"].float().cpu().numpy()
            for h in range(H):
                assert (np.abs(sc[h] - ref["I"][h]) / ref["I"][h]).max() <= hp.SCORE_RTOL
                n_band += hp.check_keep_against_oracle(orc.pool(ref["I"][h], window), int(got[h]), keeps[h],
                                                       f"{tag} h{h}")
                keep = keeps[h]
                assert np.array_equal(Kc_h[cu_h[h]:cu_h[h + 1]], L.K[h, keep])
                assert np.array_equal(Vc_h[cu_h[h]:cu_h[h + 1]], L.V[h, keep])
                want = orc.attend(L.Q[h], L.K[h, keep], L.V[h, keep], L.K[h, L.P:], L.V[h, L.P:])
                assert np.abs(O_h[0, h] - want).max() <= hp.ATTEND_ATOL_BF16, f"{tag} h{h}"
        assert n_band <= 2 * H
        return n_band

    run(torch.cuda.current_stream())
    torch.cuda.synchronize()
    check("eager")

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        run(torch.cuda.current_stream())
    for x in bufs:                           # eager work between capture and replay: wipe every output
        for k in outputs:
            x[k].zero_()
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    check("graph replay")
