"""The library allocates nothing, never synchronises (sparge_tune aside) and clears its counters with a fill
kernel, so a caller may record its calls into a HIP graph.  Recorded here: the whole of Algorithm 1
(sparge_forward) in its three product variants; every replay, with other eager work and synchronisations
in between, must reproduce the eager result bit for bit, also after the inputs change in place."""
import numpy as np
import pytest

from tests.helpers import gpu_inputs, small_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2502_18137_amd as sp
    sp.load_library()
    return sp


@pytest.mark.parametrize("variant", [{}, {"pv_fp8": True}, {"qk16": True}], ids=["int8_16bit", "fp8_pv", "qk16"])
def test_forward_replays_from_a_graph(sp, variant):
    import torch
    w = small_workload("graph", N=1500, d=128, dtype="bf16", H=3, seed=12)
    x, Q, K, V = gpu_inputs(w)
    w2 = small_workload("graph2", N=1500, d=128, dtype="bf16", H=3, seed=13)
    x2, Q2, K2, V2 = gpu_inputs(w2)
    ws = torch.empty(sp.sparge_workspace_bytes(Q, sp.WS_FORWARD, variant.get("pv_fp8", False)), dtype=torch.uint8,
                     device="cuda")
    O = torch.empty_like(V)
    eager1 = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, **variant).clone()
    eager2 = sp.sparge_forward(Q2, K2, V2, w.tau, w.theta, w.lam, **variant).clone()
    assert not torch.equal(eager1, eager2)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, ws=ws, out=O, **variant)   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, ws=ws, out=O, **variant)
    torch.cuda.synchronize()
    for rep in range(4):
        O.zero_()
        ws.random_(0, 255)                          # stale workspace contents must not matter
        if rep == 2:                                # new inputs in the same buffers
            Q.copy_(Q2); K.copy_(K2); V.copy_(V2)
        g.replay()
        torch.cuda.synchronize()
        want = eager1 if rep < 2 else eager2
        assert torch.equal(O, want), f"replay {rep} differs from the eager result"
        junk = (torch.randn(1 << 20, device="cuda") * 2).sum()   # unrelated eager work between replays
        torch.cuda.synchronize()
        assert torch.isfinite(junk)


def test_two_graphs_replayed_on_two_streams(sp):
    """Two captures of sparge_forward, each with its own workspace, outputs and inputs (one causal), replayed at
    the same time on two streams, three rounds with eager launches in between: every replay reproduces its
    eager result bit for bit.  (The item counters of the attention kernel live in each call's workspace: two
    launches in flight share nothing.)"""
    import torch
    cases = []
    for seed, causal, d in ((21, False, 128), (22, True, 64)):
        w = small_workload(f"g{seed}", N=4000, d=d, dtype="bf16", H=6, seed=seed, causal=causal)
        x, Q, K, V = gpu_inputs(w)
        eager, mask, stats = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, causal=causal, return_mask=True,
                                               return_stats=True)
        ws = torch.empty(sp.sparge_workspace_bytes(Q, sp.WS_FORWARD), dtype=torch.uint8, device="cuda")
        O = torch.empty_like(V)
        st = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, causal=causal, ws=ws, out=O)
            st.synchronize()
            with torch.cuda.graph(g, stream=st):
                sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, causal=causal, ws=ws, out=O)
        torch.cuda.synchronize()
        cases.append((w, Q, K, V, eager.clone(), O, ws, st, g))
    for rep in range(3):
        for (_, _, _, _, _, O, ws, _, _) in cases:
            O.zero_()
            ws.random_(0, 255)
        torch.cuda.synchronize()
        for (_, _, _, _, _, _, _, st, g) in cases:       # both in flight together
            with torch.cuda.stream(st):
                g.replay()
        # an eager call of a third problem on the default stream while the replays run
        w0, Q0, K0, V0, e0 = cases[0][:5]
        again = sp.sparge_forward(Q0, K0, V0, w0.tau, w0.theta, w0.lam, causal=w0.causal)
        torch.cuda.synchronize()
        assert torch.equal(again, e0)
        for n, (_, _, _, _, eager, O, _, _, _) in enumerate(cases):
            assert torch.equal(O, eager), f"round {rep}, graph {n} differs from the eager result"
