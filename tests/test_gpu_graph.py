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
