"""sparge_predict_static: the predictor with its intermediates in the library's static device array, for callers
that cannot pass a workspace or allocate.  Checked through the C ABI against sparge_predict (same kernels, caller's
workspace) bit for bit and against the oracle's mask, on two calls in a row, the second with a smaller input
(the array keeps the first call's contents); shapes beyond the array are rejected."""
import numpy as np
import pytest

from oracle import sparge_oracle as so
from tests.helpers import f32, gpu_inputs, small_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2502_18137_amd as sp
    sp.load_library()
    return sp


def test_predict_static_matches_predict_on_two_calls_in_a_row(sp):
    import torch
    for name, N, H, d, dtype, causal, seed in (("first", 5000, 4, 128, "bf16", False, 51),
                                               ("second_smaller", 700, 2, 64, "fp16", True, 52)):
        print(f"call {name}: N={N} H={H} d={d} {dtype} causal={causal}", flush=True)
        w = small_workload(name, N=N, d=d, dtype=dtype, H=H, causal=causal, seed=seed)
        x, Q, K, V = gpu_inputs(w)
        assert sp.sparge_workspace_bytes(Q, sp.WS_PREDICT) <= sp.STATIC_SCRATCH_BYTES
        ref_mask, ref_sq, ref_sk = sp.sparge_predict(Q, K, w.tau, w.theta, causal=causal, return_sims=True)
        mask = torch.full_like(ref_mask, 7)
        sq, sk = torch.full_like(ref_sq, -1.0), torch.full_like(ref_sk, -1.0)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        sp.sparge_predict_static(Q, K, w.tau, w.theta, mask, causal=causal, sim_q=sq, sim_k=sk)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(mask, ref_mask) and torch.equal(sq, ref_sq) and torch.equal(sk, ref_sk)
        m = mask.cpu().numpy()
        for h in range(H):
            pr = so.predict(x["q"][0, h], x["k"][0, h], f32(w.tau), f32(w.theta), causal=causal)
            assert not ((m[0, h] != pr.mask) & ~pr.dont_care).any()
            np.testing.assert_allclose(sq[0, h].cpu().numpy(), pr.sim_q, atol=1e-12)


def test_predict_static_rejects_what_does_not_fit(sp):
    import torch
    Q = torch.zeros((1, 24, 46080, 128), dtype=torch.bfloat16, device="cuda")
    assert sp.sparge_workspace_bytes(Q, sp.WS_PREDICT) > sp.STATIC_SCRATCH_BYTES
    mask = torch.zeros((1, 24, 360, 720), dtype=torch.uint8, device="cuda")
    with pytest.raises(sp.SpargeError, match="static buffer"):
        sp.sparge_predict_static(Q, Q, 0.9, 0.5, mask)
    assert not mask.any()
