"""GPU parity of the relative-L1 kernel and of the hyper-parameter search (Sec. 3.6) against the oracle.

The search takes discrete decisions from floating-point tables: the tables (mean sparsity, worst
relative L1 per candidate and head) must agree with the oracle's within the tolerances of the outputs
they are made of, and the decision must be the oracle's wherever the oracle's own tables decide it
with a margin larger than those tolerances; otherwise it must be admissible and as sparse by the
oracle's tables.
"""
import math

import numpy as np
import pytest

from oracle import sparge_oracle as so
from synth import make_workload
from tests.helpers import REF_SLACK, f32, small_workload, to_torch

pytestmark = pytest.mark.gpu

TOL_L1 = 5e-3        # two outputs, each within 2e-3 of its oracle counterpart
TOL_SPARSITY = 1e-2  # a few borderline stage-2 decisions per head


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2502_18137_amd as sp
    sp.load_library()
    return sp


@pytest.mark.parametrize("dtype,d,strided", [("fp16", 64, False), ("bf16", 128, True)])
def test_rel_l1_sums(sp, dtype, d, strided):
    import torch
    rng = np.random.default_rng(3)
    B, H, N = 2, 3, 333
    a = rng.standard_normal((B, H, N, d)).astype(np.float32)
    b = a + 0.05 * rng.standard_normal((B, H, N, d)).astype(np.float32)
    ta, tb = to_torch(a, dtype), to_torch(b, dtype)
    if strided:  # [B,N,H,d] storage viewed as [B,H,N,d]
        ta = ta.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        tb = tb.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    out = sp.sparge_rel_l1(ta, tb).cpu().numpy()
    xa, xb = ta.float().cpu().numpy().astype(np.float64), tb.float().cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(out[..., 0], np.abs(xb - xa).sum(axis=(2, 3)), rtol=1e-12)
    np.testing.assert_allclose(out[..., 1], np.abs(xb).sum(axis=(2, 3)), rtol=1e-12)
    for h in range(H):
        assert out[0, h, 0] / out[0, h, 1] == pytest.approx(so.rel_l1(xa[0, h], xb[0, h]), rel=1e-12)


@pytest.mark.parametrize("causal,dtype,d,pv_fp8", [(False, "bf16", 64, False), (True, "fp16", 128, False),
                                                   (False, "bf16", 128, True)])
def test_tuner_matches_the_oracle(sp, causal, dtype, d, pv_fp8):
    N, H = 640, 2
    ws = [small_workload(f"tune{i}", N=N, d=d, dtype=dtype, H=H, causal=causal, seed=20 + i, noise=0.5)
          for i in range(2)]
    xs = [make_workload(w) for w in ws]
    inputs = [tuple(to_torch(x[t], dtype) for t in "qkv") for x in xs]
    taus, thetas, lams = [0.5, 0.8, 0.95], [-0.5, 0.4, 0.8], [-10.0, -5.0, -2.5]
    l1, l2 = 0.05, 0.07
    print("running the GPU search", flush=True)
    got = sp.sparge_tune(inputs, taus, thetas, lams, l1, l2, causal=causal, pv_fp8=pv_fp8)
    slack = sp.REF_SLACK_LOG2_FP8 * math.log(2.0) if pv_fp8 else REF_SLACK
    for h in range(H):
        print(f"oracle search, head {h}", flush=True)
        ref = so.tune_head([(x["q"][0, h], x["k"][0, h], x["v"][0, h]) for x in xs],
                           [f32(t) for t in taus], [f32(t) for t in thetas], [f32(t) for t in lams],
                           f32(l1), f32(l2), causal=causal, pv_dtype="fp8e4m3" if pv_fp8 else dtype,
                           ref_slack=slack)
        s1 = got["stage1"][:, :, h, :]
        print(f"  oracle: tau {ref.tau} theta {ref.theta} lam {ref.lam} sparsity {ref.sparsity:.4f} l1 {ref.l1:.4f}; "
              f"gpu: tau {got['tau'][h]} theta {got['theta'][h]} lam {got['lam'][h]} "
              f"sparsity {got['sparsity'][h]:.4f} l1 {got['l1'][h]:.4f}", flush=True)
        np.testing.assert_allclose(s1[..., 0], ref.stage1[..., 0], atol=TOL_SPARSITY)
        np.testing.assert_allclose(s1[..., 1], ref.stage1[..., 1], atol=TOL_L1)
        # stage 1 decision: unambiguous for the oracle -> identical; else admissible and as sparse by its tables
        flat = ref.stage1.reshape(-1, 2)
        k_ref = taus.index(pytest.approx(ref.tau)) * len(thetas) + thetas.index(pytest.approx(ref.theta))
        k_got = [f32(t) for t in taus].index(got["tau"][h]) * len(thetas) + [f32(t) for t in thetas].index(got["theta"][h])
        clear_l1 = np.all(np.abs(flat[:, 1] - l1) > TOL_L1)
        others = np.delete(flat, k_ref, axis=0)
        adm_others = others[others[:, 1] < l1]
        clear_sp = adm_others.size == 0 or np.all(np.abs(adm_others[:, 0] - flat[k_ref, 0]) > 2 * TOL_SPARSITY)
        if clear_l1 and clear_sp:
            assert k_got == k_ref
        else:
            assert flat[k_got, 1] < l1 + TOL_L1 and flat[k_got, 0] >= flat[k_ref, 0] - 2 * TOL_SPARSITY
        if k_got == k_ref:
            s2 = got["stage2"][:, h, :]
            np.testing.assert_allclose(s2[:, 0], ref.stage2[:, 0], atol=TOL_SPARSITY)
            np.testing.assert_allclose(s2[:, 1], ref.stage2[:, 1], atol=TOL_L1)
            clear2 = np.all(np.abs(ref.stage2[:, 1] - l2) > TOL_L1)
            if clear2 and clear_l1 and clear_sp:
                sp_sorted = np.sort(np.concatenate([ref.stage2[ref.stage2[:, 1] < l2, 0], [flat[k_ref, 0]]]))[::-1]
                if len(sp_sorted) < 2 or sp_sorted[0] - sp_sorted[1] > 2 * TOL_SPARSITY:
                    assert got["lam"][h] == (f32(ref.lam) if np.isfinite(ref.lam) else -math.inf)
            assert got["sparsity"][h] == pytest.approx(ref.sparsity, abs=2 * TOL_SPARSITY)
        assert got["l1"][h] < l2 + TOL_L1


def test_rel_l1_and_tuner_are_reproducible(sp):
    """The error sums are reduced in a fixed order: the same inputs give the same bits on every call, and the
    search, which compares those sums with its bounds, returns identical tables and choices."""
    import torch
    ws = [small_workload(f"rep{i}", N=3000, d=128, dtype="bf16", H=3, seed=60 + i, noise=0.6) for i in range(2)]
    xs = [make_workload(w) for w in ws]
    inputs = [tuple(to_torch(x[t], "bf16") for t in "qkv") for x in xs]
    a, b = inputs[0][2], inputs[1][2]
    first = sp.sparge_rel_l1(a, b)
    for _ in range(5):
        assert torch.equal(sp.sparge_rel_l1(a, b), first)
    runs = [sp.sparge_tune(inputs, [0.6, 0.9], [0.3, 0.6], [-6.0, -3.0], 0.05, 0.06) for _ in range(3)]
    for r in runs[1:]:
        assert np.array_equal(r["stage1"], runs[0]["stage1"]) and np.array_equal(r["stage2"], runs[0]["stage2"])
        assert r["tau"] == runs[0]["tau"] and r["theta"] == runs[0]["theta"] and r["lam"] == runs[0]["lam"]
