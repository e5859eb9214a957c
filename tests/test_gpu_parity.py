"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: INT8 values, scales, K mean and block masks bit-exact (mask entries the oracle flags as within
1e-5 of a threshold are exempt; INT8 values also against the exactly rounded quotient away from ties);
outputs, per head and per row, against three evaluations of Alg. 1 by the oracle -- P~ rounded where the
kernel rounds it (relative L1 2e-3), the recurrence as printed with P~ rounded to 16 bits, and the loop
with nothing rounded -- at the bars of tests/helpers.py, and within 3e-2 of exact fp64 attention
restricted to the same blocks.
"""
import math

import numpy as np
import pytest

from oracle import sparge_oracle as so
from synth import CONFIGS
from synth.workloads import scaled
from tests.helpers import REF_SLACK, check_output_parity, f32, gpu_inputs, small_workload, to_torch

pytestmark = pytest.mark.gpu

REL_L1_EMUL = 2e-3
REL_L1_EXACT = 3e-2


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2502_18137_amd as sp
    sp.load_library()
    return sp


def cpu(t):
    import torch
    if t.dtype in (torch.float16, torch.bfloat16):
        t = t.float()
    return t.detach().cpu().numpy()


CASES = [
    CONFIGS["tiny"],
    small_workload("ragged64", N=700, d=64, dtype="bf16", seed=2),
    small_workload("ragged128", N=1000, d=128, dtype="bf16", seed=3),
    small_workload("short", N=77, d=128, dtype="fp16", H=1, seed=4),
    small_workload("one_row", N=1, d=64, dtype="fp16", H=1, seed=5),
    small_workload("causal128", N=1100, d=128, dtype="bf16", causal=True, seed=6),
    small_workload("causal64", N=520, d=64, dtype="fp16", causal=True, seed=7),
]
IDS = [w.name for w in CASES]


@pytest.mark.parametrize("w", CASES, ids=IDS)
def test_quantize_bit_exact(sp, w):
    print(f"case {w.name} N={w.N} d={w.d} {w.dtype}", flush=True)
    x, Q, K, V = gpu_inputs(w)
    Qq, Kq, qs, ks, km = (cpu(t) for t in sp.sparge_quantize(Q, K))
    for h in range(w.H):
        oq, odq = so.quantize_q(x["q"][0, h])
        ok, odk, omean = so.quantize_k(x["k"][0, h])
        assert (Qq[0, h] == oq).all()
        assert (qs[0, h].view(np.uint32) == odq.view(np.uint32)).all()
        assert (km[0, h].view(np.uint32) == omean.view(np.uint32)).all()
        assert (Kq[0, h] == ok).all()
        assert (ks[0, h].view(np.uint32) == odk.view(np.uint32)).all()
        # and against the mathematics: the exactly rounded quotient 127 x / amax wherever it is not within
        # 2^-15 of a tie (there the fp32 sequence above is the specification)
        qe, q_tie = so.quantize_exact(np.asarray(x["q"][0, h], dtype=np.float32), so.BQ)
        ke, k_tie = so.quantize_exact(np.asarray(x["k"][0, h], dtype=np.float32) - omean[None, :], so.BK)
        assert ((Qq[0, h] == qe) | q_tie).all() and ((Kq[0, h] == ke) | k_tie).all()
        print(f"  head {h}: quotients within 2^-15 of a tie: Q {int(q_tie.sum())}, K {int(k_tie.sum())} of {q_tie.size}",
              flush=True)


@pytest.mark.parametrize("w", CASES, ids=IDS)
def test_predict_mask_matches(sp, w):
    print(f"case {w.name}", flush=True)
    x, Q, K, V = gpu_inputs(w)
    mask, sq, sk = sp.sparge_predict(Q, K, w.tau, w.theta, causal=w.causal, return_sims=True)
    mask, sq, sk = cpu(mask), cpu(sq), cpu(sk)
    for h in range(w.H):
        pr = so.predict(x["q"][0, h], x["k"][0, h], f32(w.tau), f32(w.theta), causal=w.causal)
        np.testing.assert_allclose(sq[0, h], pr.sim_q, atol=1e-12)
        np.testing.assert_allclose(sk[0, h], pr.sim_k, atol=1e-12)
        bad = (mask[0, h] != pr.mask) & ~pr.dont_care
        assert not bad.any(), (h, np.argwhere(bad)[:5])
        assert pr.dont_care.mean() < 0.05


@pytest.mark.parametrize("theta,tau", [(-math.inf, 0.5), (1.5, 0.5), (0.5, 1.0), (0.85, 0.7)])
def test_predict_switches(sp, theta, tau):
    w = CONFIGS["tiny"]
    x, Q, K, V = gpu_inputs(w)
    mask = cpu(sp.sparge_predict(Q, K, tau, theta))
    for h in range(w.H):
        pr = so.predict(x["q"][0, h], x["k"][0, h], f32(tau), f32(theta))
        assert not ((mask[0, h] != pr.mask) & ~pr.dont_care).any()
    if theta > 1:
        assert mask.all()


def check_attention(sp, w, x, Q, K, V, mask_np, lam, heads=None):
    """GPU sparge_attn against the oracle loop on the same mask and lambda: the three evaluations and the bars
    of helpers.check_output_parity (head level and per row), the counters, and, with the stage-2 test off,
    exact fp64 attention on the same blocks."""
    import torch
    mask_t = None if mask_np is None else torch.from_numpy(mask_np).to("cuda")
    O, stats = sp.sparge_attn(Q, K, V, mask_t, lam, causal=w.causal, return_stats=True)
    O, stats = cpu(O).astype(np.float64), cpu(stats)
    rows = np.arange(w.N)
    for h in (range(w.H) if heads is None else heads):
        q, k, v = x["q"][0, h], x["k"][0, h], x["v"][0, h]
        m = None if mask_np is None else mask_np[0, h]
        res = check_output_parity(so, O[0, h], q, k, v, m, f32(lam), w.causal, w.dtype, rows,
                                  label=f"{w.name} head {h} lambda {lam}")
        ref = res["ref"]
        if not np.isfinite(lam):
            e_exact = so.rel_l1(O[0, h], so.dense_attention(q, k, v, causal=w.causal, block_mask=m))
            print(f"    exact fp64 on the same blocks: {e_exact:.2e}; stats {stats[0, h].tolist()}", flush=True)
            assert e_exact <= REL_L1_EXACT
        assert stats[0, h, 0] == ref.qk_tiles
        assert stats[0, h, 2] == ref.valid_tiles and stats[0, h, 3] == ref.valid_groups
        # the stage-2 decision is taken in fp32 on the GPU: allow a few borderline groups
        assert abs(int(stats[0, h, 1]) - ref.pv_groups) <= max(2, ref.pv_groups // 500)
    return O, stats


@pytest.mark.parametrize("w", CASES, ids=IDS)
def test_attn_dense_switches(sp, w):
    """mask = all ones, lambda = -inf: quantized dense attention; also <= 3e-2 from exact fp64."""
    print(f"case {w.name}", flush=True)
    x, Q, K, V = gpu_inputs(w)
    check_attention(sp, w, x, Q, K, V, None, -math.inf)


@pytest.mark.parametrize("w", CASES, ids=IDS)
def test_attn_masked_with_lambda(sp, w):
    print(f"case {w.name}", flush=True)
    x, Q, K, V = gpu_inputs(w)
    masks = np.stack([so.predict(x["q"][0, h], x["k"][0, h], f32(w.tau), f32(w.theta), causal=w.causal).mask
                      for h in range(w.H)])[None]
    check_attention(sp, w, x, Q, K, V, masks, -math.inf)
    O, stats = check_attention(sp, w, x, Q, K, V, masks, w.lam)


@pytest.mark.parametrize("w", [CASES[0], CASES[2], CASES[5]], ids=[IDS[0], IDS[2], IDS[5]])
def test_forward_equals_the_three_calls(sp, w):
    import torch
    x, Q, K, V = gpu_inputs(w)
    O, mask, stats = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, causal=w.causal, return_mask=True,
                                       return_stats=True)
    mask2 = sp.sparge_predict(Q, K, w.tau, w.theta, causal=w.causal)
    assert torch.equal(mask, mask2)
    Qq, Kq, qs, ks, _ = sp.sparge_quantize(Q, K)
    O2, stats2 = sp.sparge_attn_quantized(Qq, Kq, qs, ks, V, mask2, w.lam, causal=w.causal, return_stats=True)
    assert torch.equal(O, O2) and torch.equal(stats, stats2)
    for h in range(w.H):
        res, pred = so.spargeattn(x["q"][0, h], x["k"][0, h], x["v"][0, h], f32(w.tau), f32(w.theta), f32(w.lam),
                                  causal=w.causal, quant=True, pv_dtype=w.dtype, ref_slack=REF_SLACK)
        if not pred.dont_care.any():
            assert so.rel_l1(cpu(O)[0, h].astype(np.float64), so.round16(res.O, w.dtype)) <= REL_L1_EMUL
            s = cpu(stats)[0, h]
            sparsity = 1.0 - 0.5 * (s[0] / s[2] + s[1] / s[3])
            assert abs(sparsity - res.sparsity) < 5e-3


def test_strided_bnhd_layout_and_determinism(sp):
    import torch
    w = small_workload("strided", N=600, d=64, dtype="bf16", H=3, seed=8)
    x, Q, K, V = gpu_inputs(w)
    def bnhd(t):
        return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)   # [B,H,N,d] view of [B,N,H,d] memory
    Qs, Ks, Vs = bnhd(Q), bnhd(K), bnhd(V)
    assert not Qs.is_contiguous()
    O1 = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam)
    O2 = sp.sparge_forward(Qs, Ks, Vs, w.tau, w.theta, w.lam)
    assert O2.stride() == Qs.stride()
    assert torch.equal(O1, O2)
    assert torch.equal(O1, sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam))


def test_fully_masked_row_gives_zeros(sp):
    import torch
    w = small_workload("masked", N=512, d=64, dtype="fp16", H=1, seed=9)
    x, Q, K, V = gpu_inputs(w)
    mask = torch.ones((1, 1, 4, 8), dtype=torch.uint8, device="cuda")
    mask[0, 0, 2] = 0
    O = cpu(sp.sparge_attn(Q, K, V, mask, -math.inf))
    assert np.all(O[0, 0, 256:384] == 0) and np.isfinite(O).all()
    assert np.abs(O[0, 0, :256]).sum() > 0


def test_per_head_hyper_parameters(sp):
    w = small_workload("perhead", N=1024, d=64, dtype="fp16", H=2, seed=10)
    x, Q, K, V = gpu_inputs(w)
    taus, thetas = [0.5, 0.95], [0.4, 0.7]
    mask = cpu(sp.sparge_predict(Q, K, taus, thetas))
    for h in range(2):
        pr = so.predict(x["q"][0, h], x["k"][0, h], f32(taus[h]), f32(thetas[h]))
        assert not ((mask[0, h] != pr.mask) & ~pr.dont_care).any()


def test_errors_are_raised_not_swallowed(sp):
    import torch
    w = small_workload("err", N=256, d=64, dtype="fp16", H=1, seed=11)
    x, Q, K, V = gpu_inputs(w)
    with pytest.raises(sp.SpargeError):
        sp.sparge_predict(Q, K, 1.5, 0.5)            # tau outside (0,1]
    with pytest.raises(sp.SpargeError):
        sp.sparge_attn(Q, K, V, None, 0.5)           # lambda must be negative
    with pytest.raises(sp.SpargeError):
        sp.sparge_attn(Q, K, V, None, -1.0, ws=torch.empty(256, dtype=torch.uint8, device="cuda"))  # ws too small
    with pytest.raises(sp.SpargeError):
        sp.sparge_quantize(Q.float(), K.float())     # unsupported dtype
    Q96 = torch.zeros((1, 1, 256, 96), dtype=torch.float16, device="cuda")
    with pytest.raises(sp.SpargeError):
        sp.sparge_quantize(Q96, Q96)


def test_image_config_two_heads(sp):
    """Config 2 (image-like, d=128 bf16) at its real N on two heads."""
    w = scaled(CONFIGS["image"], H=2)
    x, Q, K, V = gpu_inputs(w, heads=[0, 1])
    masks = []
    m_gpu = cpu(sp.sparge_predict(Q, K, w.tau, w.theta))
    for h in range(2):
        pr = so.predict(x["q"][0, h], x["k"][0, h], f32(w.tau), f32(w.theta))
        assert not ((m_gpu[0, h] != pr.mask) & ~pr.dont_care).any()
        masks.append(pr.mask)
    check_attention(sp, w, x, Q, K, V, np.stack(masks)[None], w.lam)


@pytest.mark.parametrize("variant", [{}, {"pv_fp8": True}, {"qk16": True}], ids=["int8_16bit", "fp8_pv", "qk16"])
def test_batch_of_two_equals_two_single_calls(sp, variant):
    """B = 2 (a batch stride next to the head stride): every (batch, head) is an independent problem, so the
    batched call must reproduce the two single calls bit for bit, mask, counters and all."""
    import torch
    wa = small_workload("batch_a", N=900, d=128, dtype="bf16", H=2, seed=14)
    wb = small_workload("batch_b", N=900, d=128, dtype="bf16", H=2, seed=15)
    _, Qa, Ka, Va = gpu_inputs(wa)
    _, Qb, Kb, Vb = gpu_inputs(wb)
    Q, K, V = (torch.cat(p, dim=0) for p in ((Qa, Qb), (Ka, Kb), (Va, Vb)))
    O, mask, stats = sp.sparge_forward(Q, K, V, wa.tau, wa.theta, wa.lam, return_mask=True, return_stats=True, **variant)
    for b, (q, k, v) in enumerate(((Qa, Ka, Va), (Qb, Kb, Vb))):
        o1, m1, s1 = sp.sparge_forward(q, k, v, wa.tau, wa.theta, wa.lam, return_mask=True, return_stats=True, **variant)
        assert torch.equal(O[b:b + 1], o1) and torch.equal(mask[b:b + 1], m1) and torch.equal(stats[b:b + 1], s1)
