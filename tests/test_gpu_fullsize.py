"""Parity at the full benchmark sizes, in the launch configuration bench.py times (all heads, one
sparge_forward call).  The oracle cannot run a whole configuration, so it checks what it can compute
one by one: for two heads the INT8 tensors, scales, K mean and block mask in full, and the output
rows of a few evenly spaced Q blocks (first, ragged last, middle); for every head the properties that
hold at any size (counters against the mask and against closed forms, finite output, no dead rows).
"""
import math
import os

import numpy as np
import pytest

from oracle import sparge_oracle as so
from synth import CONFIGS, make_workload
from tests.helpers import REF_SLACK, check_output_parity, f32, to_torch

pytestmark = pytest.mark.gpu

CHECK_HEADS = 2
Q_BLOCKS_PER_HEAD = 5


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available()
    import paper_2502_18137_amd as sp
    sp.load_library()
    return sp


def closed_form_valid(N, causal):
    Tm, Tn = so.nblocks(N, 128), so.nblocks(N, 64)
    tiles = groups = 0
    for i in range(Tm):
        jmax = min(Tn, (i * 128 + 127) // 64 + 1) if causal else Tn
        tiles += jmax
        rows = min(128, N - 128 * i)
        for g0 in range(0, rows, 32):
            last = i * 128 + min(g0 + 32, rows) - 1
            groups += min(jmax, last // 64 + 1) if causal else jmax
    return tiles, groups


@pytest.mark.parametrize("name", ["video", "language", "longvideo"])
def test_full_configuration(sp, name):
    import torch
    w = CONFIGS[name]
    print(f"generating {name}: H={w.H} N={w.N} d={w.d}", flush=True)
    x = make_workload(w, workers=min(16, os.cpu_count() or 1))
    Q, K, V = (to_torch(x[t], w.dtype) for t in "qkv")
    print("running sparge_forward", flush=True)
    O, mask, stats = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, causal=w.causal, return_mask=True,
                                       return_stats=True)
    Qq, Kq, qs, ks, km = sp.sparge_quantize(Q, K)
    torch.cuda.synchronize()
    mask_np, stats_np = mask.cpu().numpy(), stats.cpu().numpy()

    # ---- properties for every head -----------------------------------------------------------
    assert torch.isfinite(O.float()).all()
    tiles, groups = closed_form_valid(w.N, w.causal)
    assert (stats_np[0, :, 2] == tiles).all() and (stats_np[0, :, 3] == groups).all()
    assert (stats_np[0, :, 0] == mask_np[0].reshape(w.H, -1).sum(1)).all()       # QK^T tiles = kept blocks
    assert (stats_np[0, :, 1] <= 4 * stats_np[0, :, 0]).all()
    assert (mask_np[0].sum(-1) >= 1).all()                                       # no Q block without keys
    if w.causal:
        Tm, Tn = mask_np.shape[2:]
        future = np.triu(np.ones((Tm, Tn), dtype=bool), k=0)
        for i in range(Tm):
            future[i] = np.arange(Tn) * 64 > i * 128 + 127
        assert not mask_np[0][:, future].any()
    sparsity = 1.0 - 0.5 * (stats_np[0, :, 0].sum() / stats_np[0, :, 2].sum()
                            + stats_np[0, :, 1].sum() / stats_np[0, :, 3].sum())
    print(f"{name}: sparsity {sparsity:.3f}", flush=True)

    # ---- element-wise checks on a few heads ----------------------------------------------------
    Tm = so.nblocks(w.N, 128)
    blocks = sorted(set(np.linspace(0, Tm - 1, Q_BLOCKS_PER_HEAD).astype(int).tolist()))
    for h in (0, w.H - 1)[:CHECK_HEADS]:
        q, k, v = x["q"][0, h], x["k"][0, h], x["v"][0, h]
        oq, odq = so.quantize_q(q)
        ok, odk, omean = so.quantize_k(k)
        assert (Qq[0, h].cpu().numpy() == oq).all() and (Kq[0, h].cpu().numpy() == ok).all()
        assert (qs[0, h].cpu().numpy().view(np.uint32) == odq.view(np.uint32)).all()
        assert (ks[0, h].cpu().numpy().view(np.uint32) == odk.view(np.uint32)).all()
        assert (km[0, h].cpu().numpy().view(np.uint32) == omean.view(np.uint32)).all()
        qe, q_tie = so.quantize_exact(np.asarray(q, dtype=np.float32), so.BQ)     # exact rounding away from ties
        ke, k_tie = so.quantize_exact(np.asarray(k, dtype=np.float32) - omean[None, :], so.BK)
        assert ((oq == qe) | q_tie).all() and ((ok == ke) | k_tie).all()
        print(f"  head {h}: quotients within 2^-15 of a tie: Q {int(q_tie.sum())}, K {int(k_tie.sum())} of {q_tie.size}",
              flush=True)
        pred = so.predict(q, k, f32(w.tau), f32(w.theta), causal=w.causal)
        bad = (mask_np[0, h] != pred.mask) & ~pred.dont_care
        assert not bad.any(), (h, np.argwhere(bad)[:5])
        assert pred.dont_care.mean() < 0.01
        # output rows of the sampled Q blocks, with the GPU's own mask so that exempt entries cannot matter:
        # head-level and per-row bars against the three evaluations of the loop (tests/helpers.py)
        rows = np.concatenate([np.arange(128 * i, min(128 * (i + 1), w.N)) for i in blocks])
        got = O[0, h].float().cpu().numpy().astype(np.float64)[rows]
        check_output_parity(so, got, q, k, v, mask_np[0, h], f32(w.lam), w.causal, w.dtype, rows, q_blocks=blocks,
                            label=f"{name} head {h}, {len(blocks)} Q blocks, dont-care {int(pred.dont_care.sum())}")

    # ---- the FP8 (E4M3) P~V product on the same inputs: same mask and tile counters; sampled rows of one head
    O8, mask8, stats8 = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, causal=w.causal, return_mask=True,
                                          return_stats=True, pv_fp8=True)
    torch.cuda.synchronize()
    assert torch.equal(mask8, mask) and torch.isfinite(O8.float()).all()
    s8 = stats8.cpu().numpy()
    assert (s8[0, :, [0, 2, 3]] == stats_np[0, :, [0, 2, 3]]).all()
    h = w.H - 1
    ref8 = so.sparse_attention(x["q"][0, h], x["k"][0, h], x["v"][0, h], mask_np[0, h], lam=f32(w.lam),
                               causal=w.causal, quant=True, pv_dtype="fp8e4m3", q_blocks=blocks,
                               ref_slack=sp.REF_SLACK_LOG2_FP8 * math.log(2.0))
    got8 = O8[0, h].float().cpu().numpy().astype(np.float64)[rows]
    err8 = so.rel_l1(got8, so.round16(ref8.O[rows], w.dtype))
    print(f"  head {h}, FP8 P~V: rel-L1 vs oracle {err8:.2e}, vs the 16-bit product {so.rel_l1(got8, got):.2e}",
          flush=True)
    assert err8 <= 2e-3


@pytest.mark.parametrize("causal,dtype,d,pv_fp8,qk16", [(False, "bf16", 128, False, False), (True, "fp16", 64, False, False),
                                                        (False, "fp16", 128, True, False), (True, "bf16", 64, True, False),
                                                        (True, "bf16", 128, False, True), (False, "fp16", 64, False, True)])
def test_long_list_two_stage_kernel(sp, causal, dtype, d, pv_fp8, qk16):
    """T_n > 1024 selects the kernel variants with two LDS stages and the long tile list (2048 entries for the
    16-bit Q K^T product, whose K tiles are twice as large, 4096 otherwise): N = 70 000
    (ragged: last Q block 112 rows, last K block 48 keys), one head, a random block mask with a forced
    first column (and diagonal when causal); the output rows of a few Q blocks against the oracle loop."""
    import torch
    from tests.helpers import small_workload
    N = 70000
    w = small_workload(name="long", N=N, d=d, dtype=dtype, H=1, causal=causal, lam=-6.0, seed=11, segment=512)
    x = make_workload(w)
    Q, K, V = (to_torch(x[t], w.dtype) for t in "qkv")
    Tm, Tn = so.nblocks(N, 128), so.nblocks(N, 64)
    assert Tn > 1024
    rng = np.random.default_rng(5)
    mask_np = (rng.random((1, 1, Tm, Tn)) < 0.3).astype(np.uint8)
    mask_np[..., 0] = 1
    if causal:
        mask_np[0, 0, np.arange(Tm), np.minimum(2 * np.arange(Tm), Tn - 1)] = 1
    mask_np[0, 0, -1, -1] = 1   # the partial last key block is used by the ragged last Q block
    mask_t = torch.from_numpy(mask_np).to("cuda")
    O, stats = sp.sparge_attn(Q, K, V, mask_t, w.lam, causal=causal, return_stats=True, pv_fp8=pv_fp8, qk16=qk16)
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all()
    q, k, v = x["q"][0, 0], x["k"][0, 0], x["v"][0, 0]
    blocks = [0, 1, Tm // 3, Tm - 2, Tm - 1]
    ref = so.sparse_attention(q, k, v, mask_np[0, 0], lam=f32(w.lam), causal=causal, quant=not qk16,
                              pv_dtype="fp8e4m3" if pv_fp8 else dtype, q_blocks=blocks,
                              ref_slack=sp.REF_SLACK_LOG2_FP8 * math.log(2.0) if pv_fp8 else REF_SLACK)
    assert ref.zero_rows == 0
    rows = np.concatenate([np.arange(128 * i, min(128 * (i + 1), N)) for i in blocks])
    got = O[0, 0].float().cpu().numpy().astype(np.float64)[rows]
    err = so.rel_l1(got, so.round16(ref.O[rows], dtype))
    print(f"  long list causal={causal} fp8={pv_fp8} qk16={qk16}: rel-L1 vs oracle {err:.2e}", flush=True)
    assert err <= 2e-3
    if not pv_fp8:
        check_output_parity(so, got, q, k, v, mask_np[0, 0], f32(w.lam), causal, dtype, rows, q_blocks=blocks,
                            label=f"long list causal={causal} qk16={qk16}", quant=not qk16)
    tiles, groups = closed_form_valid(N, causal)
    s = stats.cpu().numpy()[0, 0]
    assert s[2] == tiles and s[3] == groups
    visible = mask_np[0, 0].astype(bool)
    if causal:
        for i in range(Tm):
            visible[i, np.arange(Tn) * 64 > i * 128 + 127] = False
    assert s[0] == visible.sum()


@pytest.mark.parametrize("causal", [False, True])
def test_predict_long_rows(sp, causal):
    """T_n in (1024, 2048]: the widest per-wave TopCdf variant (32 ranks per lane).  N = 70 000, one head."""
    from tests.helpers import small_workload
    w = small_workload(name="longpred", N=70000, d=64, dtype="bf16", H=1, causal=causal, seed=21, segment=448, noise=0.4)
    x = make_workload(w)
    Q, K = (to_torch(x[t], w.dtype) for t in "qk")
    for tau, theta in ((0.9, 0.5), (0.6, -1.0)):
        mask = sp.sparge_predict(Q, K, tau, theta, causal=causal).cpu().numpy()
        pr = so.predict(x["q"][0, 0], x["k"][0, 0], f32(tau), f32(theta), causal=causal)
        bad = (mask[0, 0] != pr.mask) & ~pr.dont_care
        print(f"  causal={causal} tau={tau} theta={theta}: kept {mask.mean():.3f}, dont-care {int(pr.dont_care.sum())}", flush=True)
        assert not bad.any(), np.argwhere(bad)[:5]
        assert pr.dont_care.mean() < 0.01
