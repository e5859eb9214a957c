"""Degenerate inputs and the longest rows the library accepts, through the C ABI: an all-zero Q block and an
all-zero V channel, K constant over a head (closed forms for the mask and the output), K entries spread over
2^30 in magnitude (the exactness of the K mean), and T_n > 2048 (TopCdf sorted in LDS, attention lists built in
three chunks)."""
import math

import numpy as np
import pytest

from oracle import sparge_oracle as so
from synth import make_workload
from tests.helpers import check_output_parity, f32, gpu_inputs, small_workload, to_torch, unit_roundoff

pytestmark = pytest.mark.gpu


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


@pytest.mark.parametrize("d,dtype,pv_fp8", [(64, "fp16", False), (128, "bf16", False), (128, "bf16", True)])
def test_zero_q_block_and_zero_v_channel(sp, d, dtype, pv_fp8):
    """Q block 1 is all zeros: amax = 0, so delta_Q = 0 and Q-hat = 0 there, every score of the block is 0 and
    its rows average V over the kept keys; the block has no direction, its self-similarity is 0, and the
    judge keeps its whole mask row.  Channel 3 of V is all zeros: that output channel is exactly 0."""
    w = small_workload("zeroq", N=600, d=d, dtype=dtype, H=2, seed=31, lam=-5.0)
    x = make_workload(w)
    x["q"][0, :, 128:256, :] = 0.0
    x["v"][0, :, :, 3] = 0.0
    Q, K, V = (to_torch(x[t], dtype) for t in "qkv")
    Qq, Kq, qs, ks, km = (cpu(t) for t in sp.sparge_quantize(Q, K))
    O, mask, stats = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, return_mask=True, return_stats=True, pv_fp8=pv_fp8)
    O, mask = cpu(O).astype(np.float64), cpu(mask)
    assert np.isfinite(O).all()
    assert (O[0, :, :, 3] == 0).all()
    for h in range(w.H):
        q, k, v = x["q"][0, h], x["k"][0, h], x["v"][0, h]
        oq, odq = so.quantize_q(q)
        assert odq[1] == 0 and qs[0, h, 1] == 0 and not Qq[0, h, 128:256].any() and (Qq[0, h] == oq).all()
        pr = so.predict(q, k, f32(w.tau), f32(w.theta))
        assert pr.sim_q[1] == 0 and mask[0, h, 1].all()
        assert not ((mask[0, h] != pr.mask) & ~pr.dont_care).any()
        # rows of the zero block: the plain mean of V (every key kept, all weights equal)
        # (P~ = 1 exactly: what remains is the fp32 accumulation and the final rounding; FP8: V-hat's rounding)
        mean_v, weight = v.mean(axis=0)[None, :], np.abs(v).mean(axis=0)[None, :]
        tol = 2.0 ** -4 * weight if pv_fp8 else 1.01 * (unit_roundoff(dtype) * np.abs(mean_v) + 1e-4 * weight)
        assert (np.abs(O[0, h, 128:256] - mean_v) <= tol).all()
        if not pv_fp8:
            check_output_parity(so, O[0, h], q, k, v, mask[0, h], f32(w.lam), False, dtype, np.arange(w.N),
                                label=f"zero Q block, head {h}")


@pytest.mark.parametrize("d,dtype,causal", [(64, "bf16", False), (128, "fp16", False), (128, "bf16", True)])
def test_constant_k_gives_the_mean_of_v(sp, d, dtype, causal):
    """Every key equals one vector c: the K mean is c exactly, K - mean = 0, every delta_K = 0 and K-hat = 0,
    all scores are equal, and with every block kept a row's output is the mean of the V rows it may see
    (all of them; causally, those up to its own position).  In the predictor every K block has
    self-similarity 1 and the same pooled vector, so a selective mask row is a uniform P-hat: TopCdf keeps the
    ceil(tau * n) lowest indices of the n visible blocks."""
    import torch
    N, H = 1000, 2
    w = small_workload("constk", N=N, d=d, dtype=dtype, H=H, seed=33, causal=causal)
    x = make_workload(w)
    c = so.round16(np.linspace(-1.5, 2.0, d), dtype)
    x["k"][0, :, :, :] = c[None, None, :]
    Q, K, V = (to_torch(x[t], dtype) for t in "qkv")
    Qq, Kq, qs, ks, km = (cpu(t) for t in sp.sparge_quantize(Q, K))
    assert (km[0] == c[None, :].astype(np.float32)).all() and not Kq.any() and not ks.any()
    O = cpu(sp.sparge_attn(Q, K, V, None, -math.inf, causal=causal)).astype(np.float64)
    u = unit_roundoff(dtype)
    for h in range(H):
        v = x["v"][0, h]
        csum, cabs = np.cumsum(v, axis=0), np.cumsum(np.abs(v), axis=0)
        n = np.arange(1, N + 1)[:, None]
        expect = csum / n if causal else np.broadcast_to(v.mean(axis=0), v.shape)
        weight = cabs / n if causal else np.broadcast_to(np.abs(v).mean(axis=0), v.shape)
        # P~ = 1 exactly for every visible key, so only the fp32 accumulation and the final rounding remain
        assert (np.abs(O[0, h] - expect) <= 1.01 * (u * np.abs(expect) + 1e-4 * weight)).all()
    # the predictor on the first 960 tokens (whole key blocks only: block sums 64 c scale exactly, so all
    # compressed logits of a row are the same number and ties fall to the lowest indices)
    tau, theta, N = 0.37, 0.5, 960
    mask, sq, sk = sp.sparge_predict(Q[:, :, :N].contiguous(), K[:, :, :N].contiguous(), tau, theta, causal=causal,
                                     return_sims=True)
    mask, sq, sk = cpu(mask), cpu(sq), cpu(sk)
    np.testing.assert_allclose(sk, 1.0, atol=1e-12)
    Tm, Tn = so.nblocks(N, 128), so.nblocks(N, 64)
    for h in range(H):
        for i in range(Tm):
            nvis = min(Tn, (i * 128 + 127) // 64 + 1) if causal else Tn
            if sq[0, h, i] < theta:
                expect = np.arange(Tn) < nvis
            else:
                keep = math.ceil(f32(tau) * nvis - 1e-9)
                assert abs(f32(tau) * nvis - round(f32(tau) * nvis)) > 1e-3
                expect = np.arange(Tn) < keep
                if causal:
                    expect = expect | (np.arange(Tn) == 2 * i)
            assert (mask[0, h, i].astype(bool) == expect).all(), (h, i)


def test_k_of_wide_dynamic_range(sp):
    """K entries (bf16) spread over 2^30 in magnitude.  While (exponent spread + 8 significand bits + log2 N) stays
    below 53 bits every fp64 partial sum is exact, whatever its order, and the K mean, K-hat and delta_K must
    equal the oracle's (exactly rounded sum) bit for bit; that is the case for N = 700.  At N = 4096 with a
    spread of 2^40 the budget is exceeded: the kernel's fixed-order fp64 sum may differ from the exactly
    rounded one in its last bit, which moves the fp32 mean only if the sum sits within 2^-29 (relative) of an
    fp32 rounding boundary -- the test then asserts the mean to one fp32 ulp and K-hat against the oracle's
    quantizer applied to the kernel's own mean."""
    r = np.random.default_rng(35)
    for N, spread, exact in ((700, 30, True), (4096, 40, False)):
        d, H = 64, 2
        k = r.choice([-1.0, 1.0], size=(1, H, N, d)) * (1.0 + r.random((1, H, N, d))) * \
            np.exp2(r.integers(-spread // 2, spread // 2, size=(1, H, N, d)))     # |k| in [2^-s/2, 2^s/2)
        q = r.standard_normal((1, H, N, d))
        Q, K = to_torch(q, "bf16"), to_torch(k, "bf16")
        kb = np.asarray(K.float().cpu(), dtype=np.float64)
        assert np.log2(np.abs(kb).max() / np.abs(kb).min()) >= spread - 1
        Qq, Kq, qs, ks, km = (cpu(t) for t in sp.sparge_quantize(Q, K))
        _, sq, sk = sp.sparge_predict(Q, K, 0.9, 0.5, return_sims=True)
        for h in range(H):
            okq, odk, omean = so.quantize_k(kb[0, h])
            if exact:
                assert (km[0, h].view(np.uint32) == omean.view(np.uint32)).all()
                assert (Kq[0, h] == okq).all() and (ks[0, h].view(np.uint32) == odk.view(np.uint32)).all()
            else:
                ulp = np.spacing(np.abs(omean))
                assert (np.abs(km[0, h] - omean) <= ulp).all()
                kq2, dk2 = so._quant_blocks(kb[0, h].astype(np.float32) - km[0, h][None, :], so.BK)
                assert (Kq[0, h] == kq2).all() and (ks[0, h].view(np.uint32) == dk2.view(np.uint32)).all()
            np.testing.assert_allclose(cpu(sk)[0, h], so.cossim_blocks(kb[0, h], so.BK), atol=1e-12)
        same = sum(int((km[0, h].view(np.uint32) == so.k_mean(kb[0, h]).view(np.uint32)).sum()) for h in range(H))
        print(f"  N={N}, spread 2^{spread}: K mean bit-exact on {same} of {H * d} channels", flush=True)


@pytest.mark.parametrize("causal", [False, True])
def test_rows_longer_than_2048_blocks(sp, causal):
    """N = 140 000 (T_n = 2188, T_m = 1094; last Q block 96 rows, last K block 32 keys), one head, d = 64: the
    predictor's LDS-sorted TopCdf against the oracle, then the whole path (lists of more than 2048 tiles are
    built in three chunks) on the output rows of five Q blocks."""
    N = 140000
    w = small_workload("verylong", N=N, d=64, dtype="bf16", H=1, causal=causal, seed=41, segment=832, noise=0.4,
                       tau=0.8, theta=0.45, lam=-7.0)
    x = make_workload(w)
    Tm = so.nblocks(N, 128)
    # a Q block without a common direction is a fix block: its row keeps every visible key block (2184 of them)
    x["q"][0, 0, 128 * (Tm - 3):128 * (Tm - 2)] = so.round16(np.random.default_rng(43).standard_normal((128, 64)), w.dtype)
    Q, K, V = (to_torch(x[t], w.dtype) for t in "qkv")
    q, k, v = x["q"][0, 0], x["k"][0, 0], x["v"][0, 0]
    print("  oracle predictor ...", flush=True)
    pr = so.predict(q, k, f32(w.tau), f32(w.theta), causal=causal)
    mask, sq, sk = sp.sparge_predict(Q, K, w.tau, w.theta, causal=causal, return_sims=True)
    mask = cpu(mask)
    np.testing.assert_allclose(cpu(sq)[0, 0], pr.sim_q, atol=1e-12)
    np.testing.assert_allclose(cpu(sk)[0, 0], pr.sim_k, atol=1e-12)
    bad = (mask[0, 0] != pr.mask) & ~pr.dont_care
    print(f"  causal={causal}: kept {mask.mean():.3f}, dont-care {int(pr.dont_care.sum())}, "
          f"longest row {int(mask[0, 0].sum(1).max())} blocks", flush=True)
    assert not bad.any(), np.argwhere(bad)[:5]
    assert pr.dont_care.mean() < 0.01
    assert mask[0, 0, Tm - 3].sum() > 2048         # a list that spans three chunks of 1024
    O, mask2, stats = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, causal=causal, return_mask=True,
                                        return_stats=True)
    assert (cpu(mask2) == mask).all()
    O = cpu(O).astype(np.float64)
    assert np.isfinite(O).all()
    blocks = [0, Tm // 2, Tm - 3, Tm - 2, Tm - 1]
    rows = np.concatenate([np.arange(128 * i, min(128 * (i + 1), N)) for i in blocks])
    check_output_parity(so, O[0, 0][rows], q, k, v, mask[0, 0], f32(w.lam), causal, w.dtype, rows, q_blocks=blocks,
                        label=f"N={N} causal={causal}")
    s = cpu(stats)[0, 0]
    visible = mask[0, 0].astype(bool)
    assert s[0] == visible.sum()


def test_longest_rows_the_library_takes(sp):
    """T_n = SPARGE_MAX_TN = 4096 (N = 262 144, T_m = 2048), one head, d = 64, fp16: the predictor against the
    oracle and the output rows of four Q blocks, one of them a fix block whose list holds all 4096 key blocks
    (four chunks of the list build, the whole list capacity of the kernel)."""
    N = 64 * 4096
    w = small_workload("maxlen", N=N, d=64, dtype="fp16", H=1, seed=47, segment=1536, noise=0.35,
                       tau=0.7, theta=0.45, lam=-6.0)
    x = make_workload(w)
    Tm = so.nblocks(N, 128)
    x["q"][0, 0, 128 * 1000:128 * 1001] = so.round16(np.random.default_rng(48).standard_normal((128, 64)), w.dtype)
    Q, K, V = (to_torch(x[t], w.dtype) for t in "qkv")
    q, k, v = x["q"][0, 0], x["k"][0, 0], x["v"][0, 0]
    print("  oracle predictor ...", flush=True)
    pr = so.predict(q, k, f32(w.tau), f32(w.theta))
    O, mask, stats = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, return_mask=True, return_stats=True)
    mask, O = cpu(mask), cpu(O).astype(np.float64)
    bad = (mask[0, 0] != pr.mask) & ~pr.dont_care
    print(f"  kept {mask.mean():.3f}, dont-care {int(pr.dont_care.sum())}", flush=True)
    assert not bad.any(), np.argwhere(bad)[:5]
    assert pr.dont_care.mean() < 0.01 and mask[0, 0, 1000].sum() == 4096
    assert np.isfinite(O).all() and cpu(stats)[0, 0, 0] == mask.sum()
    blocks = [0, 1000, Tm // 2 + 1, Tm - 1]
    rows = np.concatenate([np.arange(128 * i, 128 * (i + 1)) for i in blocks])
    check_output_parity(so, O[0, 0][rows], q, k, v, mask[0, 0], f32(w.lam), False, w.dtype, rows, q_blocks=blocks,
                        label=f"N={N}")
