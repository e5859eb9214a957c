"""GPU parity of the FP8 (E4M3) P~V product against the CPU oracle.

Bars: the E4M3 tiles of V and the channel scales bit-exact; outputs within relative L1 2e-3 of the
oracle that emulates the same quantization and rounding points (pv_dtype="fp8e4m3", the same lag of
the reference maximum), and within one unit roundoff of E4M3, u = 2^-4 = 6.25e-2, of exact fp64 attention on
the same blocks: P~ and V-hat are each rounded once to 4 significant bits (relative error of rms 0.4247 u for a
log-uniform significand), which for outputs that are random combinations of V rows gives a relative L1
distance of sqrt(2) * 0.4247 u = 0.60 u = 3.75e-2 (measured 3.5e-2 ... 4.2e-2); the bar leaves the same
room as the 16-bit product's bars in tests/helpers.py (the benchmark spec's 3e-2 belongs to the 16-bit product).
"""
import math

import numpy as np
import pytest

from oracle import sparge_oracle as so
from synth import CONFIGS
from tests.helpers import f32, gpu_inputs, small_workload

pytestmark = pytest.mark.gpu

REL_L1_EMUL = 2e-3
REL_L1_EXACT_FP8 = 2.0 ** -4


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
    small_workload("causal128", N=1100, d=128, dtype="bf16", causal=True, seed=6),
    small_workload("causal64", N=520, d=64, dtype="fp16", causal=True, seed=7),
]
IDS = [w.name for w in CASES]


def slack(sp):
    return sp.REF_SLACK_LOG2_FP8 * math.log(2.0)


@pytest.mark.parametrize("w", CASES, ids=IDS)
def test_v_tiles_fp8_bit_exact(sp, w):
    print(f"case {w.name}", flush=True)
    x, Q, K, V = gpu_inputs(w)
    buf = cpu(sp.sparge_v_tiles(V, pv_fp8=True))
    Tn = (w.N + 63) // 64
    n_tiles = w.H * Tn * w.d * 64
    off_scale = (n_tiles + 255) // 256 * 256
    tiles = buf[:n_tiles].reshape(w.H, Tn, w.d // 32, 2, 64, 16)
    scales = buf[off_scale:off_scale + 4 * w.H * w.d].view(np.float32).reshape(w.H, w.d)
    for h in range(w.H):
        v = x["v"][0, h].astype(np.float64)
        Vq, delta = so.quantize_v_fp8(v)
        np.testing.assert_array_equal(scales[h], delta)
        codes = np.zeros((Tn * 64, w.d), dtype=np.uint8)
        codes[:w.N] = so.encode_e4m3(Vq)
        codes = codes.reshape(Tn, 64, w.d)
        # (dt, h2, lane = c%32 + 32 g, byte b) holds channel c of key 32 h2 + 8 (b/4) + 4 g + b%4
        dt, h2, lane, b = np.meshgrid(np.arange(w.d // 32), np.arange(2), np.arange(64), np.arange(16), indexing="ij")
        key = 32 * h2 + 8 * (b // 4) + 4 * (lane // 32) + b % 4
        c = 32 * dt + lane % 32
        want = codes[:, key, c]
        np.testing.assert_array_equal(tiles[h], want)


def check(sp, w, x, Q, K, V, mask_np, lam):
    import torch
    mask_t = None if mask_np is None else torch.from_numpy(mask_np).to("cuda")
    O, stats = sp.sparge_attn(Q, K, V, mask_t, lam, causal=w.causal, return_stats=True, pv_fp8=True)
    O, stats = cpu(O).astype(np.float64), cpu(stats)
    for h in range(w.H):
        q, k, v = x["q"][0, h], x["k"][0, h], x["v"][0, h]
        m = None if mask_np is None else mask_np[0, h]
        ref = so.sparse_attention(q, k, v, m, lam=f32(lam), causal=w.causal, quant=True, pv_dtype="fp8e4m3",
                                  ref_slack=slack(sp))
        e_emul = so.rel_l1(O[0, h], so.round16(ref.O, w.dtype))
        exact = so.dense_attention(q, k, v, causal=w.causal, block_mask=m)
        e_exact = so.rel_l1(O[0, h], exact)
        print(f"  head {h}: rel-L1 emul {e_emul:.2e} exact {e_exact:.2e} stats {stats[0, h].tolist()}", flush=True)
        assert e_emul <= REL_L1_EMUL
        if not np.isfinite(lam):
            assert e_exact <= REL_L1_EXACT_FP8
        assert stats[0, h, 0] == ref.qk_tiles
        assert abs(int(stats[0, h, 1]) - ref.pv_groups) <= max(2, ref.pv_groups // 500)


@pytest.mark.parametrize("w", CASES, ids=IDS)
def test_attn_fp8_dense_switches(sp, w):
    print(f"case {w.name}", flush=True)
    x, Q, K, V = gpu_inputs(w)
    check(sp, w, x, Q, K, V, None, -math.inf)


@pytest.mark.parametrize("w", CASES, ids=IDS)
def test_attn_fp8_masked_with_lambda(sp, w):
    print(f"case {w.name}", flush=True)
    x, Q, K, V = gpu_inputs(w)
    masks = np.stack([so.predict(x["q"][0, h], x["k"][0, h], f32(w.tau), f32(w.theta), causal=w.causal).mask
                      for h in range(w.H)])[None]
    check(sp, w, x, Q, K, V, masks, -math.inf)
    check(sp, w, x, Q, K, V, masks, w.lam)


def test_forward_fp8_equals_the_three_calls(sp):
    import torch
    w = CASES[2]
    x, Q, K, V = gpu_inputs(w)
    O, mask, stats = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, causal=w.causal, return_mask=True,
                                       return_stats=True, pv_fp8=True)
    Qq, Kq, qs, ks, _ = sp.sparge_quantize(Q, K)
    O2, stats2 = sp.sparge_attn_quantized(Qq, Kq, qs, ks, V, mask, w.lam, causal=w.causal, return_stats=True,
                                          pv_fp8=True)
    vt = sp.sparge_v_tiles(V, pv_fp8=True)
    O3 = sp.sparge_attn_tiled(Qq, Kq, qs, ks, vt, V, mask, w.lam, causal=w.causal, pv_fp8=True)
    assert torch.equal(O, O2) and torch.equal(stats, stats2) and torch.equal(O, O3)
    O16 = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, causal=w.causal)
    assert not torch.equal(O, O16)          # the 16-bit product is a different computation ...
    assert so.rel_l1(cpu(O).astype(np.float64), cpu(O16).astype(np.float64)) < REL_L1_EXACT_FP8  # ... of the same thing
