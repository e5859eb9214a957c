"""GPU parity of the unquantized variant (the paper's "SpargeAttn+FA2", Sec. 4.3): the same two-stage
filter with the Q K^T product on the 16-bit tensors themselves.  Oracle: the loop of Alg. 1 with
quant=False (scores in fp64), P~ rounded to the tensors' type at the same point as the kernel.
Bars: relative L1 2e-3 against that oracle, 3e-2 against exact fp64 attention on the same blocks."""
import math

import numpy as np
import pytest

from oracle import sparge_oracle as so
from synth import CONFIGS
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
    small_workload("causal128", N=1100, d=128, dtype="fp16", causal=True, seed=6),
    small_workload("causal64", N=520, d=64, dtype="bf16", causal=True, seed=7),
]
IDS = [w.name for w in CASES]


def check(sp, w, x, Q, K, V, mask_np, lam):
    import torch
    mask_t = None if mask_np is None else torch.from_numpy(mask_np).to("cuda")
    O, stats = sp.sparge_attn(Q, K, V, mask_t, lam, causal=w.causal, return_stats=True, qk16=True)
    O, stats = cpu(O).astype(np.float64), cpu(stats)
    for h in range(w.H):
        q, k, v = x["q"][0, h], x["k"][0, h], x["v"][0, h]
        m = None if mask_np is None else mask_np[0, h]
        ref = so.sparse_attention(q, k, v, m, lam=f32(lam), causal=w.causal, quant=False, pv_dtype=w.dtype,
                                  ref_slack=REF_SLACK)
        e_emul = so.rel_l1(O[0, h], so.round16(ref.O, w.dtype))
        e_exact = so.rel_l1(O[0, h], so.dense_attention(q, k, v, causal=w.causal, block_mask=m))
        print(f"  head {h}: rel-L1 emul {e_emul:.2e} exact {e_exact:.2e} stats {stats[0, h].tolist()}", flush=True)
        assert e_emul <= REL_L1_EMUL
        if not np.isfinite(lam):
            assert e_exact <= REL_L1_EXACT
        # per head, row and element against the recurrence as printed and the loop in exact arithmetic
        check_output_parity(so, O[0, h], q, k, v, m, f32(lam), w.causal, w.dtype, np.arange(w.N), quant=False,
                            label=f"{w.name} head {h} lambda {lam}")
        assert stats[0, h, 0] == ref.qk_tiles
        assert stats[0, h, 2] == ref.valid_tiles and stats[0, h, 3] == ref.valid_groups
        assert abs(int(stats[0, h, 1]) - ref.pv_groups) <= max(2, ref.pv_groups // 500)


@pytest.mark.parametrize("w", CASES, ids=IDS)
def test_qk16_dense_switches(sp, w):
    print(f"case {w.name}", flush=True)
    x, Q, K, V = gpu_inputs(w)
    check(sp, w, x, Q, K, V, None, -math.inf)


@pytest.mark.parametrize("w", CASES, ids=IDS)
def test_qk16_masked_with_lambda(sp, w):
    print(f"case {w.name}", flush=True)
    x, Q, K, V = gpu_inputs(w)
    masks = np.stack([so.predict(x["q"][0, h], x["k"][0, h], f32(w.tau), f32(w.theta), causal=w.causal).mask
                      for h in range(w.H)])[None]
    check(sp, w, x, Q, K, V, masks, -math.inf)
    check(sp, w, x, Q, K, V, masks, w.lam)


def test_qk16_strided_layout_and_forward(sp):
    """[B,N,H,d] storage (token stride H*d): the K tiles are copied straight from the caller's tensor."""
    import torch
    w = small_workload("strided", N=900, d=128, dtype="bf16", H=3, seed=9)
    x, Q, K, V = gpu_inputs(w)
    Qs, Ks, Vs = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (Q, K, V))
    assert Qs.stride(2) == w.H * w.d
    O, mask, stats = sp.sparge_forward(Qs, Ks, Vs, w.tau, w.theta, w.lam, return_mask=True, return_stats=True, qk16=True)
    mask2 = sp.sparge_predict(Q, K, w.tau, w.theta)
    assert torch.equal(mask, mask2)
    O2, stats2 = sp.sparge_attn(Q, K, V, mask, w.lam, return_stats=True, qk16=True)
    assert torch.equal(O.contiguous(), O2) and torch.equal(stats, stats2)
    O8 = sp.sparge_attn(Q, K, V, mask, w.lam)                   # the INT8 product: close, not equal
    assert not torch.equal(O2, O8)
    assert so.rel_l1(cpu(O8).astype(np.float64), cpu(O2).astype(np.float64)) < REL_L1_EXACT


def test_qk16_unsupported_combinations_raise(sp):
    w = small_workload("e", N=256, d=64, dtype="fp16", H=1, seed=1)
    x, Q, K, V = gpu_inputs(w)
    with pytest.raises(sp.SpargeError):
        sp.sparge_attn(Q, K, V, None, -math.inf, qk16=True, pv_fp8=True)


def test_qk16_video_configuration_sampled_rows(sp):
    """The N = 17550 video configuration in full (48 heads, one sparge_forward call) with the 16-bit Q K^T
    product: same mask as the INT8 path, counters against the mask, and the output rows of five Q blocks of two
    heads against the oracle loop without quantization."""
    import os
    import torch
    from synth import make_workload
    w = CONFIGS["video"]
    x = make_workload(w, workers=min(16, os.cpu_count() or 1))
    Q, K, V = (to_torch(x[t], w.dtype) for t in "qkv")
    O, mask, stats = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, return_mask=True, return_stats=True, qk16=True)
    mask8 = sp.sparge_predict(Q, K, w.tau, w.theta)
    assert torch.equal(mask, mask8) and torch.isfinite(O.float()).all()
    mask_np, stats_np = cpu(mask), cpu(stats)
    assert (stats_np[0, :, 0] == mask_np[0].reshape(w.H, -1).sum(1)).all()
    Tm = so.nblocks(w.N, 128)
    blocks = sorted(set(np.linspace(0, Tm - 1, 5).astype(int).tolist()))
    rows = np.concatenate([np.arange(128 * i, min(128 * (i + 1), w.N)) for i in blocks])
    for h in (0, w.H - 1):
        got = O[0, h].float().cpu().numpy().astype(np.float64)[rows]
        check_output_parity(so, got, x["q"][0, h], x["k"][0, h], x["v"][0, h], mask_np[0, h], f32(w.lam), False,
                            w.dtype, rows, q_blocks=blocks, quant=False, label=f"video, 16-bit Q K^T, head {h}")
