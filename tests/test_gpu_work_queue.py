"""Work distribution of the attention kernel: resident workgroups take (head, Q block) items from one counter per
XCD range and move on to the other ranges when their own is empty.  Cases where that matters: more items than
resident workgroups, a head count that is no multiple of 8 (ranges cut heads), fewer items than ranges, and
heads of very different density (one range holds almost all the work, the others finish and take from it).
Every output row is checked against the oracle loop on the same mask: an item computed twice, skipped, or
computed with another item's lists would show."""
import math

import numpy as np
import pytest

from oracle import sparge_oracle as so
from tests.helpers import REF_SLACK, check_output_parity, f32, gpu_inputs, small_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2502_18137_amd as sp
    sp.load_library()
    return sp


@pytest.mark.parametrize("H,N,d,causal,dense_heads", [
    (9, 8192, 64, False, (0,)),        # 576 items > 512 resident workgroups; ranges cut heads; head 0 dense
    (16, 4224, 128, False, (3, 4)),    # 528 items; two dense heads in one range
    (3, 300, 64, True, (1,)),          # 9 items: fewer than 8 ranges of 2
    (24, 2944, 128, True, (23,)),      # 552 items, causal, the last range holds the dense head
    (7, 1700, 64, True, (3,)),         # 98 items, causal: ranges of 13 items against heads of 14 Q blocks (two passes per range)
])
def test_unbalanced_heads(sp, H, N, d, causal, dense_heads):
    import torch
    w = small_workload(f"wq{H}_{N}", N=N, d=d, dtype="bf16", H=H, causal=causal, seed=77, noise=1.0, segment=160)
    x, Q, K, V = gpu_inputs(w)
    Tm, Tn = so.nblocks(N, 128), so.nblocks(N, 64)
    r = np.random.default_rng(5)
    mask = (r.random((1, H, Tm, Tn)) < 0.04).astype(np.uint8)
    for h in dense_heads:
        mask[0, h] = 1
    mask[..., 0] = 1
    if causal:
        mask[0, :, np.arange(Tm), np.minimum(2 * np.arange(Tm), Tn - 1)] = 1
    lam = -6.0
    m_gpu = torch.from_numpy(mask).to("cuda")
    O, stats = sp.sparge_attn(Q, K, V, m_gpu, lam, causal=causal, return_stats=True)
    O2 = sp.sparge_attn(Q, K, V, m_gpu, lam, causal=causal)          # a second launch: another counter set
    assert torch.equal(O, O2)
    O = O.float().cpu().numpy().astype(np.float64)[0]
    stats = stats.cpu().numpy()[0]
    assert np.isfinite(O).all()
    # all rows of a dense head, a sparse head next to it and the last head; a few Q blocks of every other head
    full = sorted(set(dense_heads) | {(dense_heads[0] + 1) % H, H - 1})
    blocks = sorted({0, Tm // 2, Tm - 1})
    for h in range(H):
        qb = None if h in full and Tm <= 40 else blocks
        ref = so.sparse_attention(x["q"][0, h], x["k"][0, h], x["v"][0, h], mask[0, h], lam=f32(lam), causal=causal,
                                  quant=True, pv_dtype="bf16", ref_slack=REF_SLACK, q_blocks=qb)
        rows = np.arange(N) if qb is None else np.concatenate([np.arange(128 * i, min(128 * (i + 1), N)) for i in qb])
        err = so.rel_l1(O[h][rows], so.round16(ref.O[rows], "bf16"))
        assert err <= 2e-3, (h, err)
        if h in full:
            check_output_parity(so, O[h][rows], x["q"][0, h], x["k"][0, h], x["v"][0, h], mask[0, h], f32(lam), causal,
                                "bf16", rows, q_blocks=qb, label=f"H={H} N={N} head {h}")
        if qb is None:
            assert stats[h][0] == ref.qk_tiles and stats[h][2] == ref.valid_tiles
    # the counters of every head: executed tiles = kept blocks of its mask (causal: the visible ones)
    for h in range(H):
        kept = mask[0, h].copy()
        if causal:
            for i in range(Tm):
                kept[i, np.arange(Tn) * 64 > i * 128 + 127] = 0
        assert stats[h][0] == kept.sum(), h
