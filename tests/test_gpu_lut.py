"""The block mask as an index list (Sec. 3.2, Def. 2), through the C ABI: bit-exact against the oracle on random
masks (ragged row lengths, empty and full rows, rows longer than one 64-entry step) and on a predicted mask."""
import numpy as np
import pytest

from oracle import sparge_oracle as so
from tests.helpers import gpu_inputs, small_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2502_18137_amd as sp
    sp.load_library()
    return sp


def check(sp, mask_np, like):
    import torch
    lut, cnt = sp.sparge_mask_to_lut(torch.from_numpy(mask_np).cuda(), like)
    lut, cnt = lut.cpu().numpy(), cnt.cpu().numpy()
    B, H = mask_np.shape[:2]
    for b in range(B):
        for h in range(H):
            ref_lut, ref_cnt = so.mask_to_lut(mask_np[b, h])
            assert np.array_equal(cnt[b, h], ref_cnt), (b, h)
            assert np.array_equal(lut[b, h], ref_lut), (b, h)


@pytest.mark.parametrize("N,density", [(100, 0.5), (4096, 0.3), (8200, 0.05), (17550, 0.7), (140000, 0.02)])
def test_random_masks(sp, N, density):
    import torch
    B, H, d = (1, 1, 64) if N > 100000 else (2, 3, 64)   # (the oracle walks the mask entry by entry)
    like = torch.empty((B, H, N, d), dtype=torch.bfloat16, device="cuda")
    Tm, Tn = (N + 127) // 128, (N + 63) // 64
    rng = np.random.default_rng(N)
    m = (rng.random((B, H, Tm, Tn)) < density).astype(np.uint8)
    m[0, 0, 0, :] = 0          # an empty row
    m[B - 1, H - 1, Tm - 1, :] = 1   # a full row
    m[0, H - 1, Tm // 2, :] = 0
    m[0, H - 1, Tm // 2, Tn - 1] = 7     # any non-zero byte counts as kept
    check(sp, m, like)


def test_predicted_mask(sp):
    w = small_workload("lut", N=3000, d=128, dtype="bf16", H=2, seed=3, causal=True)
    _, Q, K, _ = gpu_inputs(w)
    mask = sp.sparge_predict(Q, K, w.tau, w.theta, causal=True)
    m = mask.cpu().numpy()
    check(sp, m, Q)
    # the list of a row is what Alg. 1's loop visits: its length is the row's kept-block count
    _, cnt = sp.sparge_mask_to_lut(mask, Q)
    assert np.array_equal(cnt.cpu().numpy(), m.sum(axis=-1))
