"""GPU parity of the token permutation kernels (Sec. 3.7) against the oracle: byte-exact gathers, an exact
round trip, and the effect the paper uses them for (more sparsity at Hilbert order than at row-major order)."""
import numpy as np
import pytest

from oracle import sparge_oracle as so
from synth import CONFIGS, make_workload
from synth.workloads import scaled
from tests.helpers import to_torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2502_18137_amd as sp
    sp.load_library()
    return sp


@pytest.mark.parametrize("dtype,d,grid,offset,tail,strided", [("fp16", 64, (3, 5, 7), 0, 0, False),
                                                              ("bf16", 128, (2, 9, 11), 37, 50, True),
                                                              ("bf16", 64, (1, 1, 1), 5, 0, False)])
def test_permute_and_inverse_are_exact(sp, dtype, d, grid, offset, tail, strided):
    import torch
    L = int(np.prod(grid))
    B, H, N = 2, 3, offset + L + tail
    x = np.random.default_rng(7).standard_normal((B, H, N, d)).astype(np.float32)
    t = to_torch(x, dtype)
    if strided:
        t = t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    perm_lib = sp.sparge_hilbert_order(*grid)
    perm = so.hilbert_order(grid[1:] if grid[0] == 1 else grid)
    np.testing.assert_array_equal(perm_lib.numpy(), perm)
    pd = perm_lib.to("cuda")
    y = sp.sparge_permute_tokens(t, pd, offset)
    xs = t.float().cpu().numpy()
    want = np.stack([[so.permute_tokens(xs[b, h], perm, offset) for h in range(H)] for b in range(B)])
    np.testing.assert_array_equal(y.float().cpu().numpy(), want)
    back = sp.sparge_permute_tokens(y, pd, offset, inverse=True)
    assert torch.equal(back, t)
    # an entry outside the permutation's range leaves its token where it is
    bad = pd.clone()
    bad[0] = L + 5
    yb = sp.sparge_permute_tokens(t, bad, offset)
    assert torch.equal(yb[:, :, offset], t[:, :, offset]) and torch.equal(yb[:, :, offset + 1:], y[:, :, offset + 1:])


def test_hilbert_order_raises_sparsity_and_attention_is_invariant(sp):
    """The image workload is generated along the Hilbert curve; un-permuting gives the same tokens in
    row-major order.  Same hyper-parameters: the Hilbert order must be sparser (Sec. 3.7), and the
    outputs, brought to a common order, must agree like two evaluations of the same attention."""
    import torch
    w = scaled(CONFIGS["image"], H=4)
    x = make_workload(w)
    Q, K, V = (to_torch(x[t], w.dtype) for t in "qkv")
    perm = sp.sparge_hilbert_order(1, *w.grid).to("cuda")   # the generator's 64 x 64 image grid
    Qr, Kr, Vr = (sp.sparge_permute_tokens(T, perm, inverse=True) for T in (Q, K, V))   # row-major order
    Oh, sh = sp.sparge_forward(Q, K, V, w.tau, w.theta, w.lam, return_stats=True)
    Or, sr = sp.sparge_forward(Qr, Kr, Vr, w.tau, w.theta, w.lam, return_stats=True)

    def sparsity(s):
        s = s.cpu().numpy().reshape(-1, 4).sum(0).astype(np.float64)
        return 1.0 - 0.5 * (s[0] / s[2] + s[1] / s[3])
    print(f"sparsity: Hilbert order {sparsity(sh):.3f}, row-major order {sparsity(sr):.3f}", flush=True)
    assert sparsity(sh) > sparsity(sr)
    # full attention is invariant under the permutation up to the quantization blocks, which differ
    dense_r = sp.sparge_attn(Qr, Kr, Vr, None, -np.inf)
    dense_h = sp.sparge_permute_tokens(sp.sparge_attn(Q, K, V, None, -np.inf), perm, inverse=True)
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    assert so.rel_l1(f64(dense_h), f64(dense_r)) < 3e-2
    Oh_r = sp.sparge_permute_tokens(Oh, perm, inverse=True)
    print(f"relative L1 against full attention: Hilbert order {so.rel_l1(f64(Oh_r), f64(dense_r)):.3f}, "
          f"row-major order {so.rel_l1(f64(Or), f64(dense_r)):.3f}", flush=True)
