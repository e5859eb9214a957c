"""The attention kernel's work-item order, through the library's host-side diagnostic (no GPU needed): every
(batch, head, Q block) exactly once whatever the shape, index order without a causal mask, and with one the
property the order exists for -- inside each of the eight ranges the later (longer) half of every head's rows
comes before any earlier half, longest first inside a head."""
import numpy as np
import pytest


def ranges(n):
    per = (n + 7) // 8
    return [(y * per, min(per, n - y * per)) for y in range(8) if n - y * per > 0]


@pytest.mark.parametrize("B,H,N", [(1, 32, 32768), (1, 24, 46080), (2, 3, 700), (1, 1, 100), (1, 5, 128 * 7), (3, 7, 128 * 9 + 5),
                                   (1, 2, 128 * 3), (1, 64, 128 * 2), (1, 9, 128)])
@pytest.mark.parametrize("causal", [False, True])
def test_every_item_once_and_causal_halves(B, H, N, causal):
    import paper_2502_18137_amd as sp
    Tm = (N + 127) // 128
    order = sp.sparge_item_order(B, H, N, 128, causal).numpy()
    n = B * H * Tm
    assert order.shape == (n,)
    assert np.array_equal(np.sort(order), np.arange(n))
    if not causal:
        assert np.array_equal(order, np.arange(n))
        return
    longer = Tm - Tm // 2   # the i >= Tm - longer are the longer rows
    pos = 0
    for r0, ln in ranges(n):
        part = order[pos:pos + ln]
        pos += ln
        # a range covers a contiguous stretch of (head, position-from-the-end) numbers
        heads, i = part // Tm, part % Tm
        g = heads * Tm + (Tm - 1 - i)
        assert np.array_equal(np.sort(g), np.arange(r0, r0 + ln))
        is_long = i >= Tm - longer
        k = int(is_long.sum())
        assert is_long[:k].all() and not is_long[k:].any()
        for half in (part[:k], part[k:]):
            hh, ii = half // Tm, half % Tm
            assert (np.diff(hh) >= 0).all()                       # head by head
            same = np.diff(hh) == 0
            assert (np.diff(ii)[same] == -1).all()                 # longest first inside a head
