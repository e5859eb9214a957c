"""The library's host-side Hilbert order (no GPU needed) against the oracle's, which generates the curve
in the other direction (index -> cell instead of cell -> index)."""
import numpy as np
import pytest

from oracle import sparge_oracle as so


@pytest.mark.parametrize("grid", [(1, 6, 6), (13, 30, 45), (20, 48, 48), (1, 1, 1), (2, 1, 3), (7, 7, 7), (1, 64, 64)])
def test_hilbert_order_matches_oracle(grid):
    import paper_2502_18137_amd as sp
    got = sp.sparge_hilbert_order(*grid).numpy()
    np.testing.assert_array_equal(got, so.hilbert_order(grid[1:] if grid[0] == 1 else grid))


def test_hilbert_order_rejects_bad_grids():
    import paper_2502_18137_amd as sp
    with pytest.raises(sp.SpargeError):
        sp.sparge_hilbert_order(0, 4, 4)
    with pytest.raises(sp.SpargeError):
        sp.sparge_hilbert_order(2048, 4, 4)
