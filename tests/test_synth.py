"""Checks of the seeded input generators (host logic only)."""
import numpy as np

from synth import CONFIGS, hilbert_order, make_head
from synth.workloads import scaled


def test_hilbert_curve_visits_neighbouring_cells_on_full_cubes():
    for grid in ((8, 8), (8, 8, 8), (64, 64), (16, 16, 16)):
        p = hilbert_order(grid)
        assert sorted(p.tolist()) == list(range(int(np.prod(grid))))
        c = np.stack(np.unravel_index(p, grid), 1)
        assert (np.abs(np.diff(c, axis=0)).sum(1) == 1).all()   # unit steps: a space-filling walk


def test_hilbert_order_on_non_power_of_two_grid_is_a_local_permutation():
    grid = (13, 30, 45)
    p = hilbert_order(grid)
    assert sorted(p.tolist()) == list(range(13 * 30 * 45))
    c = np.stack(np.unravel_index(p, grid), 1)
    step = np.abs(np.diff(c, axis=0)).sum(1)
    assert np.median(step) == 1 and (step == 1).mean() > 0.9


def test_generators_are_seeded_and_exact_in_their_dtype():
    w = CONFIGS["tiny"]
    a, b = make_head(w, 1), make_head(w, 1)
    for t in "qkv":
        assert a[t].dtype == np.float32 and a[t].shape == (w.N, w.d)
        assert (a[t] == b[t]).all()
        assert (a[t].astype(np.float16).astype(np.float32) == a[t]).all()
    assert not (make_head(w, 0)["q"] == a["q"]).all()
    wi = scaled(CONFIGS["image"], H=1)
    x = make_head(wi, 0)
    for t in "qkv":
        assert (x[t].view(np.uint32) & 0xFFFF == 0).all()      # bf16-representable
    assert abs(float(x["q"].std()) - 1.0) < 0.1
