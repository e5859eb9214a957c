"""Seeded sweep over small random problems: sequence length, head dimension, dtype, causality, block-mask
density, lambda and the product variant are drawn per case, so that short lists (one to a few tiles),
ragged tails, rows that lose tiles to lambda and reference-maximum moves meet in combinations the fixed
cases do not list.  Each case: the GPU loop against the oracle loop on the same mask (bars as in the
parity tests)."""
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


def draw(seed):
    r = np.random.default_rng(1000 + seed)
    N = int(r.choice([1, 17, 64, 65, 127, 128, 129, 191, 192, 200, 333, 512, 777, 1025, 1400]))
    d = int(r.choice([64, 128]))
    dtype = str(r.choice(["fp16", "bf16"]))
    causal = bool(r.integers(0, 2))
    variant = str(r.choice(["int8", "int8", "fp8", "qk16"]))
    density = float(r.choice([0.15, 0.4, 0.7, 1.0]))
    lam = float(r.choice([-math.inf, -8.0, -2.0, -0.5]))
    noise = float(r.choice([0.3, 1.0, 3.0]))       # larger noise: flatter attention, more reference moves
    return N, d, dtype, causal, variant, density, lam, noise


@pytest.mark.parametrize("seed", range(36))
def test_random_problem(sp, seed):
    import torch
    N, d, dtype, causal, variant, density, lam, noise = draw(seed)
    print(f"seed {seed}: N={N} d={d} {dtype} causal={causal} {variant} density={density} lambda={lam} noise={noise}",
          flush=True)
    w = small_workload(f"rnd{seed}", N=N, d=d, dtype=dtype, H=1, causal=causal, seed=100 + seed, noise=noise,
                       segment=96)
    x, Q, K, V = gpu_inputs(w)
    Tm, Tn = so.nblocks(N, 128), so.nblocks(N, 64)
    r = np.random.default_rng(2000 + seed)
    mask = (r.random((1, 1, Tm, Tn)) < density).astype(np.uint8)
    mask[..., 0] = 1                                            # every row keeps a visible key block
    if causal:
        mask[0, 0, np.arange(Tm), np.minimum(2 * np.arange(Tm), Tn - 1)] = 1
    kw = {"pv_fp8": variant == "fp8", "qk16": variant == "qk16"}
    O, stats = sp.sparge_attn(Q, K, V, torch.from_numpy(mask).to("cuda"), lam, causal=causal, return_stats=True, **kw)
    O = O.float().cpu().numpy().astype(np.float64)[0, 0]
    stats = stats.cpu().numpy()[0, 0]
    assert np.isfinite(O).all()
    slack = sp.REF_SLACK_LOG2_FP8 * math.log(2.0) if variant == "fp8" else REF_SLACK
    ref = so.sparse_attention(x["q"][0, 0], x["k"][0, 0], x["v"][0, 0], mask[0, 0], lam=f32(lam), causal=causal,
                              quant=variant != "qk16", pv_dtype="fp8e4m3" if variant == "fp8" else dtype,
                              ref_slack=slack)
    assert ref.zero_rows == 0
    err = so.rel_l1(O, so.round16(ref.O, dtype))
    print(f"  rel-L1 {err:.2e}; tiles {stats[0]}/{stats[2]}, row groups {stats[1]}/{stats[3]}", flush=True)
    assert err <= 2e-3
    if variant == "int8":
        check_output_parity(so, O, x["q"][0, 0], x["k"][0, 0], x["v"][0, 0], mask[0, 0], f32(lam), causal, dtype,
                            np.arange(N), label=f"seed {seed}")
    assert stats[0] == ref.qk_tiles and stats[2] == ref.valid_tiles and stats[3] == ref.valid_groups
    assert abs(int(stats[1]) - ref.pv_groups) <= max(2, ref.pv_groups // 200)
