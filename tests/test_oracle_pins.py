"""Pins for the CPU oracle: closed forms, invariants, brute force and library special cases.

Nothing here compares the oracle with itself through the same formula: every check is either a
value fixed by the mathematics (closed form), an independent brute-force evaluation written a
different way, or a property the paper states (Sec. 3.1-3.4, Def. 2, Alg. 1).
"""
import itertools
import math

import numpy as np
import pytest

from oracle import sparge_oracle as so


def rng(seed):
    return np.random.default_rng(seed)


def as16(x, dtype="fp16"):
    if dtype == "fp16":
        return x.astype(np.float16).astype(np.float64)
    return so.round16(x, "bf16")


# ------------------------------------------------------------------ pooling (Alg. 1 line 4)
def test_pool_constant_block_and_linearity():
    X = np.repeat(rng(0).standard_normal((3, 8)), 64, axis=0)  # 3 constant blocks of 64 rows
    np.testing.assert_allclose(so.pool_blocks(X, 64), X[::64], rtol=0, atol=1e-14)
    A, B = rng(1).standard_normal((200, 8)), rng(2).standard_normal((200, 8))
    lhs = so.pool_blocks(2.0 * A - 3.0 * B, 64)
    rhs = 2.0 * so.pool_blocks(A, 64) - 3.0 * so.pool_blocks(B, 64)
    np.testing.assert_allclose(lhs, rhs, atol=1e-13)


def test_pool_partial_block_uses_valid_rows_only():
    X = np.arange(70 * 2, dtype=np.float64).reshape(70, 2)
    p = so.pool_blocks(X, 64)
    assert p.shape == (2, 2)
    np.testing.assert_allclose(p[1], X[64:].sum(0) / 6.0)


# ------------------------------------------------------------------ CosSim (Sec. 3.2)
def test_cossim_closed_forms():
    d, b = 16, 8
    v = rng(3).standard_normal(d)
    same = np.tile(v, (b, 1)) * rng(4).uniform(0.5, 2.0, (b, 1))   # same direction, any length
    assert so.cossim_blocks(same, b)[0] == pytest.approx(1.0, abs=1e-14)
    ortho = np.eye(d)[:b] * 3.0                                     # b orthogonal tokens -> 1/b
    assert so.cossim_blocks(ortho, b)[0] == pytest.approx(1.0 / b, abs=1e-14)
    anti = np.concatenate([np.tile(v, (b // 2, 1)), np.tile(-v, (b // 2, 1))])
    assert so.cossim_blocks(anti, b)[0] == pytest.approx(0.0, abs=1e-14)
    # two directions at angle phi, half the tokens each: mean cosine = (1 + cos phi) / 2
    phi = 0.7
    e1, e2 = np.eye(d)[0], math.cos(phi) * np.eye(d)[0] + math.sin(phi) * np.eye(d)[1]
    two = np.concatenate([np.tile(e1, (b // 2, 1)), np.tile(e2, (b // 2, 1))])
    assert so.cossim_blocks(two, b)[0] == pytest.approx((1 + math.cos(phi)) / 2, abs=1e-14)


def test_cossim_equals_squared_norm_of_mean_unit_vector():
    X = rng(5).standard_normal((3 * 64 + 10, 32))
    s = so.cossim_blocks(X, 64)
    for t in range(4):
        blk = X[t * 64:(t + 1) * 64]
        u = blk / np.linalg.norm(blk, axis=1, keepdims=True)
        assert s[t] == pytest.approx(float(np.sum(u.mean(0) ** 2)), abs=1e-12)


def test_cossim_pairwise_brute_force_and_zero_token():
    X = rng(6).standard_normal((8, 5))
    X[3] = 0.0
    tot = 0.0
    for a in range(8):
        for b in range(8):
            na, nb = np.linalg.norm(X[a]), np.linalg.norm(X[b])
            tot += 0.0 if na == 0 or nb == 0 else float(X[a] @ X[b]) / (na * nb)
    assert so.cossim_blocks(X, 8)[0] == pytest.approx(tot / 64.0, abs=1e-14)
    # per-token rescaling leaves it unchanged
    Y = X * rng(7).uniform(0.1, 9.0, (8, 1))
    assert so.cossim_blocks(Y, 8)[0] == pytest.approx(tot / 64.0, abs=1e-13)


def test_cossim_literal_formula_differs():
    X = rng(8).standard_normal((64, 16)) + 2.0
    G = X @ X.T
    assert so.cossim_blocks(X, 64, literal=True)[0] == pytest.approx((G / abs(G.max())).mean())
    assert abs(so.cossim_blocks(X, 64, literal=True)[0] - so.cossim_blocks(X, 64)[0]) > 1e-3


# ------------------------------------------------------------------ compressed map (Alg. 1 lines 5-6)
def test_compressed_map_rows_sum_to_one_and_uniform_for_zero_q():
    q = np.zeros((2, 8))
    k = rng(9).standard_normal((7, 8))
    s_k = np.array([1, 1, 0.1, 1, 1, 0.2, 1.0])
    P = so.compressed_map(q, k, s_k, theta=0.5, scale=0.3, causal=False)
    np.testing.assert_allclose(P.sum(1), 1.0, atol=1e-15)
    np.testing.assert_allclose(P[0, [0, 1, 3, 4, 6]], 0.2, atol=1e-15)
    assert P[0, 2] == 0 and P[0, 5] == 0
    q2 = rng(10).standard_normal((3, 8))
    P2 = so.compressed_map(q2, k, np.ones(7), theta=0.5, scale=0.25, causal=False)
    S = 0.25 * q2 @ k.T
    ref = np.exp(S) / np.exp(S).sum(1, keepdims=True)     # textbook softmax
    np.testing.assert_allclose(P2, ref, rtol=1e-13)


def test_compressed_map_all_columns_masked_gives_zero_row():
    P = so.compressed_map(np.ones((1, 4)), np.ones((3, 4)), np.zeros(3), 0.5, 1.0, False)
    assert np.all(P == 0)


def test_compressed_map_is_stable_for_large_logits():
    """Row softmax with the maximum subtracted: logits of +-3000 neither overflow nor lose the runner-up."""
    q = np.array([[30.0, 0.0], [0.0, -30.0]])
    k = np.array([[100.0, 0.0], [99.9, 0.0], [0.0, 100.0], [-100.0, 100.0]])
    P = so.compressed_map(q, k, np.ones(4), 0.0, 1.0, False)
    assert np.isfinite(P).all()
    np.testing.assert_allclose(P.sum(axis=1), 1.0, atol=1e-14)
    np.testing.assert_allclose(P[0, 1] / P[0, 0], math.exp(-3.0), rtol=1e-12)
    assert P[0, 2] == 0.0 and P[0, 3] == 0.0
    np.testing.assert_allclose(P[1, :2], 0.5, atol=1e-14)           # logits 0, 0, -3000, -3000


def test_compressed_map_scale_matters_and_causal_future_is_zero():
    q = rng(11).standard_normal((2, 8))
    k = rng(12).standard_normal((4, 8))
    P = so.compressed_map(q, k, np.ones(4), -1.0, 1.0, causal=True)
    # Q block 0 covers rows 0..127 -> K blocks 0,1 visible, 2,3 entirely future
    assert P[0, 2] == 0 and P[0, 3] == 0 and P[0, :2].sum() == pytest.approx(1.0)
    assert np.all(P[1] > 0)


# ------------------------------------------------------------------ TopCdf (Sec. 3.2)
def test_topcdf_uniform_row_keeps_ceil_tau_n_lowest_indices():
    for n, tau in ((10, 0.55), (7, 0.5), (33, 0.9), (16, 0.33)):
        p = np.full(n, 1.0 / n)
        m, _ = so.top_cdf(p, tau)
        kkeep = math.ceil(tau * n - 1e-9)
        assert m.sum() == kkeep and m[:kkeep].all(), (n, tau)


def test_topcdf_minimal_prefix_with_mass_at_least_tau():
    r = rng(13)
    for trial in range(200):
        n = int(r.integers(2, 40))
        p = r.dirichlet(np.full(n, 0.3))
        tau = float(r.uniform(0.05, 0.99))
        m, dc = so.top_cdf(p, tau)
        if dc.any():
            continue
        kept = p[m]
        assert kept.sum() >= tau * p.sum() - 1e-15
        assert kept.sum() - kept.min() < tau * p.sum()          # minimal: drop the smallest -> below
        assert kept.min() >= p[~m].max() if (~m).any() else True  # it is a top-k set


def test_topcdf_brute_force_smallest_subset():
    r = rng(14)
    for trial in range(30):
        n = int(r.integers(2, 10))
        p = r.dirichlet(np.full(n, 0.5))
        tau = float(r.uniform(0.1, 0.95))
        m, dc = so.top_cdf(p, tau)
        if dc.any():
            continue
        best = None
        for ksz in range(1, n + 1):
            masses = [sum(p[list(c)]) for c in itertools.combinations(range(n), ksz)]
            if max(masses) >= tau * p.sum():
                best = (ksz, max(masses))
                break
        assert m.sum() == best[0]
        assert p[m].sum() == pytest.approx(best[1], abs=1e-14)


def test_topcdf_top_value_above_tau_keeps_exactly_it_and_zeros_never_kept():
    p = np.array([0.05, 0.9, 0.05, 0.0])
    m, _ = so.top_cdf(p, 0.5)
    assert m.tolist() == [False, True, False, False]
    m, _ = so.top_cdf(p, 1.0)       # tau = 1 keeps every positive entry, never a zero one
    assert m.tolist() == [True, True, True, False]
    m, _ = so.top_cdf(np.zeros(5), 0.9)
    assert not m.any()


def test_topcdf_stops_when_the_mass_before_an_entry_equals_the_target():
    """The prefix is the smallest one that reaches tau * sum: an entry whose preceding mass equals the target
    exactly is not kept.  Exact binary fractions, so no rounding blurs the comparison."""
    mask, _ = so.top_cdf(np.array([0.5, 0.25, 0.25]), 0.5)
    assert mask.tolist() == [True, False, False]
    mask, _ = so.top_cdf(np.array([0.125, 0.5, 0.125, 0.25]), 0.75)        # ranks: 0.5, 0.25 | 0.125, 0.125
    assert mask.tolist() == [False, True, False, True]
    mask, _ = so.top_cdf(np.array([0.125, 0.5, 0.125, 0.25]), 0.75 + 2.0 ** -40)
    assert mask.tolist() == [True, True, False, True]


def test_topcdf_with_tau_one_keeps_every_positive_entry_and_no_zero():
    """tau = 1: the positive support (entries so small that the running sum no longer moves may fall to the
    rounding of the sums, and are flagged), and never an entry of probability zero -- also when the prefix sums,
    accumulated in another order than the total, stay a rounding error below it."""
    r = rng(12)
    seen_short = False
    for _ in range(300):
        n = int(r.integers(50, 400))
        p = r.random(n) ** 8
        p[r.random(n) < 0.3] = 0.0
        p /= p.sum()
        mask, dc = so.top_cdf(p, 1.0)
        assert not mask[p == 0].any()                 # a zero is never selected ...
        assert (mask | dc | (p == 0)).all()           # ... and a positive entry is dropped only inside the rounding band
        sp = np.sort(p)[::-1]
        seen_short |= np.cumsum(sp)[(p > 0).sum() - 1] < sp.sum()       # the case in which a zero could slip in
    assert seen_short


def test_topcdf_dont_care_flags_threshold_hits():
    p = np.array([0.5, 0.25, 0.25])
    m, dc = so.top_cdf(p, 0.5)       # mass before rank 1 equals tau*sum exactly
    assert dc[1] or dc[2]
    m, dc = so.top_cdf(np.array([0.6, 0.3, 0.1]), 0.5)
    assert not dc.any() and m.tolist() == [True, False, False]


# ------------------------------------------------------------------ predict: overrides (Sec. 3.2 end)
def _blocks_with_similarity(r, nblk, b, d, similar):
    out = []
    for t in range(nblk):
        if similar[t]:
            c = r.standard_normal(d)
            out.append(c[None] + 0.05 * r.standard_normal((b, d)))
        else:
            out.append(r.standard_normal((b, d)))
    return np.concatenate(out)


def test_predict_overrides_and_pure_topcdf():
    r = rng(15)
    d = 32
    Q = _blocks_with_similarity(r, 4, so.BQ, d, [True, False, True, True])
    K = _blocks_with_similarity(r, 8, so.BK, d, [True, True, False, True, True, True, False, True])
    pr = so.predict(Q, K, tau=0.5, theta=0.5)
    assert pr.sim_q[1] < 0.5 < pr.sim_q[0]
    assert pr.mask[1].all()                      # non-self-similar Q block: whole row
    assert pr.mask[:, 2].all() and pr.mask[:, 6].all()   # non-self-similar K blocks: whole column
    assert pr.p_hat[:, 2].max() == 0 and pr.p_hat[:, 6].max() == 0
    assert not pr.mask.all()                     # something was filtered
    # every selective row keeps mass >= tau among the selective columns
    for i in (0, 2, 3):
        assert pr.p_hat[i][pr.mask[i] == 1].sum() >= 0.5 - 1e-12
    # theta = -inf disables the judge: the mask is TopCdf of the plain compressed map
    pr2 = so.predict(Q, K, tau=0.5, theta=-np.inf)
    q, k = so.pool_blocks(Q, so.BQ), so.pool_blocks(K, so.BK)
    S = q @ k.T / math.sqrt(d)
    P = np.exp(S - S.max(1, keepdims=True))
    P /= P.sum(1, keepdims=True)
    for i in range(4):
        order = np.argsort(-P[i], kind="stable")
        csum = np.cumsum(P[i][order])
        nkeep = int(np.searchsorted(csum, 0.5 * P[i].sum(), side="left")) + 1
        exp = np.zeros(8, dtype=np.uint8)
        exp[order[:nkeep]] = 1
        assert (pr2.mask[i] == exp).all()
    # theta > 1: every block is a fix block -> all ones
    assert so.predict(Q, K, tau=0.5, theta=1.5).mask.all()


def test_predict_fix_rows_are_decided_whatever_topcdf_says():
    """A Q block that is not self-similar keeps its whole row: nothing in it is undecided, even when the row's
    TopCdf sits exactly on its threshold (uniform P-hat, tau * n an integer)."""
    r = rng(27)
    d = 16
    K = _blocks_with_similarity(r, 8, so.BK, d, [True] * 8)
    Q = _blocks_with_similarity(r, 2, so.BQ, d, [True, False])
    Q[so.BQ:] -= Q[so.BQ:].mean(axis=0)          # pooled token of block 1 is zero: its P-hat row is uniform
    pr = so.predict(Q, K, tau=0.5, theta=0.5)
    assert pr.sim_q[1] < 0.5 < pr.sim_q[0]
    np.testing.assert_allclose(pr.p_hat[1], 1.0 / 8.0, atol=1e-12)
    _, flagged = so.top_cdf(pr.p_hat[1], 0.5)
    assert flagged.any()                          # TopCdf alone would call this row undecided ...
    assert pr.mask[1].all() and not pr.dont_care[1].any()      # ... the fix-block rule decides it


def test_predict_causal_rules():
    r = rng(16)
    N, d = 1024, 16
    Q = _blocks_with_similarity(r, 8, so.BQ, d, [True] * 8)
    K = _blocks_with_similarity(r, 16, so.BK, d, [True] * 16)
    pr = so.predict(Q, K, tau=0.3, theta=0.2, causal=True)
    for i in range(8):
        assert not pr.mask[i, 2 * i + 2:].any()      # entirely-future blocks never computed
        assert pr.mask[i, 2 * i] == 1                # block with the first row's own key is kept
    pr_fix = so.predict(Q, K, tau=0.3, theta=1.5, causal=True)   # all fix blocks
    for i in range(8):
        assert pr_fix.mask[i, :2 * i + 2].all() and not pr_fix.mask[i, 2 * i + 2:].any()


def _block_with_cossim(n, d, target):
    """n tokens on two orthonormal directions, half each: cosine similarity (1 + cos phi) / 2 = target."""
    phi = math.acos(2.0 * target - 1.0)
    a = np.zeros(d); a[0] = 1.0
    b = np.zeros(d); b[0], b[1] = math.cos(phi), math.sin(phi)
    return np.stack([a if t % 2 == 0 else b for t in range(n)])


def test_predict_marks_similarities_on_the_threshold_as_undecidable():
    """A block whose self-similarity lies within 1e-5 of theta is neither a fix block nor a selective one
    for certain: a Q block in that band makes its own mask row don't-care, a K block the whole head (it
    changes every row's softmax); 1e-4 away on either side nothing is exempt, and the decision itself
    follows the side the similarity is on."""
    r = rng(25)
    d, theta = 16, 0.5
    base_q = [_block_with_cossim(so.BQ, d, 0.9) * (1 + 0.1 * i) for i in range(3)]
    base_k = [_block_with_cossim(so.BK, d, 0.9) * (1 + 0.05 * j) for j in range(6)]
    for off, band in ((-1e-4, False), (-1e-6, True), (1e-6, True), (1e-4, False)):
        Qb = list(base_q)
        Qb[1] = _block_with_cossim(so.BQ, d, theta + off)
        pr = so.predict(np.concatenate(Qb), np.concatenate(base_k), tau=0.4, theta=theta)
        assert abs(pr.sim_q[1] - (theta + off)) < 1e-12
        assert pr.dont_care[1].all() == band and not pr.dont_care[[0, 2]].any()
        assert pr.mask[1].all() == (off < 0)          # below theta: fix block, whole row kept
        Kb = list(base_k)
        Kb[4] = _block_with_cossim(so.BK, d, theta + off)
        pr = so.predict(np.concatenate(base_q), np.concatenate(Kb), tau=0.4, theta=theta)
        assert abs(pr.sim_k[4] - (theta + off)) < 1e-12
        assert pr.dont_care.all() == band and (band or not pr.dont_care.any())
        assert pr.mask[:, 4].all() == (off < 0) or off > 0
        if off < 0:
            assert pr.mask[:, 4].all() and (pr.p_hat[:, 4] == 0).all()
    # causal: entirely-future blocks and the forced diagonal block are decided whatever the band says
    Qb = list(base_q)
    Qb[1] = _block_with_cossim(so.BQ, d, theta + 1e-6)
    pr = so.predict(np.concatenate(Qb), np.concatenate(base_k), tau=0.4, theta=theta, causal=True)
    assert pr.dont_care[1, :2].all() and not pr.dont_care[1, 2] and not pr.dont_care[1, 4:].any()


# ------------------------------------------------------------------ quantization (Alg. 1 line 3)
def test_quant_roundtrip_within_half_step_and_amax_hits_127():
    X = as16(rng(17).standard_normal((300, 64)) * 3.0)
    Xq, delta = so.quantize_q(X)
    assert Xq.dtype == np.int8 and delta.dtype == np.float32 and delta.shape == (3,)
    for t in range(3):
        blk = X[t * 128:(t + 1) * 128]
        q = Xq[t * 128:(t + 1) * 128].astype(np.float64)
        dl = float(delta[t])
        assert np.abs(blk - q * dl).max() <= dl * (0.5 + 1e-6)
        amax_pos = np.unravel_index(np.abs(blk).argmax(), blk.shape)
        assert abs(q[amax_pos]) == 127
        assert np.abs(q).max() == 127
        assert dl == pytest.approx(np.abs(blk).max() / 127.0, rel=1e-7)


def test_quant_is_nearest_integer_of_the_exact_quotient_up_to_fp32_rounding():
    # x_hat must be a nearest integer of the exactly computed 127*x/amax (python fractions =
    # independent arithmetic) whenever that quotient is further than 2^-15 from a half-integer;
    # closer than that the fp32 product may legitimately land on either neighbour.
    from fractions import Fraction
    X = as16(rng(18).standard_normal((128, 16)))
    Xq, _ = so.quantize_q(X)
    amax = Fraction(float(np.abs(X).max()))
    checked = 0
    for (a, b), x in np.ndenumerate(X):
        y = Fraction(127) * Fraction(float(x)) / amax
        fl = math.floor(y)
        rem = y - fl
        if abs(rem - Fraction(1, 2)) < Fraction(1, 2 ** 15):
            continue
        checked += 1
        assert int(Xq[a, b]) == (fl + 1 if rem > Fraction(1, 2) else fl)
    assert checked > 2000


def test_quant_zero_block_and_power_of_two_scaling():
    X = as16(rng(19).standard_normal((256, 32)))
    X[128:] = 0.0
    Xq, delta = so.quantize_q(X)
    assert delta[1] == 0 and not Xq[128:].any()
    Xq2, delta2 = so.quantize_q(X * 8.0)
    assert (Xq2 == Xq).all() and delta2[0] == delta[0] * 8.0


def test_quant_half_to_even():
    # amax = 127 -> y = x exactly; x = 0.5, 1.5, 2.5, -0.5, -1.5 round to 0, 2, 2, -0, -2
    X = np.zeros((128, 8))
    X[0, 0] = 127.0
    X[1, :5] = [0.5, 1.5, 2.5, -0.5, -1.5]
    Xq, delta = so.quantize_q(X)
    assert delta[0] == 1.0
    assert Xq[1, :5].tolist() == [0, 2, 2, 0, -2]


def test_exact_quantizer_against_rational_arithmetic_and_tie_flags():
    """quantize_exact = round-half-even of the exact quotient 127 x / amax, and its flag marks exactly the
    quotients within 2^-15 of a half-integer: python fractions on every element of blocks that hold random
    values, exact ties, near ties on both sides, values far below the block maximum and a zero row."""
    from fractions import Fraction
    r = rng(23)
    X = (r.standard_normal((256, 16)) * np.exp(2.0 * r.standard_normal((256, 1)))).astype(np.float32)
    X[0, 0] = 127.0 * 2.0 ** 20                        # block 0: amax = 127 * 2^20 -> quotient = x / 2^20
    X[0, 1:] = 0.0
    X[1, :6] = np.array([0.5, 1.5, 2.5, -3.5, 126.5, -0.5]) * 2.0 ** 20          # exact ties
    X[2, :4] = np.float32(2.0 ** 20) * np.array([0.5, 1.5, -2.5, 7.5], dtype=np.float32) * \
        np.array([1 + 2.0 ** -22, 1 - 2.0 ** -23, 1 + 2.0 ** -21, 1 - 2.0 ** -20], dtype=np.float32)  # near ties
    X[3, :3] = [2.0 ** -30, -2.0 ** -60, 1e-38]        # negligible against amax
    X[4] = 0.0
    X = np.minimum(np.abs(X), 127.0 * 2.0 ** 20).astype(np.float32) * np.sign(X).astype(np.float32)
    X[0, 0] = 127.0 * 2.0 ** 20
    X[130:, :] = np.abs(X[130:, :]) * np.float32(1e-3)                      # block 1: ordinary values
    xe, near = so.quantize_exact(X, so.BQ)
    for t in range(2):
        blk = X[t * 128:(t + 1) * 128]
        amax = Fraction(float(np.abs(blk).max()))
        for (a, b), x in np.ndenumerate(blk):
            y = 127 * Fraction(float(x)) / amax
            assert int(xe[t * 128 + a, b]) == round(y)            # python rounds fractions half to even
            frac = abs(y) - math.floor(abs(y))
            assert bool(near[t * 128 + a, b]) == (abs(frac - Fraction(1, 2)) < Fraction(1, 2 ** 15))
    assert xe[1, :6].tolist() == [0, 2, 2, -4, 126, 0] and near[1, :6].all()     # ties go to even
    assert near[2, :4].all() and not near[3:5].any() and not xe[3:5].any()
    assert near.sum() >= 10


def test_fp32_quantizer_equals_the_exact_rounding_away_from_ties():
    """The specified fp32 sequence x * fl(127/amax) rounds to the exact result wherever the exact quotient is
    not flagged, for 16-bit inputs (Q) and for the fp32 differences K - mean alike; the flagged elements are
    few.  (Inside the flag the two may differ: there the sequence is the specification.)"""
    r = rng(24)
    for dtype in ("fp16", "bf16"):
        Q = as16(r.standard_normal((640, 64)) * np.exp(r.standard_normal((640, 1))), dtype)
        xq, _ = so.quantize_q(Q)
        xe, near = so.quantize_exact(Q.astype(np.float32), so.BQ)
        assert ((xq == xe) | near).all() and near.mean() < 1e-3
        K = as16(r.standard_normal((640, 64)) + 0.7, dtype)
        kq, _, mean = so.quantize_k(K)
        ke, neark = so.quantize_exact(K.astype(np.float32) - mean[None, :], so.BK)
        assert ((kq == ke) | neark).all() and neark.mean() < 1e-3
    # every finite non-negative fp16 value up to the block maximum, for a handful of maxima (each block of the
    # column ends with the maximum itself)
    allh = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float32)
    for amax in (1.0, 3.0, 127.0, 0.3330078125, 1000.0, 65504.0, 6.103515625e-05):
        col = allh[allh <= amax]
        col = np.concatenate([col, np.zeros((-len(col)) % 128, dtype=np.float32)])[:, None]
        col[127::128, 0] = amax
        xq, _ = so._quant_blocks(col, 128)
        xe, near = so.quantize_exact(col, 128)
        assert ((xq == xe) | near).all(), amax


def test_k_smoothing_mean_and_shift_invariance():
    r = rng(20)
    K = as16(r.standard_normal((320, 16)) + 1.5, "bf16")
    Kq, dK, mean = so.quantize_k(K)
    assert mean.dtype == np.float32
    np.testing.assert_allclose(mean, K.mean(0), rtol=1e-6)
    assert abs(float((Kq.astype(np.float64) * np.repeat(dK, 64)[:, None]).mean())) < 0.05
    # softmax attention does not change when a constant vector is removed from every key
    Q, V = r.standard_normal((320, 16)), r.standard_normal((320, 16))
    np.testing.assert_allclose(so.dense_attention(Q, K, V), so.dense_attention(Q, K - K.mean(0), V),
                               atol=1e-12)
    # nor does the compressed map P-hat
    q, k1, k2 = so.pool_blocks(Q, 128), so.pool_blocks(K, 64), so.pool_blocks(K - K.mean(0), 64)
    ones = np.ones(5)
    np.testing.assert_allclose(so.compressed_map(q, k1, ones, 0.0, 0.25, False),
                               so.compressed_map(q, k2, ones, 0.0, 0.25, False), atol=1e-13)


def test_k_mean_is_exact_sum_over_n():
    from fractions import Fraction
    K = as16(rng(21).standard_normal((130, 3)) * 100.0, "bf16")
    mean = so.k_mean(K)
    for c in range(3):
        exact = sum(Fraction(float(v)) for v in K[:, c]) / 130
        assert float(mean[c]) == float(np.float32(float(exact)))
    # thousands of terms of mixed magnitude and sign: a sum that rounds along the way (fp32, or fp64 in an
    # unlucky order) no longer lands on the correctly rounded mean in every channel
    r = rng(26)
    K = as16(r.standard_normal((6000, 8)) * np.exp2(r.integers(-12, 13, size=(6000, 8))) + 3.0, "bf16")
    mean = so.k_mean(K)
    for c in range(8):
        exact = sum(Fraction(float(v)) for v in K[:, c]) / 6000
        assert float(mean[c]) == float(np.float32(exact.numerator / exact.denominator))


# ------------------------------------------------------------------ dense reference vs textbook
def test_dense_attention_textbook_and_rows_of_p_sum_to_one():
    r = rng(22)
    Q, K, V = r.standard_normal((70, 8)), r.standard_normal((70, 8)), r.standard_normal((70, 8))
    O = so.dense_attention(Q, K, V)
    ref = np.zeros_like(O)
    for a in range(70):      # scalar loops: independent of the matrix code
        w = [math.exp(sum(Q[a, c] * K[b, c] for c in range(8)) / math.sqrt(8)) for b in range(70)]
        z = sum(w)
        for c in range(8):
            ref[a, c] = sum(w[b] * V[b, c] for b in range(70)) / z
    np.testing.assert_allclose(O, ref, atol=1e-12)
    # V = ones -> every output is exactly the row sum of P = 1
    np.testing.assert_allclose(so.dense_attention(Q, K, np.ones((70, 8))), 1.0, atol=1e-14)
    Oc = so.dense_attention(Q, K, V, causal=True)
    np.testing.assert_allclose(Oc[0], V[0], atol=1e-14)      # first row sees only itself


def test_dense_attention_permutation_invariance():
    r = rng(23)
    Q, K, V = (r.standard_normal((50, 8)) for _ in range(3))
    p, pq = r.permutation(50), r.permutation(50)
    O = so.dense_attention(Q, K, V)
    np.testing.assert_allclose(so.dense_attention(Q[pq], K[p], V[p]), O[pq], atol=1e-13)


# ------------------------------------------------------------------ flash loop (Sec. 3.1, Def. 2)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N", [256, 300, 77])
def test_loop_all_ones_no_skip_no_quant_equals_dense(N, causal):
    r = rng(24 + N)
    Q, K, V = (r.standard_normal((N, 16)) for _ in range(3))
    res = so.sparse_attention(Q, K, V, None, lam=-np.inf, causal=causal, quant=False)
    np.testing.assert_allclose(res.O, so.dense_attention(Q, K, V, causal=causal), atol=1e-12)
    assert res.zero_rows == 0 and res.sparsity == pytest.approx(0.0)
    # independent count: a (row group, K block) pair is needed iff some key of the block is visible
    need = 0
    for g in range(math.ceil(N / 32)):
        last_row = min(32 * g + 31, N - 1)
        for j in range(so.nblocks(N, 64)):
            need += (not causal) or (64 * j <= last_row)
    assert res.pv_groups == need == res.valid_groups


def test_whole_operator_dense_switches_equal_brute_force():
    # tau=1, theta>1 (all fix blocks), lambda=-inf, quantization off -> plain softmax attention
    r = rng(30)
    Q, K, V = (r.standard_normal((200, 16)) for _ in range(3))
    res, pred = so.spargeattn(Q, K, V, tau=1.0, theta=1.5, lam=-np.inf, quant=False)
    assert pred.mask.all()
    np.testing.assert_allclose(res.O, so.dense_attention(Q, K, V), atol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
def test_loop_with_block_mask_equals_dense_with_minus_inf_blocks(causal):
    r = rng(31)
    N = 520
    Q, K, V = (r.standard_normal((N, 16)) for _ in range(3))
    Tm, Tn = so.nblocks(N, 128), so.nblocks(N, 64)
    mask = (r.uniform(size=(Tm, Tn)) < 0.5).astype(np.uint8)
    for i in range(Tm):
        mask[i, 2 * i] = 1           # keep every row alive (also under causal)
    res = so.sparse_attention(Q, K, V, mask, lam=-np.inf, causal=causal, quant=False)
    ref = so.dense_attention(Q, K, V, causal=causal, block_mask=mask)
    np.testing.assert_allclose(res.O, ref, atol=1e-12)
    assert res.zero_rows == 0


def test_loop_quantized_equals_dense_on_dequantized_operands():
    r = rng(32)
    N = 330
    Q, K, V = as16(r.standard_normal((N, 32))), as16(r.standard_normal((N, 32)) + 0.7), r.standard_normal((N, 32))
    res = so.sparse_attention(Q, K, V, None, lam=-np.inf, quant=True)
    Qd, Kd = so.dequantized_qk(Q, K)
    np.testing.assert_allclose(res.O, so.dense_attention(Qd, Kd, V), atol=1e-11)
    # and INT8 quantization stays close to the exact result
    assert so.rel_l1(res.O, so.dense_attention(Q, K, V)) < 3e-2


def test_fully_masked_row_reports_zero_rows():
    r = rng(33)
    Q, K, V = (r.standard_normal((256, 8)) for _ in range(3))
    mask = np.ones((2, 4), dtype=np.uint8)
    mask[1] = 0
    res = so.sparse_attention(Q, K, V, mask, quant=False)
    assert res.zero_rows == 128 and np.all(res.O[128:] == 0)


# ------------------------------------------------------------------ lambda skip (Sec. 3.4)
def _peaky_inputs(seed, N=512, d=16):
    r = rng(seed)
    cent = r.standard_normal((N // 64, d)) * 2.5
    K = np.repeat(cent, 64, axis=0) + 0.2 * r.standard_normal((N, d))
    Q = np.repeat(cent, 64, axis=0) * 1.5 + 0.2 * r.standard_normal((N, d))
    V = r.standard_normal((N, d))
    return Q, K, V


def test_lambda_minus_inf_is_mask_only_and_skips_grow_with_lambda():
    Q, K, V = _peaky_inputs(40)
    base = so.sparse_attention(Q, K, V, None, lam=-np.inf, quant=False)
    prev = base.pv_groups
    seen_skip = False
    for lam in (-60.0, -30.0, -15.0, -8.0, -4.0, -2.0):
        res = so.sparse_attention(Q, K, V, None, lam=lam, quant=False)
        assert res.pv_groups <= prev
        assert res.qk_tiles == base.qk_tiles
        prev = res.pv_groups
        seen_skip |= res.pv_groups < base.pv_groups
    assert seen_skip


def test_lambda_error_bound_per_row():
    Q, K, V = _peaky_inputs(41)
    N = Q.shape[0]
    base = so.sparse_attention(Q, K, V, None, lam=-np.inf, quant=False)
    for lam in (-12.0, -6.0, -3.0):
        res = so.sparse_attention(Q, K, V, None, lam=lam, quant=False)
        skipped_groups = base.pv_groups - res.pv_groups
        assert skipped_groups > 0
        # every dropped term is <= e^lam * |V| relative to the running max at that time, which is
        # <= the final max; l >= 1 in units of the final max; at most N columns are dropped
        bound = N * math.exp(lam) * np.abs(V).max()
        assert np.abs(res.O - base.O).max() <= bound
    # a looser analytic check with fewer dropped columns: error shrinks as lambda decreases
    e3 = np.abs(so.sparse_attention(Q, K, V, None, lam=-3.0, quant=False).O - base.O).max()
    e12 = np.abs(so.sparse_attention(Q, K, V, None, lam=-12.0, quant=False).O - base.O).max()
    assert e12 < e3


def test_lambda_threshold_is_strict_and_per_row_group():
    # one Q block (128 rows), two K blocks; all scores in block 0 are 0, block 1 scores are -g per
    # row group g: row group w has m_local - m = -(w+1)*2 in block 1 -> executed iff -(w+1)*2 > lam
    d = 4
    Q = np.zeros((128, d))
    for w in range(4):
        Q[32 * w:32 * (w + 1), 0] = (w + 1) * 2.0
    K = np.zeros((128, d))
    K[64:, 0] = -1.0
    V = rng(42).standard_normal((128, d))
    for lam, expect in ((-1.0, 4 + 0), (-2.0, 4 + 0), (-2.5, 4 + 1), (-4.0, 4 + 1), (-4.5, 4 + 2), (-100.0, 8)):
        res = so.sparse_attention(Q, K, V, None, lam=lam, scale=1.0, quant=False)
        assert res.pv_groups == expect, (lam, res.pv_groups)
    # sparsity counts both kinds of skipped products (Sec. 4.1): here both tiles run, 5 of 8 row-group products do
    res = so.sparse_attention(Q, K, V, None, lam=-2.5, scale=1.0, quant=False)
    assert (res.qk_tiles, res.valid_tiles, res.pv_groups, res.valid_groups) == (2, 2, 5, 8)
    assert res.sparsity == pytest.approx(1.0 - 0.5 * (1.0 + 5.0 / 8.0))
    # the reported distance of the statistic from lambda: tile 0 has m_local - m = 0, tile 1 has -2(w+1)
    res = so.sparse_attention(Q, K, V, None, lam=-4.25, scale=1.0, quant=False)
    np.testing.assert_allclose(res.lam_margin[0], [2.25, 0.25, 1.75, 3.75], atol=1e-12)
    assert np.isinf(so.sparse_attention(Q, K, V, None, scale=1.0, quant=False).lam_margin).all()
    K2 = K.copy()
    K2[:64, 0] = 1.0                  # tile 0 scores 2(w+1), tile 1 scores -2(w+1): the statistic is -4(w+1), not m_local
    res = so.sparse_attention(Q, K2, V, None, lam=-9.0, scale=1.0, quant=False)
    np.testing.assert_allclose(res.lam_margin[0], [5.0, 1.0, 3.0, 7.0], atol=1e-12)
    assert res.pv_groups == 4 + 2
    # l is updated even for skipped groups: output = sum over block 0 of V / (64 + 64 e^{-2(w+1)})
    res = so.sparse_attention(Q, K, V, None, lam=-1.0, scale=1.0, quant=False)
    for w in range(4):
        expect = V[:64].sum(0) / (64.0 + 64.0 * math.exp(-2.0 * (w + 1)))
        np.testing.assert_allclose(res.O[32 * w], expect, atol=1e-13)


def test_sparsity_accounting():
    Q, K, V = (rng(43).standard_normal((256, 8)) for _ in range(3))
    mask = np.array([[1, 0, 0, 0], [1, 1, 0, 0]], dtype=np.uint8)
    res = so.sparse_attention(Q, K, V, mask, quant=False)
    assert (res.qk_tiles, res.pv_groups, res.valid_tiles, res.valid_groups) == (3, 12, 8, 32)
    assert res.sparsity == pytest.approx(1 - (3 + 3) / 16)
    resc = so.sparse_attention(Q, K, V, None, causal=True, quant=False)
    assert resc.valid_tiles == 2 + 4 and resc.sparsity == pytest.approx(0.0)


def test_pv_rounding_only_touches_numerator():
    Q, K, V = _peaky_inputs(44, N=256)
    a = so.sparse_attention(Q, K, V, None, quant=False, pv_dtype="none")
    b = so.sparse_attention(Q, K, np.ones_like(V), None, quant=False, pv_dtype="bf16")
    # with V = 1 the output is rowsum(round(P~))/rowsum(P~): close to, but not exactly, 1
    assert np.abs(b.O - 1.0).max() < 2 ** -8 and np.abs(b.O - 1.0).max() > 0
    assert so.rel_l1(so.sparse_attention(Q, K, V, None, quant=False, pv_dtype="fp16").O, a.O) < 1e-3


def test_round16_ties_and_exactness():
    assert so.round16(np.array([1.0 + 2 ** -8]), "bf16")[0] == 1.0            # tie -> even
    assert so.round16(np.array([1.0 + 3 * 2 ** -8]), "bf16")[0] == 1.0 + 2 ** -6
    assert so.round16(np.array([0.333251953125]), "fp16")[0] == 0.333251953125  # exact fp16 value
    assert so.rel_l1(np.array([1.0, -3.0]), np.array([2.0, -2.0])) == pytest.approx(0.5)


def test_judge_matters_on_non_self_similar_blocks():
    # synthetic analogue of the self-similarity-judge ablation (App. A.2): keys of block 5 are not
    # self-similar but a few of them matter a lot; without the judge (theta=-inf) the compressed
    # token hides them and the error grows
    r = rng(45)
    N, d = 1024, 32
    cent = r.standard_normal((N // 64, d))
    K = np.repeat(cent, 64, axis=0) + 0.1 * r.standard_normal((N, d))
    Q = r.standard_normal((N // 128, d)).repeat(128, axis=0) + 0.1 * r.standard_normal((N, d))
    K[5 * 64:6 * 64] = r.standard_normal((64, d)) * 0.3
    K[5 * 64:5 * 64 + 4] = Q[::128][:4] * 3.0       # needles inside the noisy block
    V = r.standard_normal((N, d))
    ref = so.dense_attention(Q, K, V)
    with_j, _ = so.spargeattn(Q, K, V, tau=0.6, theta=0.5, lam=-np.inf, quant=False)
    no_j, _ = so.spargeattn(Q, K, V, tau=0.6, theta=-np.inf, lam=-np.inf, quant=False)
    assert so.rel_l1(with_j.O, ref) < so.rel_l1(no_j.O, ref)


# ---------------------------------------------------------------------------------------------
# The reference maximum inside exp is free (rescaling identity of Sec. 3.1)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_reference_slack_does_not_change_the_result_without_rounding(causal):
    """O/l does not depend on the reference that exp subtracts: any slack gives the same output up to
    fp64 rounding, the same executed groups and the same counters (the stage-2 test uses the true m)."""
    rng = np.random.default_rng(31)
    N, d = 333, 16
    Q, K, V = 3.0 * rng.standard_normal((N, d)), rng.standard_normal((N, d)), rng.standard_normal((N, d))
    mask = rng.random((so.nblocks(N, so.BQ), so.nblocks(N, so.BK))) < 0.7
    mask[:, 0] = True
    if causal:
        mask[np.arange(mask.shape[0]), 2 * np.arange(mask.shape[0])] = True
    base = so.sparse_attention(Q, K, V, mask, lam=-3.0, causal=causal, quant=True, pv_dtype="none")
    for slack in (0.5, 8 * math.log(2.0), 1e9):
        r = so.sparse_attention(Q, K, V, mask, lam=-3.0, causal=causal, quant=True, pv_dtype="none", ref_slack=slack)
        assert np.abs(r.O - base.O).max() < 1e-12
        assert (r.qk_tiles, r.pv_groups, r.valid_tiles, r.valid_groups) == \
            (base.qk_tiles, base.pv_groups, base.valid_tiles, base.valid_groups)
    dense = so.dense_attention(*so.dequantized_qk(Q, K), V, causal=causal, block_mask=mask)
    nolam = so.sparse_attention(Q, K, V, mask, causal=causal, quant=True, pv_dtype="none", ref_slack=8 * math.log(2.0))
    assert np.abs(nolam.O - dense).max() < 1e-10


def test_reference_slack_only_moves_the_16_bit_rounding_of_p():
    """With P~ rounded to 16 bits the slack changes the result by rounding noise only, and P~ stays
    below exp(slack) (it is at most 1 with slack 0)."""
    rng = np.random.default_rng(32)
    N, d = 400, 32
    Q, K, V = 2.0 * rng.standard_normal((N, d)), rng.standard_normal((N, d)), rng.standard_normal((N, d))
    exact = so.sparse_attention(Q, K, V, None, quant=True, pv_dtype="none")
    for dt, tol in (("fp16", 2e-3), ("bf16", 1.2e-2)):
        a = so.sparse_attention(Q, K, V, None, quant=True, pv_dtype=dt)
        b = so.sparse_attention(Q, K, V, None, quant=True, pv_dtype=dt, ref_slack=8 * math.log(2.0))
        assert so.rel_l1(a.O, exact.O) < tol and so.rel_l1(b.O, exact.O) < tol
        assert 0 < so.rel_l1(b.O, a.O) < tol


def test_reference_moves_per_row_group_when_one_row_runs_ahead():
    """Two tiles, one row of the first 32-row group gets a much larger score in the second tile:
    with slack s that group's reference moves (its P~ are again <= 1), the other groups keep theirs.
    Checked through the rounding: V = e_0, P~ rounded to bf16, compare with a direct evaluation."""
    N, d = 128, 8
    Q = np.zeros((N, d)); K = np.zeros((N, d)); V = np.zeros((N, d))
    Q[:, 0] = 1.0
    K[:64, 0] = 1.0                      # tile 0: every score equal
    K[64:, 0] = np.linspace(1.0, 1.5, 64)  # tile 1: slightly larger scores
    Q[5, 0] = 40.0                       # row 5 (group 0): its scores run ahead by far more than the slack
    V[:, 0] = np.arange(N) / N
    slack = 2.0
    r = so.sparse_attention(Q, K, V, None, scale=1.0, quant=False, pv_dtype="bf16", ref_slack=slack)
    S = Q @ K.T
    for row, moved in ((5, True), (6, True), (40, False)):   # rows 5, 6 share group 0; row 40 is in group 1
        m0 = S[row, :64].max()
        m1 = S[row].max()
        ref1 = m1 if moved else m0       # reference in force for tile 1
        # tile 0 is rounded against m0; when the reference moves its contribution is rescaled exactly
        p0 = so.round16(np.exp(S[row, :64] - m0), "bf16") * np.exp(m0 - ref1)
        p1 = so.round16(np.exp(S[row, 64:] - ref1), "bf16")
        l = np.exp(S[row, :64] - m0).sum() * np.exp(m0 - ref1) + np.exp(S[row, 64:] - ref1).sum()
        want = (p0 @ V[:64, 0] + p1 @ V[64:, 0]) / l
        assert abs(r.O[row, 0] - want) < 1e-12, (row, r.O[row, 0], want)


# ------------------------------------------------------------------ FP8 (E4M3) P~V product
def _e4m3_values():
    """All non-negative finite E4M3 numbers, written out from the format definition."""
    vals = [m / 8.0 * 2.0 ** -6 for m in range(8)]                                   # zero and subnormals
    vals += [2.0 ** (E - 7) * (1 + m / 8.0) for E in range(1, 16) for m in range(8)]  # normals
    return np.array(vals[:-1])                                                       # S.1111.111 is NaN


def test_e4m3_grid_nearest_even_and_library_conversion():
    torch = pytest.importorskip("torch")
    g = _e4m3_values()
    assert g.size == 127 and g.max() == 448.0 and g[1] == 2.0 ** -9
    np.testing.assert_array_equal(so.round_e4m3(g), g)                 # idempotent on the grid
    np.testing.assert_array_equal(so.round_e4m3(-g), -g)
    np.testing.assert_array_equal(so.encode_e4m3(g), np.arange(127, dtype=np.uint8))
    np.testing.assert_array_equal(so.encode_e4m3(-g[1:]), np.arange(1, 127, dtype=np.uint8) | 0x80)
    # nearest grid value for random fp32 inputs, by brute force over the grid
    x = rng(70).uniform(-448, 448, 20000).astype(np.float32).astype(np.float64)
    x = np.concatenate([x, rng(71).uniform(-0.04, 0.04, 20000).astype(np.float32).astype(np.float64)])
    r = so.round_e4m3(x)
    full = np.concatenate([-g[::-1], g])
    best = np.abs(x[:, None] - full[None, :]).min(axis=1)
    np.testing.assert_array_equal(np.abs(r - x), best)
    # ties go to the even mantissa: midpoints of neighbouring grid values
    mid = (g[:-1] + g[1:]) / 2
    even = np.where(np.arange(126) % 2 == 0, g[:-1], g[1:])
    np.testing.assert_array_equal(so.round_e4m3(mid), even)
    assert so.round_e4m3(np.array([1.0625]))[0] == 1.0 and so.round_e4m3(np.array([1.1875]))[0] == 1.25
    assert so.round_e4m3(np.array([2.0 ** -10]))[0] == 0.0 and so.round_e4m3(np.array([0.00098]))[0] == 2.0 ** -9
    with pytest.raises(ValueError):
        so.round_e4m3(np.array([480.0]))
    # the library's conversion (fp32 -> float8_e4m3fn) agrees on fp32 inputs
    t = torch.tensor(x, dtype=torch.float32).to(torch.float8_e4m3fn)
    np.testing.assert_array_equal(t.to(torch.float64).numpy(), r)
    np.testing.assert_array_equal(t.view(torch.uint8).numpy(), so.encode_e4m3(x))


def test_fp8_v_quantization_per_channel():
    r = rng(72)
    V = as16(r.standard_normal((300, 16)) * r.uniform(0.01, 30, 16)[None, :])
    V[:, 3] = 0.0
    Vq, delta = so.quantize_v_fp8(V)
    amax = np.abs(V).max(axis=0)
    np.testing.assert_allclose(delta, amax / 448.0, rtol=2e-7)
    assert delta[3] == 0 and np.all(Vq[:, 3] == 0)
    assert np.abs(Vq).max() == 448.0 and np.all(np.abs(Vq).max(axis=0)[delta > 0] == 448.0)
    # dequantized values lie within half an E4M3 step (2^-4 relative, 2^-10 of the range near zero) of V
    err = np.abs(Vq * delta[None, :] - V)
    assert np.all(err <= np.maximum(np.abs(V) * 2.0 ** -4, amax[None, :] / 448 * 2.0 ** -10) * (1 + 1e-6))


def test_fp8_product_exact_when_operands_sit_on_the_grid():
    # one-hot attention (each query sees one key overwhelmingly) with V on a per-channel E4M3 grid:
    # P~ is 1 at one key, c_P = 448 e^{-slack} = 112 is an E4M3 number, so O must equal that V row
    N, d = 256, 64
    g = _e4m3_values()
    r = rng(73)
    ch_scale = 2.0 ** r.integers(-3, 4, d)
    V = r.choice(g[40:], (N, d)) * r.choice([-1.0, 1.0], (N, d))
    V[0] = 448.0                                  # every channel's amax is 448 -> delta = its scale
    V = V * ch_scale[None, :]
    Q = np.zeros((N, d)); K = np.zeros((N, d))
    dirs = r.standard_normal((N, d)); dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
    Q[:] = dirs * 300.0; K[:] = dirs            # q_t . k_t = 300, q_t . k_s ~ N(0, 300^2/d): far below
    res = so.sparse_attention(Q, K, V, None, quant=False, pv_dtype="fp8e4m3", ref_slack=2 * math.log(2.0),
                              scale=1.0)
    exact = so.dense_attention(Q, K, V, scale=1.0)
    assert so.rel_l1(exact, V) < 1e-12          # the construction is one-hot
    np.testing.assert_allclose(res.O, V, rtol=1e-12, atol=0)


def test_fp8_product_error_is_a_few_percent_and_above_the_16_bit_one():
    Q, K, V = _peaky_inputs(74, N=512)
    exact = so.sparse_attention(Q, K, V, None, quant=False, pv_dtype="none").O
    e8 = so.rel_l1(so.sparse_attention(Q, K, V, None, quant=False, pv_dtype="fp8e4m3",
                                       ref_slack=2 * math.log(2.0)).O, exact)
    e16 = so.rel_l1(so.sparse_attention(Q, K, V, None, quant=False, pv_dtype="bf16").O, exact)
    # two roundings with unit roundoff 2^-4 per product, averaged over the keys a row attends to
    assert e16 < e8 < 2 * 2.0 ** -4
    # with V = 1 in every channel, V-hat = 448 exactly and only the rounding of P~ is left
    ones = so.sparse_attention(Q, K, np.ones_like(V), None, quant=False, pv_dtype="fp8e4m3",
                               ref_slack=2 * math.log(2.0)).O
    assert 0 < np.abs(ones - 1.0).max() < 2.0 ** -4


# ------------------------------------------------------------------ hyper-parameter search (Sec. 3.6)
def _tune_inputs(n=2, N=384, d=32):
    return [_peaky_inputs(80 + i, N=N, d=d) for i in range(n)]


def test_tuner_choice_is_admissible_and_no_admissible_setting_is_sparser():
    inputs = _tune_inputs()
    taus, thetas, lams = [0.5, 0.8, 0.95], [-1.0, 0.3, 0.9], [-12.0, -6.0, -3.0]
    l1, l2 = 0.06, 0.08
    t = so.tune_head(inputs, taus, thetas, lams, l1, l2)
    # an independent sweep: full attention by the textbook formula on the dequantized operands
    def sweep(tau, theta, lam):
        sp, err = [], []
        for Q, K, V in inputs:
            Qd, Kd = so.dequantized_qk(Q, K)
            full = so.dense_attention(Qd, Kd, V)
            res, _ = so.spargeattn(Q, K, V, tau, theta, lam)
            sp.append(res.sparsity)
            err.append(np.abs(res.O - full).sum() / np.abs(full).sum())
        return np.mean(sp), np.max(err)
    table = {(a, b): sweep(a, b, -np.inf) for a in taus for b in thetas}
    admissible = {k: v for k, v in table.items() if v[1] < l1}
    assert admissible, "thresholds of this test must leave something admissible"
    s1, e1 = table[(t.tau, t.theta)]
    assert e1 < l1 and s1 == pytest.approx(max(v[0] for v in admissible.values()), abs=1e-12)
    np.testing.assert_allclose(t.stage1.reshape(-1, 2), [table[(a, b)] for a in taus for b in thetas], atol=1e-9)
    # stage 2 never lowers the sparsity, respects l2, and is the best admissible lambda
    lam_table = {c: sweep(t.tau, t.theta, c) for c in lams}
    adm2 = {c: v for c, v in lam_table.items() if v[1] < l2 and v[0] > s1}
    if adm2:
        assert t.lam in adm2 and t.sparsity == pytest.approx(max(v[0] for v in adm2.values()), abs=1e-12)
        assert t.l1 < l2
    else:
        assert t.lam == -np.inf and t.sparsity == pytest.approx(s1, abs=1e-12)
    assert t.sparsity >= s1 - 1e-12


def test_tuner_limits():
    inputs = _tune_inputs(n=2)
    taus, thetas, lams = [0.6, 0.9], [0.0, 0.5], [-8.0, -2.0]
    loose = so.tune_head(inputs, taus, thetas, lams, 10.0, 10.0)
    # every setting is admissible: the sparsest pair of the table and the sparsest lambda win
    assert loose.stage1[..., 0].max() == pytest.approx(loose.stage1[taus.index(loose.tau), thetas.index(loose.theta), 0])
    assert loose.sparsity == pytest.approx(max(loose.stage2[:, 0].max(), loose.stage1[..., 0].max()))
    tight = so.tune_head(inputs, taus, thetas, lams, 0.0, 0.0)
    # nothing is admissible: the most accurate pair, stage 2 off
    assert tight.lam == -np.inf
    assert tight.l1 == pytest.approx(tight.stage1[..., 1].min())
    mid = so.tune_head(inputs, taus, thetas, lams, 0.05, 0.05)
    assert tight.sparsity - 1e-12 <= mid.sparsity <= loose.sparsity + 1e-12
    # a lambda that never skips anything does not beat leaving the stage-2 test off: it is not taken
    same = so.tune_head(inputs, taus, thetas, [-1e9], 10.0, 10.0)
    assert same.lam == -np.inf and same.stage2[0, 0] == pytest.approx(same.sparsity)
    # a single-entry grid with tau = 1, theta > 1 is full attention: zero error, zero sparsity
    one = so.tune_head(inputs, [1.0], [2.0], [], 0.01, 0.01)
    assert one.sparsity == 0.0 and one.l1 == 0.0


# ------------------------------------------------------------------ HilbertCurve permutation (Sec. 3.7)
@pytest.mark.parametrize("bits,ndim", [(1, 2), (2, 2), (4, 2), (1, 3), (2, 3), (4, 3)])
def test_hilbert_curve_is_a_continuous_space_filling_walk(bits, ndim):
    c = so.hilbert_cells(bits, ndim)
    side = 1 << bits
    assert c.shape == (side ** ndim, ndim) and c.min() == 0 and c.max() == side - 1
    assert len({tuple(x) for x in c}) == len(c)                          # every cell once
    assert (np.abs(np.diff(c, axis=0)).sum(axis=1) == 1).all()           # neighbours along the curve touch
    assert not c[0].any()                                                # starts in the corner at the origin
    assert sorted(c[-1].tolist()) == [0] * (ndim - 1) + [side - 1]       # ends in the corner one edge away
    if bits > 1:
        # self-similarity: each 2^-ndim part of the curve fills one half-size sub-cube
        part = len(c) >> ndim
        for k in range(1 << ndim):
            sub = c[k * part:(k + 1) * part] >> (bits - 1)
            assert (sub == sub[0]).all()


def test_hilbert_order_of_a_grid_and_the_generators_encoder():
    from synth import hilbert_order as encode_side   # index computed per cell, then sorted: the other direction
    for grid in [(1, 6, 6), (3, 5, 7), (13, 30, 45), (8, 8), (2, 1, 3)]:
        p = so.hilbert_order(grid)
        assert sorted(p.tolist()) == list(range(int(np.prod(grid))))
        np.testing.assert_array_equal(p, encode_side(grid))
    # on a power-of-two grid consecutive tokens are grid neighbours
    p = so.hilbert_order((4, 8, 8))
    cells = np.stack(np.unravel_index(p[:], (4, 8, 8)), axis=1)
    # the enclosing cube is 8^3; inside the 4x8x8 slab the walk may leave and re-enter, but never jumps far on average
    assert np.abs(np.diff(cells, axis=0)).sum(axis=1).mean() < 1.5


def test_token_permutation_round_trip_and_attention_invariance():
    r = rng(90)
    N, d, off = 200, 16, 30
    perm = so.hilbert_order((2, 5, 9))                    # 90 visual tokens after 30 text tokens; 80 more behind
    X = r.standard_normal((N, d))
    Y = so.permute_tokens(X, perm, off)
    np.testing.assert_array_equal(Y[:off], X[:off])
    np.testing.assert_array_equal(Y[off + len(perm):], X[off + len(perm):])
    np.testing.assert_array_equal(Y[off + 7], X[off + perm[7]])
    np.testing.assert_array_equal(so.permute_tokens(Y, perm, off, inverse=True), X)
    # attention is invariant: permute Q, K, V alike, attend, un-permute the output (Sec. 3.7)
    Q, K, V = (r.standard_normal((N, d)) for _ in range(3))
    O = so.dense_attention(Q, K, V)
    Op = so.dense_attention(*(so.permute_tokens(T, perm, off) for T in (Q, K, V)))
    np.testing.assert_allclose(so.permute_tokens(Op, perm, off, inverse=True), O, rtol=0, atol=1e-12)


def test_mask_to_lut_literal_and_round_trip():
    """Index-list form of M_g: a literal case, and the properties that define it on random masks."""
    m = np.array([[1, 0, 1, 1], [0, 0, 0, 0], [0, 1, 0, 0]], dtype=np.uint8)
    lut, cnt = so.mask_to_lut(m)
    assert lut.tolist() == [[0, 2, 3, -1], [-1, -1, -1, -1], [1, -1, -1, -1]]
    assert cnt.tolist() == [3, 0, 1]
    rng = np.random.default_rng(5)
    m = (rng.random((37, 150)) < 0.3).astype(np.uint8)
    lut, cnt = so.mask_to_lut(m)
    assert np.array_equal(cnt, m.sum(axis=1))
    back = np.zeros_like(m)
    for i in range(m.shape[0]):
        js = lut[i, :cnt[i]]
        assert (np.diff(js) > 0).all() and (lut[i, cnt[i]:] == -1).all()
        back[i, js] = 1
    assert np.array_equal(back, m)
