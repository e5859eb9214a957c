"""CPU oracle for SpargeAttn's hot path (test infrastructure, NOT a product path).

Plain numpy, fp64 unless the text below says otherwise, one (batch, head) at a time, block by
block, in the order and notation of the paper's Algorithm 1.  Nothing here is blocked, fused or
re-ordered beyond what the algorithm states, and nothing is shared with the HIP kernels.
Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.

Notation (Sec. 3.1, Def. 1, Alg. 1): N tokens, head dim d, Q blocks of b_q = 128 rows, K/V blocks
of b_k = 64 rows, T_m = ceil(N/b_q), T_n = ceil(N/b_k); c_w = 4 "warps" split a Q block into row
groups I_w of 32 rows (Alg. 1 line 13).  Hyper-parameters tau, theta, lambda (Sec. 3.6).

Readings of the paper where it is silent or ambiguous (each also listed in the design notes):
  * CosSim (Sec. 3.2): mean cosine similarity over all ordered token pairs of a block (diagonal
    included); a zero token has zero cosine with everything.  The literal printed formula
    mean(XX^T/|max(XX^T)|) is available as cossim_blocks(..., literal=True) for comparison only.
  * S-hat carries the 1/sqrt(d) softmax scale (it is a compressed version of P = softmax(QK^T/sqrt d)).
  * TopCdf (Sec. 3.2): smallest descending prefix whose mass reaches tau * sum, i.e. an entry is kept
    iff the mass ranked strictly before it is < tau * sum; ties rank by ascending block index;
    entries with zero probability are never selected.
  * Causal attention: blocks entirely in the future are -inf in S-hat and 0 in the mask, even under
    the fix-block overrides; the K block that holds a Q block's first diagonal key is always kept.
  * Partial last blocks: statistics over valid rows only.
  * lambda test (Alg. 1 line 15): execute iff max over the row group's valid rows of
    (m_local - m_ij) > lambda; l is always updated (line 13 precedes line 15).
  * Quant (Alg. 1 line 3, SageAttention per-block INT8): symmetric, scale = amax/127, round half to
    even, K smoothed by its per-head token mean.  The fp32 operation sequence (one reciprocal per
    block, one multiplication per element) is spelled out in
    quantize_q / quantize_k and is part of the specification.
  * 16-bit rounding of P~ (not in the paper, whose Alg. 1 is in real arithmetic): P~ is rounded to the
    matrix unit's input type where it enters the P~V product.  By the rescaling identity of Sec. 3.1
    the maximum subtracted inside exp is a free reference: O and l may be kept relative to any
    per-row reference m_ref as long as both are rescaled when it moves, and O/l does not depend on
    it.  The loop below carries that reference explicitly.  ref_slack = 0 makes it the running
    maximum itself at every tile (the recurrence exactly as printed); ref_slack > 0 lets it lag:
    before a tile's softmax, if some row of a 32-row group has m - m_ref > ref_slack, the whole
    group's reference moves to the running maximum.  Only the rounding of P~ can tell the difference.
  * FP8 P~V (the paper only credits a SageAttention2-based kernel with it, footnote of Sec. 1; no
    formulas): pv_dtype = "fp8e4m3".  V is quantized per (head, channel) over all tokens to OCP E4M3
    (1-4-3 bits, bias 7, subnormals, largest finite value 448, round to nearest even):
    delta_V[c] = fp32(max_t |V[t,c]|) / 448 in fp32, V-hat = e4m3(fp32(V[t,c]) / delta_V[c]), a zero
    channel gives 0.  P~ is scaled by c_P = 448 * exp(-ref_slack) -- the largest value the lagging
    reference lets it take, mapped onto the largest E4M3 value -- and rounded to E4M3; products are
    exact and accumulate in fp64 here (fp32 on the GPU); O = (sum P~_q V-hat) * delta_V / (c_P * l), l
    from the unrounded P~ as always.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np

BQ = 128
BK = 64
ROW_GROUP = 32  # b_q / c_w with c_w = 4
NEG_INF = -np.inf
DONT_CARE_EPS = 1e-5


def nblocks(N: int, b: int) -> int:
    return (N + b - 1) // b


# ----------------------------------------------------------------------------------------------
# Stage 1: predictor (Sec. 3.2, Alg. 1 lines 4-6)
# ----------------------------------------------------------------------------------------------
def pool_blocks(X: np.ndarray, b: int) -> np.ndarray:
    """Block means over tokens (Alg. 1 line 4): X [N,d] -> [T,d]; a partial block averages its valid rows."""
    X = np.asarray(X, dtype=np.float64)
    T = nblocks(X.shape[0], b)
    out = np.empty((T, X.shape[1]), dtype=np.float64)
    for t in range(T):
        out[t] = X[t * b:(t + 1) * b].mean(axis=0)
    return out


def cossim_blocks(X: np.ndarray, b: int, literal: bool = False) -> np.ndarray:
    """Block self-similarity s = CosSim(X_t) (Alg. 1 line 5; Sec. 3.2): X [N,d] -> [T].

    Default reading: normalise every token, form the b x b Gram matrix of cosines, take its mean.
    literal=True evaluates the printed expression mean(XX^T / |max(XX^T)|) instead.
    """
    X = np.asarray(X, dtype=np.float64)
    T = nblocks(X.shape[0], b)
    out = np.empty(T, dtype=np.float64)
    for t in range(T):
        blk = X[t * b:(t + 1) * b]
        if literal:
            G = blk @ blk.T
            mx = abs(G.max())
            out[t] = (G / mx).mean() if mx > 0 else 0.0
            continue
        nrm = np.sqrt((blk * blk).sum(axis=1, keepdims=True))
        unit = np.divide(blk, nrm, out=np.zeros_like(blk), where=nrm > 0)
        out[t] = (unit @ unit.T).mean()
    return out


def block_causal_future(i: int, j: int) -> bool:
    """True if K block j lies entirely after every row of Q block i (nothing in it may be attended)."""
    return j * BK > i * BQ + (BQ - 1)


def compressed_map(q: np.ndarray, k: np.ndarray, s_k: np.ndarray, theta: float, scale: float,
                   causal: bool) -> np.ndarray:
    """P-hat = row softmax of S-hat = scale * q k^T with -inf columns (Alg. 1 lines 5-6).

    Columns of non-self-similar K blocks (s_k < theta) and, if causal, entirely-future blocks are
    -inf.  A row without any finite entry is all zeros.
    """
    S = scale * (q @ k.T)
    S[:, s_k < theta] = NEG_INF
    if causal:
        for i in range(S.shape[0]):
            for j in range(S.shape[1]):
                if block_causal_future(i, j):
                    S[i, j] = NEG_INF
    P = np.zeros_like(S)
    for i in range(S.shape[0]):
        row = S[i]
        mx = row.max()
        if mx == NEG_INF:
            continue
        e = np.exp(row - mx)
        P[i] = e / e.sum()
    return P


def top_cdf(p: np.ndarray, tau: float) -> Tuple[np.ndarray, np.ndarray]:
    """TopCdf(P-hat[i], tau) (Sec. 3.2).  Returns (mask, dont_care), both bool [n].

    Rank entries by (value descending, index ascending); entry at rank r is kept iff the mass of
    the entries ranked before it is < tau * sum(p) and its own value is > 0.
    dont_care marks entries whose decision sits within 1e-5 of the threshold: either their
    preceding mass is within 1e-5 of tau*sum, or their value is within 1e-5 (relative) of the
    smallest kept value while lying on the other side of the cut.
    """
    n = p.shape[0]
    order = np.lexsort((np.arange(n), -p))  # primary key -p, ties by index
    sp = p[order]
    total = sp.sum()
    before = np.concatenate(([0.0], np.cumsum(sp)[:-1]))
    keep_sorted = (before < tau * total) & (sp > 0)
    mask = np.zeros(n, dtype=bool)
    mask[order] = keep_sorted
    dc_sorted = (np.abs(before - tau * total) <= DONT_CARE_EPS) & (sp > 0)
    if keep_sorted.any():
        p_cut = sp[keep_sorted].min()
        near = np.abs(sp - p_cut) <= DONT_CARE_EPS * max(p_cut, 1e-30)
        # values tied (to 1e-5) with the cut value: which of them fall before the cut depends on
        # rounding of the ranking, unless all of them are on the same side
        if near.any() and not (keep_sorted[near].all() or (~keep_sorted[near]).all()):
            dc_sorted |= near
    dont_care = np.zeros(n, dtype=bool)
    dont_care[order] = dc_sorted
    return mask, dont_care


@dataclass
class Prediction:
    mask: np.ndarray        # uint8 [T_m, T_n], 1 = compute the block (M_g)
    dont_care: np.ndarray   # bool  [T_m, T_n], decision within 1e-5 of a threshold
    sim_q: np.ndarray       # [T_m]
    sim_k: np.ndarray       # [T_n]
    pooled_q: np.ndarray    # [T_m, d]
    pooled_k: np.ndarray    # [T_n, d]
    p_hat: np.ndarray       # [T_m, T_n]


def predict(Q: np.ndarray, K: np.ndarray, tau: float, theta: float, scale: Optional[float] = None,
            causal: bool = False) -> Prediction:
    """Stage-1 block mask M_g of one head (Alg. 1 lines 4-6; Sec. 3.2, Eq. for M_g overrides)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    N, d = Q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    q = pool_blocks(Q, BQ)
    k = pool_blocks(K, BK)
    s_q = cossim_blocks(Q, BQ)
    s_k = cossim_blocks(K, BK)
    P = compressed_map(q, k, s_k, theta, scale, causal)
    Tm, Tn = P.shape
    mask = np.zeros((Tm, Tn), dtype=bool)
    dc = np.zeros((Tm, Tn), dtype=bool)
    for i in range(Tm):
        mask[i], dc[i] = top_cdf(P[i], tau)
    # fix-block overrides: non-self-similar Q rows / K columns are always computed
    fix_q = s_q < theta
    fix_k = s_k < theta
    mask[fix_q, :] = True
    mask[:, fix_k] = True
    dc[fix_q, :] = False
    dc[:, fix_k] = False
    # a similarity within 1e-5 of theta makes the row (Q) or the whole head (K) undecidable
    near_q = np.abs(s_q - theta) <= DONT_CARE_EPS
    near_k = np.abs(s_k - theta) <= DONT_CARE_EPS
    dc[near_q, :] = True
    if near_k.any():
        dc[:, :] = True
    if causal:
        for i in range(Tm):
            for j in range(Tn):
                if block_causal_future(i, j):
                    mask[i, j] = False
                    dc[i, j] = False
            jd = (i * BQ) // BK  # block holding the first row's own position
            mask[i, jd] = True
            dc[i, jd] = False
    return Prediction(mask.astype(np.uint8), dc, s_q, s_k, q, k, P)


def mask_to_lut(mask: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """The block mask M_g (Sec. 3.2, Def. 2) of one head as an index list: row i of `lut` holds the key
    blocks j with M_g[i, j] = 1 in ascending order, then -1 up to T_n entries; count[i] is their number.
    (The loop of Alg. 1 visits exactly these j, in this order, for Q block i.)"""
    mask = np.asarray(mask)
    Tm, Tn = mask.shape
    lut = np.full((Tm, Tn), -1, dtype=np.int32)
    count = np.zeros(Tm, dtype=np.int32)
    for i in range(Tm):
        n = 0
        for j in range(Tn):
            if mask[i, j]:
                lut[i, n] = j
                n += 1
        count[i] = n
    return lut, count


# ----------------------------------------------------------------------------------------------
# Quant (Alg. 1 line 3): per-block symmetric INT8, K smoothed by its token mean
# ----------------------------------------------------------------------------------------------
def _quant_blocks(X32: np.ndarray, b: int) -> Tuple[np.ndarray, np.ndarray]:
    """Per-block INT8 quantization of an fp32 matrix, fp32 arithmetic with these rounding points:
    amax = max|x| over the block's valid rows; delta = fl32(amax/127); r = fl32(127/amax);
    x_hat = rint_half_even(fl32(x*r)); a zero block gives x_hat = 0, delta = 0."""
    assert X32.dtype == np.float32
    N = X32.shape[0]
    T = nblocks(N, b)
    Xq = np.zeros(X32.shape, dtype=np.int8)
    delta = np.zeros(T, dtype=np.float32)
    c127 = np.float32(127.0)
    for t in range(T):
        blk = X32[t * b:(t + 1) * b]
        amax = np.float32(np.abs(blk).max())
        if amax == 0:
            continue
        delta[t] = amax / c127
        r = c127 / amax
        y = blk * r  # one correctly rounded fp32 multiplication per element
        assert y.dtype == np.float32 and np.abs(y).max() <= 127.5
        Xq[t * b:(t + 1) * b] = np.rint(y).astype(np.int8)  # rint: ties to even
    return Xq, delta


def quantize_exact(X32: np.ndarray, b: int) -> Tuple[np.ndarray, np.ndarray]:
    """What Quant rounds to in exact arithmetic: x_hat = round-half-even(127 x / amax) per block, with no
    intermediate rounding, and a flag for the elements whose quotient lies within 2^-15 of a half-integer.

    Integer arithmetic throughout: an fp32 number is m * 2^e with a 24-bit integer m, so
    127 x / amax = (127 m_x) / (m_a * 2^(e_a - e_x)) is a ratio of two integers that fit 64 bits whenever the
    quotient is not negligibly small (below 2^-8 it rounds to 0 and is nowhere near a tie).
    Outside the flag every sequence of correctly rounded fp32 operations whose relative error stays below
    2^-22 -- in particular fl(x * fl(127/amax)), error < 2^-23 (1 + 2^-24), i.e. < 2^-16 absolute on a
    quotient of at most 127 -- rounds to the same integer.  Returns (x_hat int8, near_tie bool)."""
    assert X32.dtype == np.float32
    N = X32.shape[0]
    T = nblocks(N, b)
    Xq = np.zeros(X32.shape, dtype=np.int8)
    near = np.zeros(X32.shape, dtype=bool)
    for t in range(T):
        blk = X32[t * b:(t + 1) * b]
        amax = np.float32(np.abs(blk).max())
        if amax == 0:
            continue
        fm, fe = np.frexp(blk.astype(np.float64))             # x = fm * 2^fe, |fm| in [0.5, 1): exact
        mx = np.rint(fm * 2.0 ** 24).astype(np.int64)          # 24-bit integer significand (signed)
        ex = fe.astype(np.int64) - 24
        am, ae = np.frexp(np.float64(amax))
        ma, ea = int(round(am * 2.0 ** 24)), int(ae) - 24
        sh = ea - ex                                            # >= 0 up to the significands' ratio
        tiny = (sh > 33) | (mx == 0)                            # |127 x / amax| < 2^-8: rounds to 0, far from a tie
        sh = np.where(tiny, 0, sh)
        num = 127 * np.abs(mx)
        num = np.where(sh < 0, num << np.maximum(-sh, 0), num)  # (sh = -1 can occur when m_x > m_a)
        den = np.int64(ma) << np.maximum(sh, 0)
        n = num // den
        rem2 = 2 * (num - n * den)
        up = (rem2 > den) | ((rem2 == den) & (n % 2 == 1))      # beyond the half, or a tie with n odd
        mag = np.where(tiny, 0, n + up)
        Xq[t * b:(t + 1) * b] = (np.sign(mx) * mag).astype(np.int8)
        near[t * b:(t + 1) * b] = ~tiny & (np.abs(rem2 - den) < (den >> 14))   # |frac - 1/2| < 2^-15
    return Xq, near


def quantize_q(Q: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Q-hat, delta_Q per 128-row block.  Q holds 16-bit values, taken exactly into fp32."""
    return _quant_blocks(np.asarray(Q, dtype=np.float32), BQ)


def k_mean(K: np.ndarray) -> np.ndarray:
    """Per-head token mean of K: the exactly rounded fp64 sum over tokens, divided by N in fp64,
    then rounded to fp32."""
    K = np.asarray(K, dtype=np.float64)
    N, d = K.shape
    s = np.array([math.fsum(K[:, c]) for c in range(d)], dtype=np.float64)
    return (s / float(N)).astype(np.float32)


def quantize_k(K: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """K-hat, delta_K per 64-row block, and the mean that was removed: K' = fl32(K - mean)."""
    mean = k_mean(K)
    Ks = np.asarray(K, dtype=np.float32) - mean[None, :]
    Kq, delta = _quant_blocks(Ks, BK)
    return Kq, delta, mean


# ----------------------------------------------------------------------------------------------
# rounding to the 16-bit type that feeds the P~V product / holds the output
# ----------------------------------------------------------------------------------------------
def round16(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to fp16 or bf16 (nearest, ties to even), returned as fp64."""
    if dtype == "fp16":
        return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        f = np.asarray(x, dtype=np.float64).astype(np.float32)
        u = np.ascontiguousarray(f).view(np.uint32).astype(np.uint64)
        r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
        return r.astype(np.uint32).view(np.float32).astype(np.float64).reshape(f.shape)
    if dtype == "none":
        return np.asarray(x, dtype=np.float64)
    raise ValueError(dtype)


E4M3_MAX = 448.0


def round_e4m3(x: np.ndarray) -> np.ndarray:
    """Round to the nearest OCP FP8 E4M3 value (ties to even), returned as fp64.

    E4M3: 1 sign, 4 exponent (bias 7), 3 mantissa bits; normal values 2^e (1 + m/8), e in [-6, 8],
    the code with all exponent and mantissa bits set is NaN, so the largest finite value is 448;
    subnormals m/8 * 2^-6.  Inside one binade the values are multiples of 2^(e-3): rounding the
    multiple to the nearest integer, ties to even, is round-to-nearest-even on the mantissa.
    Inputs must not round past 448 (the format has no infinity; the method never produces them).
    """
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.clip(e, -6, 8)
    step = np.exp2(e - 3)
    r = np.rint(a / step) * step
    if np.any(r > E4M3_MAX):
        raise ValueError("value rounds past the largest finite E4M3 number")
    return np.copysign(r, x)


def encode_e4m3(x: np.ndarray) -> np.ndarray:
    """The byte codes (sign << 7 | exponent << 3 | mantissa) of round_e4m3(x)."""
    r = round_e4m3(x)
    a = np.abs(r)
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    normal = a >= 2.0 ** -6
    E = np.where(normal, e + 7, 0).astype(np.int64)
    M = np.where(normal, np.rint((a / np.exp2(e) - 1.0) * 8), np.rint(a * 2.0 ** 9)).astype(np.int64)
    sign = (np.signbit(r)).astype(np.int64)
    return ((sign << 7) | (E << 3) | M).astype(np.uint8)


def quantize_v_fp8(V: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Per-channel E4M3 quantization of one head's V [N, d]: (V-hat as fp64 grid values, delta_V fp32 [d]).
    The division runs in fp32, as stated in the module header."""
    V32 = np.asarray(V, dtype=np.float32)
    amax = np.abs(V32).max(axis=0)
    delta = (amax / np.float32(E4M3_MAX)).astype(np.float32)
    safe = np.where(delta > 0, delta, np.float32(1.0)).astype(np.float32)
    scaled = (V32 / safe[None, :]).astype(np.float32)
    Vq = round_e4m3(np.where(delta[None, :] > 0, scaled, np.float32(0.0)).astype(np.float64))
    return Vq, delta


# ----------------------------------------------------------------------------------------------
# Stage 2: sparse flash loop with the lambda skip (Alg. 1 lines 7-20; Sec. 3.1, 3.3, 3.4)
# ----------------------------------------------------------------------------------------------
@dataclass
class AttnResult:
    O: np.ndarray            # fp64 [N, d]: O_i = diag(l)^-1 O_ij, not rounded
    qk_tiles: int            # Q_iK_j^T block products executed
    pv_groups: int           # P~V row-group products executed (4 per tile when nothing is skipped)
    valid_tiles: int         # tiles a full (causal) attention would need
    valid_groups: int        # row-group products of those tiles that have a visible (row, key) pair
    zero_rows: int           # rows that ended with l = 0 (must be 0 for a usable mask)
    # per (Q block, row group): how close the stage-2 statistic max(m_local - m_ij) came to lambda over the
    # row's tiles (inf when lambda = -inf or nothing was decided): a decision closer than the arithmetic of
    # an implementation can resolve is not pinned, and the rows of that group inherit the doubt
    lam_margin: Optional[np.ndarray] = None

    @property
    def sparsity(self) -> float:
        """Skipped Q_iK_j^T plus P~V products over all of them (Sec. 4.1 'Sparsity')."""
        return 1.0 - 0.5 * (self.qk_tiles / self.valid_tiles + self.pv_groups / self.valid_groups)


def sparse_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, mask: Optional[np.ndarray],
                     lam: float = -np.inf, scale: Optional[float] = None, causal: bool = False,
                     quant: bool = True, pv_dtype: str = "none",
                     q_blocks: Optional[Sequence[int]] = None, ref_slack: float = 0.0) -> AttnResult:
    """Algorithm 1's loop for one head.

    q_blocks: only these Q block indices i are processed (their rows of O and their share of the
    counters); the rest of O stays 0.  Used to sample rows of a long sequence.

    quant=True: S_ij = (Q-hat_i K-hat_j^T, exact integers) * delta_Q[i] * delta_K[j] * scale with the
    quantizers above (K smoothed).  quant=False: S_ij = scale * Q_i K_j^T in fp64.
    pv_dtype: "fp16"/"bf16" rounds P~ to that type before the P~V product (the 16-bit matrix
    unit's input); "fp8e4m3" is the FP8 product described in the module header; the row sum l always
    uses the unrounded P~.  mask=None means all ones.
    ref_slack (natural-log units): how far the running maximum may run ahead of the reference that
    exp subtracts (see the module header); 0 = the recurrence of Alg. 1 lines 12-16 as printed.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    N, d = Q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    Tm, Tn = nblocks(N, BQ), nblocks(N, BK)
    if quant:
        Qh, dQ = quantize_q(Q)
        Kh, dK, _ = quantize_k(K)
        Qh = Qh.astype(np.float64)
        Kh = Kh.astype(np.float64)
    fp8 = pv_dtype == "fp8e4m3"
    if fp8:
        V, delta_V = quantize_v_fp8(V)           # from here on V holds V-hat
        c_P = E4M3_MAX * math.exp(-ref_slack)
    O = np.zeros((N, d), dtype=np.float64)
    qk_tiles = pv_groups = valid_tiles = valid_groups = zero_rows = 0
    lam_margin = np.full((Tm, BQ // ROW_GROUP), np.inf)
    for i in (range(Tm) if q_blocks is None else q_blocks):
        r0, r1 = i * BQ, min((i + 1) * BQ, N)
        nr = r1 - r0
        rows = np.arange(r0, r1)
        m = np.full(nr, NEG_INF)      # running maximum m_ij (Alg. 1 line 12)
        m_ref = np.full(nr, NEG_INF)  # reference maximum that O and l are relative to
        l = np.zeros(nr)
        Oi = np.zeros((nr, d))
        for j in range(Tn):
            if causal and block_causal_future(i, j):
                continue
            valid_tiles += 1
            c0, c1 = j * BK, min((j + 1) * BK, N)
            for g0 in range(0, nr, ROW_GROUP):
                last_row = r0 + min(g0 + ROW_GROUP, nr) - 1
                if not causal or c0 <= last_row:
                    valid_groups += 1
            if mask is not None and mask[i, j] == 0:
                continue
            qk_tiles += 1
            if quant:
                S = (Qh[r0:r1] @ Kh[c0:c1].T) * (float(dQ[i]) * float(dK[j]) * scale)
            else:
                S = (Q[r0:r1] @ K[c0:c1].T) * scale
            if causal:
                cols = np.arange(c0, c1)
                S = np.where(cols[None, :] > rows[:, None], NEG_INF, S)
            m_local = S.max(axis=1)
            m_new = np.maximum(m, m_local)
            # move the reference of every row group in which some row's maximum has run ahead of it
            # by more than ref_slack: O and l are rescaled by exp(m_ref_old - m_ref_new) (line 13, 16)
            moved = np.zeros(nr, dtype=bool)
            for g0 in range(0, nr, ROW_GROUP):
                g1 = min(g0 + ROW_GROUP, nr)
                with np.errstate(invalid="ignore"):
                    ahead = m_new[g0:g1] - m_ref[g0:g1]     # nan where both are -inf: no move
                if np.any(ahead > ref_slack):
                    with np.errstate(invalid="ignore"):
                        f = np.exp(m_ref[g0:g1] - m_new[g0:g1])
                    f = np.where(m_new[g0:g1] > NEG_INF, f, 1.0)
                    l[g0:g1] *= f
                    Oi[g0:g1] *= f[:, None]
                    m_ref[g0:g1] = m_new[g0:g1]
                    moved[g0:g1] = True
            live = m_ref > NEG_INF
            m_safe = np.where(live, m_ref, 0.0)
            P = np.exp(S - m_safe[:, None])          # exp(-inf) = 0 for masked entries
            Pr = round_e4m3(P * c_P) if fp8 else round16(P, pv_dtype)
            l = l + P.sum(axis=1)                    # line 13: the row sum sees the unrounded P~
            for g0 in range(0, nr, ROW_GROUP):
                g1 = min(g0 + ROW_GROUP, nr)
                with np.errstate(invalid="ignore"):
                    diff = np.where(m_local[g0:g1] > NEG_INF, m_local[g0:g1] - m_new[g0:g1], NEG_INF)
                if np.isfinite(lam) and diff.max() > NEG_INF:
                    lam_margin[i, g0 // ROW_GROUP] = min(lam_margin[i, g0 // ROW_GROUP], abs(diff.max() - lam))
                if diff.max() > lam:
                    pv_groups += 1
                    Oi[g0:g1] = Oi[g0:g1] + Pr[g0:g1] @ V[c0:c1]
                else:
                    # a skipped group never has a changed running max, so nothing was rescaled
                    assert not moved[g0:g1].any()
            m = m_new
        dead = l == 0
        zero_rows += int(dead.sum())
        if fp8:
            Oi = Oi * delta_V.astype(np.float64)[None, :] / c_P
        O[r0:r1] = np.where(dead[:, None], 0.0, Oi / np.where(dead, 1.0, l)[:, None])
    return AttnResult(O, qk_tiles, pv_groups, valid_tiles, valid_groups, zero_rows, lam_margin)


def dense_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: Optional[float] = None,
                    causal: bool = False, block_mask: Optional[np.ndarray] = None) -> np.ndarray:
    """O = softmax(QK^T * scale) V on the full N x N score matrix (Sec. 3.1), fp64.

    block_mask (Def. 2): -inf is written over every score of a block with M_g[i,j] = 0.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    N, d = Q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    S = (Q @ K.T) * scale
    if causal:
        S = np.where(np.arange(N)[None, :] > np.arange(N)[:, None], NEG_INF, S)
    if block_mask is not None:
        full = np.repeat(np.repeat(block_mask.astype(bool), BQ, axis=0), BK, axis=1)[:N, :N]
        S = np.where(full, S, NEG_INF)
    mx = S.max(axis=1, keepdims=True)
    E = np.exp(S - mx)
    return (E / E.sum(axis=1, keepdims=True)) @ V


def dequantized_qk(Q: np.ndarray, K: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Q-hat*delta_Q and K-hat*delta_K as fp64 matrices (what the INT8 product effectively multiplies)."""
    Qh, dQ = quantize_q(Q)
    Kh, dK, _ = quantize_k(K)
    Qd = Qh.astype(np.float64) * np.repeat(dQ.astype(np.float64), BQ)[:Qh.shape[0], None]
    Kd = Kh.astype(np.float64) * np.repeat(dK.astype(np.float64), BK)[:Kh.shape[0], None]
    return Qd, Kd


def rel_l1(O: np.ndarray, O_ref: np.ndarray) -> float:
    """Relative L1 distance sum|O - O'| / sum|O| with O the reference (Sec. 3.6)."""
    O = np.asarray(O, dtype=np.float64)
    O_ref = np.asarray(O_ref, dtype=np.float64)
    return float(np.abs(O - O_ref).sum() / np.abs(O_ref).sum())


def spargeattn(Q: np.ndarray, K: np.ndarray, V: np.ndarray, tau: float, theta: float, lam: float,
               causal: bool = False, scale: Optional[float] = None, quant: bool = True,
               pv_dtype: str = "none", ref_slack: float = 0.0) -> Tuple[AttnResult, Prediction]:
    """The whole of Algorithm 1 for one head: Quant, predict M_g, masked loop with the lambda skip."""
    pred = predict(Q, K, tau, theta, scale, causal)
    res = sparse_attention(Q, K, V, pred.mask, lam, scale, causal, quant, pv_dtype, ref_slack=ref_slack)
    return res, pred


# ----------------------------------------------------------------------------------------------
# Hyper-parameter determination for one head (Sec. 3.6)
# ----------------------------------------------------------------------------------------------
@dataclass
class TuneResult:
    tau: float
    theta: float
    lam: float               # -inf: no value of the lambda grid was admissible, stage 2 stays off
    sparsity: float          # mean over the inputs, with (tau, theta, lam)
    l1: float                # worst input's relative L1 against full attention, with (tau, theta, lam)
    stage1: np.ndarray       # [n_tau, n_theta, 2]: mean sparsity, worst relative L1 of every (tau, theta)
    stage2: np.ndarray       # [n_lambda, 2]: the same for every lambda at the chosen (tau, theta)


def tune_head(inputs: Sequence[Tuple[np.ndarray, np.ndarray, np.ndarray]], tau_grid: Sequence[float],
              theta_grid: Sequence[float], lam_grid: Sequence[float], l1: float, l2: float,
              causal: bool = False, scale: Optional[float] = None, pv_dtype: str = "none",
              ref_slack: float = 0.0) -> TuneResult:
    """Sec. 3.6 for one attention head and a handful of inputs (Q, K, V).

    The error of a setting is L1 = sum|O - O'| / sum|O| with O the full attention computed the same way
    (same quantization and rounding, every block kept, nothing skipped) and O' the sparse one.
    First the (tau, theta) grid with stage 2 off: among the pairs whose L1 stays below l1 on every
    input, the one with the largest sparsity (mean over the inputs).  Then the lambda grid at that pair:
    among the values whose L1 stays below l2 on every input, the one with the largest sparsity, if
    that beats leaving stage 2 off.
    Readings (the paper says "constrain the error across five inputs" and no more): the constraint
    binds the worst input, the objective is the mean; ties keep the earlier grid entry (tau outer,
    theta inner); if no pair is admissible the pair with the smallest worst-input L1 is taken.
    Outputs are compared after rounding to pv_dtype when that is a 16-bit type (what a kernel stores).
    """
    def out(res):
        return round16(res.O, pv_dtype) if pv_dtype in ("fp16", "bf16") else res.O

    refs = [out(sparse_attention(Q, K, V, None, -np.inf, scale, causal, True, pv_dtype, ref_slack=ref_slack))
            for (Q, K, V) in inputs]

    def evaluate(tau, theta, lam):
        sp, err = [], []
        for (Q, K, V), ref in zip(inputs, refs):
            res, _ = spargeattn(Q, K, V, tau, theta, lam, causal, scale, True, pv_dtype, ref_slack)
            sp.append(res.sparsity)
            err.append(rel_l1(out(res), ref))
        return float(np.mean(sp)), float(np.max(err))

    stage1 = np.zeros((len(tau_grid), len(theta_grid), 2))
    for a, tau in enumerate(tau_grid):
        for b, theta in enumerate(theta_grid):
            stage1[a, b] = evaluate(tau, theta, -np.inf)
    flat = stage1.reshape(-1, 2)
    ok = flat[:, 1] < l1
    if ok.any():
        best = int(np.flatnonzero(ok)[np.argmax(flat[ok, 0])])     # argmax keeps the first of equals
    else:
        best = int(np.argmin(flat[:, 1]))
    a, b = divmod(best, len(theta_grid))
    tau, theta = tau_grid[a], theta_grid[b]
    sparsity, err = flat[best]
    lam = -np.inf
    stage2 = np.zeros((len(lam_grid), 2))
    for c, cand in enumerate(lam_grid):
        stage2[c] = evaluate(tau, theta, cand)
        if stage2[c, 1] < l2 and stage2[c, 0] > sparsity:
            lam, (sparsity, err) = cand, stage2[c]
    return TuneResult(float(tau), float(theta), float(lam), float(sparsity), float(err), stage1, stage2)


# ----------------------------------------------------------------------------------------------
# HilbertCurve permutation (Sec. 3.7): visual tokens of a T x H x W grid flattened along a Hilbert curve
# ----------------------------------------------------------------------------------------------
def hilbert_cells(bits: int, ndim: int) -> np.ndarray:
    """The cells of the 2^bits hyper-cube in the order a Hilbert curve visits them: int64 [2^(bits*ndim), ndim].

    Decoding direction of Skilling's transform ("Programming the Hilbert curve", 2004): the index's
    bits are dealt out to the axes (most significant bit to axis 0), the Gray code is undone, and
    from the second-finest level upwards the low bits of axis 0 and axis i are exchanged or inverted.
    """
    total = 1 << (bits * ndim)
    h = np.arange(total, dtype=np.int64)
    X = [np.zeros(total, dtype=np.int64) for _ in range(ndim)]
    for pos in range(bits * ndim):                    # pos counts index bits from the most significant one
        bit = (h >> (bits * ndim - 1 - pos)) & 1
        X[pos % ndim] |= bit << (bits - 1 - pos // ndim)
    top = 2 << (bits - 1)
    t = X[ndim - 1] >> 1                              # Gray decode
    for i in range(ndim - 1, 0, -1):
        X[i] ^= X[i - 1]
    X[0] ^= t
    q = 2
    while q != top:                                   # undo the exchanges, coarse levels last
        p = q - 1
        for i in range(ndim - 1, -1, -1):
            hit = (X[i] & q) != 0
            if i == 0:
                X[0] = np.where(hit, X[0] ^ p, X[0])
            else:
                swap = (X[0] ^ X[i]) & p
                X[0], X[i] = np.where(hit, X[0] ^ p, X[0] ^ swap), np.where(hit, X[i], X[i] ^ swap)
        q <<= 1
    return np.stack(X, axis=1)


def hilbert_order(grid: Sequence[int]) -> np.ndarray:
    """Permutation p: sequence position s holds the row-major cell p[s] of the grid (T, H, W).
    The curve fills the enclosing 2^b cube; cells outside the grid are skipped."""
    grid = tuple(int(g) for g in grid)
    bits = max(1, int(math.ceil(math.log2(max(grid)))))
    cells = hilbert_cells(bits, len(grid))
    inside = np.all(cells < np.array(grid)[None, :], axis=1)
    cells = cells[inside]
    return np.ravel_multi_index(tuple(cells[:, i] for i in range(len(grid))), grid).astype(np.int64)


def permute_tokens(X: np.ndarray, perm: np.ndarray, offset: int = 0, inverse: bool = False) -> np.ndarray:
    """Y[offset + s] = X[offset + perm[s]] (inverse: Y[offset + perm[s]] = X[offset + s]); tokens outside
    [offset, offset + len(perm)) keep their place (App. A: only the visual tokens are permuted)."""
    Y = np.array(X, copy=True)
    L = len(perm)
    if inverse:
        Y[offset + np.asarray(perm)] = X[offset:offset + L]
    else:
        Y[offset:offset + L] = X[offset + np.asarray(perm)]
    return Y
