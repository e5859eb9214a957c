"""Are the pins tight?  Each case below plants ONE plausible mistake in a copy of the oracle's source (a dropped
term, a wrong sign or index, a swapped comparison, another rounding rule) and runs the pins of
test_oracle_pins.py against that copy: some pin must fail.  The mistakes live in a module object built here, on
the CPU; the oracle on disk and the HIP path are untouched."""
import inspect
import itertools
import os
import types

import pytest

import tests.test_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = open(os.path.join(ROOT, "oracle", "sparge_oracle.py")).read()

# (what the mistake is, text in the oracle, what replaces it)
MUTATIONS = [
    ("pooling sums instead of averaging", "out[t] = X[t * b:(t + 1) * b].mean(axis=0)", "out[t] = X[t * b:(t + 1) * b].sum(axis=0)"),
    ("self-similarity leaves the diagonal pairs out", "out[t] = (unit @ unit.T).mean()",
     "out[t] = ((unit @ unit.T).sum() - len(blk)) / max(len(blk) * (len(blk) - 1), 1)"),
    ("compressed logits without the softmax scale", "S = scale * (q @ k.T)", "S = 1.0 * (q @ k.T)"),
    ("self-similar instead of non-self-similar K columns masked", "S[:, s_k < theta] = NEG_INF", "S[:, s_k > theta] = NEG_INF"),
    ("block-causal rule off by a block", "return j * BK > i * BQ + (BQ - 1)", "return j * BK > i * BQ"),
    ("TopCdf keeps on equality", "keep_sorted = (before < tau * total) & (sp > 0)", "keep_sorted = (before <= tau * total) & (sp > 0)"),
    ("TopCdf ranks ties by descending index", "order = np.lexsort((np.arange(n), -p))", "order = np.lexsort((-np.arange(n), -p))"),
    ("TopCdf uses the inclusive cumulative sum (the printed listing)", "before = np.concatenate(([0.0], np.cumsum(sp)[:-1]))", "before = np.cumsum(sp)"),
    ("TopCdf may select zero-probability entries", "keep_sorted = (before < tau * total) & (sp > 0)", "keep_sorted = (before < tau * total)"),
    ("K-column override forgotten", "    mask[:, fix_k] = True\n", "    pass\n"),
    ("Q-row override forgotten", "    mask[fix_q, :] = True\n", "    pass\n"),
    ("forced causal block off by one", "jd = (i * BQ) // BK  #", "jd = (i * BQ) // BK + 1  #"),
    ("near-theta band applied to the K column only", "        dc[:, :] = True\n", "        dc[:, near_k] = True\n"),
    ("quantization scale amax/128", "delta[t] = amax / c127", "delta[t] = amax / np.float32(128.0)"),
    ("quantizer rounds half up", "Xq[t * b:(t + 1) * b] = np.rint(y).astype(np.int8)", "Xq[t * b:(t + 1) * b] = np.floor(y + np.float32(0.5)).astype(np.int8)"),
    ("exact quantizer resolves ties upwards", "up = (rem2 > den) | ((rem2 == den) & (n % 2 == 1))", "up = rem2 >= den"),
    ("K mean divides by N - 1", "return (s / float(N)).astype(np.float32)", "return (s / float(N - 1)).astype(np.float32)"),
    ("K mean added instead of removed", "Ks = np.asarray(K, dtype=np.float32) - mean[None, :]", "Ks = np.asarray(K, dtype=np.float32) + mean[None, :]"),
    ("dequantization forgets delta_K", "* (float(dQ[i]) * float(dK[j]) * scale)", "* (float(dQ[i]) * scale)"),
    ("causal mask hides the diagonal", "S = np.where(cols[None, :] > rows[:, None], NEG_INF, S)", "S = np.where(cols[None, :] >= rows[:, None], NEG_INF, S)"),
    ("running maximum forgets the past", "m_new = np.maximum(m, m_local)", "m_new = m_local"),
    ("row sum over the rounded P~", "l = l + P.sum(axis=1)", "l = l + Pr.sum(axis=1)"),
    ("stage-2 test executes on equality", "if diff.max() > lam:", "if diff.max() >= lam:"),
    ("stage-2 test per Q block instead of per row group", "if diff.max() > lam:",
     "if np.where(m_local > NEG_INF, m_local - m_new, NEG_INF).max() > lam:"),
    ("row sum not updated for skipped groups", "                    assert not moved[g0:g1].any()",
     "                    l[g0:g1] -= P[g0:g1].sum(axis=1)"),
    ("P~V with the keys of the tile reversed", "Oi[g0:g1] = Oi[g0:g1] + Pr[g0:g1] @ V[c0:c1]", "Oi[g0:g1] = Oi[g0:g1] + Pr[g0:g1] @ V[c0:c1][::-1]"),
    ("O not rescaled when the reference moves", "                    Oi[g0:g1] *= f[:, None]\n", ""),
    ("sparsity counts tiles only", "return 1.0 - 0.5 * (self.qk_tiles / self.valid_tiles + self.pv_groups / self.valid_groups)",
     "return 1.0 - self.qk_tiles / self.valid_tiles"),
    ("bf16 rounding truncates", "r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16", "r = (u >> 16) << 16"),
    ("E4M3 without subnormals one binade too deep", "e = np.clip(e, -6, 8)", "e = np.clip(e, -7, 8)"),
    ("FP8 V scale maps onto 240", "delta = (amax / np.float32(E4M3_MAX)).astype(np.float32)", "delta = (amax / np.float32(240.0)).astype(np.float32)"),
    ("relative L1 normalised by the wrong tensor", "return float(np.abs(O - O_ref).sum() / np.abs(O_ref).sum())",
     "return float(np.abs(O - O_ref).sum() / (np.abs(O).sum() + np.abs(O_ref).sum()))"),
    ("tuner constrains the mean error", "return float(np.mean(sp)), float(np.max(err))", "return float(np.mean(sp)), float(np.mean(err))"),
    ("tuner maximises the best input's sparsity", "return float(np.mean(sp)), float(np.max(err))", "return float(np.max(sp)), float(np.max(err))"),
    ("Hilbert curve without the Gray decoding", "    X[0] ^= t\n", "    pass\n"),
    ("inverse token permutation equals the forward one", "Y[offset + np.asarray(perm)] = X[offset:offset + L]", "Y[offset:offset + L] = X[offset + np.asarray(perm)]"),
    ("row groups that see no key of a causal tile counted as work", "if not causal or c0 <= last_row:", "if True:"),
    ("index list stores the position instead of the block", "                lut[i, n] = j\n", "                lut[i, n] = n\n"),
    ("index list count is the last kept block", "        count[i] = n\n", "        count[i] = lut[i, max(n - 1, 0)]\n"),
    ("reference moves only when every row of the group ran ahead", "if np.any(ahead > ref_slack):", "if np.all(ahead > ref_slack):"),
    ("reference moves per row instead of per row group", "                    m_ref[g0:g1] = m_new[g0:g1]\n",
     "                    m_ref[g0:g1] = np.where(ahead > ref_slack, m_new[g0:g1], m_ref[g0:g1])\n"),
    ("FP8 scale of P~ ignores the slack of the reference", "c_P = E4M3_MAX * math.exp(-ref_slack)", "c_P = E4M3_MAX"),
    ("FP8 output forgets the channel scales", "Oi = Oi * delta_V.astype(np.float64)[None, :] / c_P", "Oi = Oi / c_P"),
    ("rows without any key are not reported", "zero_rows += int(dead.sum())", "zero_rows += 0"),
    ("distance from lambda measured to the row maximum only", "abs(diff.max() - lam))", "abs(m_local[g0:g1].max() - lam))"),
    ("softmax of the compressed map without subtracting the maximum", "e = np.exp(row - mx)", "e = np.exp(np.minimum(row, 700.0))"),
    ("fix rows stay flagged as undecided", "    dc[fix_q, :] = False\n", "    pass\n"),
    ("E4M3 byte codes with the exponent bias off by one", "E = np.where(normal, e + 7, 0).astype(np.int64)", "E = np.where(normal, e + 8, 0).astype(np.int64)"),
    ("near-tie band of the exact quantizer sixteen times too wide", "(np.abs(rem2 - den) < (den >> 14))", "(np.abs(rem2 - den) < (den >> 10))"),
    ("K mean from a plain fp32 sum", "s = np.array([math.fsum(K[:, c]) for c in range(d)], dtype=np.float64)",
     "s = K.astype(np.float32).sum(axis=0, dtype=np.float32).astype(np.float64)"),
    ("tuner takes lambda on equal sparsity", "if stage2[c, 1] < l2 and stage2[c, 0] > sparsity:", "if stage2[c, 1] < l2 and stage2[c, 0] >= sparsity:"),
    ("tuner's fallback takes the sparsest pair", "best = int(np.argmin(flat[:, 1]))", "best = int(np.argmax(flat[:, 0]))"),
    ("Hilbert order keeps cells outside the grid", "cells = cells[inside]", "cells = cells[np.all(cells <= np.array(grid)[None, :], axis=1)]"),
    ("literal CosSim formula normalised by the mean", "mx = abs(G.max())", "mx = abs(G.mean())"),
    ("partial last Q block padded with zero rows in the self-similarity", "nrm = np.sqrt((blk * blk).sum(axis=1, keepdims=True))",
     "blk = np.vstack([blk, np.zeros((b - len(blk), blk.shape[1]))]); nrm = np.sqrt((blk * blk).sum(axis=1, keepdims=True))"),
    ("dense reference without the softmax scale", "    S = (Q @ K.T) * scale\n    if causal:\n        S = np.where(np.arange(N)", "    S = (Q @ K.T)\n    if causal:\n        S = np.where(np.arange(N)"),
]


def load_mutant(old: str, new: str) -> types.ModuleType:
    assert SOURCE.count(old) >= 1, f"the oracle no longer contains {old!r}: update this mutation"
    mod = types.ModuleType("sparge_oracle_mutant")
    mod.__dict__["__name__"] = "sparge_oracle_mutant"
    import sys
    sys.modules["sparge_oracle_mutant"] = mod        # dataclasses look their module up by name
    try:
        exec(compile(SOURCE.replace(old, new, 1), "sparge_oracle_mutant.py", "exec"), mod.__dict__)
    finally:
        sys.modules.pop("sparge_oracle_mutant", None)
    return mod


def pin_calls():
    """Every pin of test_oracle_pins.py as a zero-argument callable (parametrized pins once per parameter set)."""
    for name, fn in sorted(vars(pins).items(), key=lambda kv: kv[1].__code__.co_firstlineno if inspect.isfunction(kv[1]) else 0):
        if not (inspect.isfunction(fn) and name.startswith("test_")):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            yield name, fn
            continue
        names, values = [], []
        for m in marks:
            argnames = [a.strip() for a in m.args[0].split(",")] if isinstance(m.args[0], str) else list(m.args[0])
            names.append(argnames)
            values.append([v if len(argnames) > 1 else (v,) for v in m.args[1]])
        for combo in itertools.product(*values):
            kwargs = {}
            for argnames, vals in zip(names, combo):
                kwargs.update(dict(zip(argnames, vals)))
            yield f"{name}{sorted(kwargs.items())}", (lambda f=fn, kw=kwargs: f(**kw))


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_some_pin_catches_the_mistake(monkeypatch, what, old, new):
    mutant = load_mutant(old, new)
    monkeypatch.setattr(pins, "so", mutant)
    caught = None
    for name, call in pin_calls():
        try:
            call()
        except Exception as e:          # an assertion, or the mistake makes the code fall over: both are a catch
            caught = (name, type(e).__name__)
            break
    assert caught is not None, f"no pin notices: {what}"
    print(f"{what}: caught by {caught[0]} ({caught[1]})")


def test_the_unmodified_source_passes_the_same_way(monkeypatch):
    """The harness itself: a copy of the oracle without any mistake passes every pin when run like this."""
    mutant = load_mutant("NEG_INF = -np.inf", "NEG_INF = -np.inf")
    monkeypatch.setattr(pins, "so", mutant)
    for name, call in pin_calls():
        call()
