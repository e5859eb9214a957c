"""Shared helpers of the test-suite (no method arithmetic)."""
import numpy as np

from synth import make_workload
from synth.workloads import Workload


# How far a row's maximum may run ahead of the value the kernel subtracts inside exp (natural-log
# units; SPARGE_REF_SLACK_LOG2 of sparge.h): the oracle's loop takes it as ref_slack so that P~ is
# rounded to 16 bits at the same point on both sides.
REF_SLACK = 8 * float(np.log(2.0))


def f32(x) -> float:
    """The value a host float array hands to the library."""
    return float(np.float32(x))


def small_workload(name="t", N=700, d=64, dtype="fp16", H=2, causal=False, tau=0.8, theta=0.5, lam=-4.0,
                   seed=1, noise=0.3, segment=128):
    """Segment-structured inputs of arbitrary (ragged) length: same family as the tiny config."""
    return Workload(name, 90 + seed, H=H, N=N, d=d, dtype=dtype, causal=causal, tau=tau, theta=theta, lam=lam,
                    kind="segments", noise=noise, seed=seed, extra={"segment": segment})


def to_torch(x: np.ndarray, dtype: str, device="cuda"):
    from paper_2502_18137_amd import tensor_from_numpy
    return tensor_from_numpy(x, dtype, device)


def gpu_inputs(w, heads=None):
    """(numpy dict, torch Q, K, V on the GPU) for a workload."""
    x = make_workload(w, heads=heads)
    return x, to_torch(x["q"], w.dtype), to_torch(x["k"], w.dtype), to_torch(x["v"], w.dtype)


# ---- output parity bars (derived in the design notes, reading r18) -------------------------------------
# u = unit roundoff of the 16-bit type that P~ and O are rounded to.  A rounding to p significant bits of a
# value whose significand is log-uniform has relative error of rms 0.4247 u (uniform in +-u/f, f in [1,2)).
# With V white noise an output is a random combination of V rows, so a head's relative L1 distance between
# two evaluations is the rms of the relative errors that differ between them:
#   against Alg. 1 in exact arithmetic with the same quantized operands (nothing rounded):  P~ and O each
#     rounded once -> sqrt(2) * 0.4247 u = 0.60 u;
#   against the recurrence as printed (ref_slack = 0) with P~ and O rounded at its own points: up to four
#     independent roundings -> 0.85 u;
#   against the oracle that rounds P~ at the kernel's point (ref_slack = the kernel's): only fp32-vs-fp64
#     effects, the benchmark spec's 2e-3.
# Per row the same quantities fluctuate with the few keys that carry a row's mass (one dominant key: a
# single error of up to u instead of an rms) and with the d channels a row's L1 norm averages over.
def unit_roundoff(dtype: str) -> float:
    return {"bf16": 2.0 ** -8, "fp16": 2.0 ** -11}[dtype]


HEAD_BAR_EMUL = 2e-3            # spec: against the oracle that emulates quantization and rounding
HEAD_BAR_PRINTED_U = 1.0        # x u: against Alg. 1 lines 12-16 as printed, P~ rounded to 16 bits there
HEAD_BAR_UNROUNDED_U = 0.8      # x u: against the same loop with nothing rounded after the quantization
ROW_BAR_EMUL_U = 4.0            # x u per row: a P~ rounding and an output rounding that flip (one ulp = 2 u each)
ROW_BAR_PRINTED_U = 3.0         # x u per row
ROW_BAR_UNROUNDED_U = 2.5       # x u per row
# Per element there is a bound that needs no statistics.  With p_k the exact softmax weights of a row (over
# the executed tiles), the kernel computes fl16(sum_k p_k (1 + e_k) V_kc / (1 + e_l)): |e_k| <= u from the
# rounding of P~ plus the fp32 evaluation of the exponent (the dequantization FMA rounds an argument of
# magnitude up to ~6 |S| log2 e: below 1e-4 for |S| <= 300), e_l the fp32 row sum (negligible), and one final
# rounding of relative size u.  Hence, to first order,
#   |O_kernel - O_exact|_rc <= (u + FP32_SLACK + step) * sum_k p_k |V_kc| + u * |O_exact|_rc,
# and sum_k p_k |V_kc| is Alg. 1 evaluated on |V|: the oracle computes it with one more call.
# `step` belongs to the INT8 product only: the kernel keeps its integer accumulators as the floats
# 1.5 * 2^23 + acc and folds the offset into the constant of the FMA that dequantizes and subtracts the
# reference; that constant, of magnitude 1.5 * 2^23 * (delta_Q delta_K scale log2 e), is rounded to fp32 once per
# (row, tile): an error of at most 0.75 accumulator steps in the exponent, i.e. a relative error of P~ of at most
# ACC_STEP_FRACTION * delta_Q delta_K scale, common to a (row, tile) but different from tile to tile.
FP32_SLACK = 2e-4
ACC_STEP_FRACTION = 0.75
ELEMENT_BOUND_FACTOR = 1.01     # second-order terms
LAMBDA_MARGIN = 1e-3            # stage-2 statistics closer than this to lambda are not pinned (fp32 vs fp64)


def row_rel_l1(O: np.ndarray, ref: np.ndarray) -> np.ndarray:
    """Per row: sum_c |O - ref| / sum_c |ref| (rows whose reference is all zero count their absolute error)."""
    den = np.abs(ref).sum(axis=1)
    return np.abs(O - ref).sum(axis=1) / np.where(den > 0, den, 1.0)


def check_output_parity(so, got: np.ndarray, q, k, v, mask, lam: float, causal: bool, dtype: str,
                        rows: np.ndarray, q_blocks=None, label: str = "", ref_slack: float = REF_SLACK,
                        quant: bool = True) -> dict:
    """The 16-bit INT8 path's output rows `got` (fp64 copies of the stored 16-bit values, rows `rows` of the
    head) against three evaluations of Alg. 1 by the oracle on the same block mask and lambda:
    the emulating one (P~ rounded at the kernel's point), the recurrence as printed with P~ rounded to the
    16-bit type (ref_slack = 0), and the loop with nothing rounded after the INT8 quantization (quant = False:
    after nothing at all).  Bars: see above, for the head (relative L1 over the rows), for every single row,
    and for every element against the unrounded loop.  Rows of a 32-row group whose
    stage-2 statistic came within LAMBDA_MARGIN of lambda on some tile are left out (a flipped decision
    there is not an error).  Returns the measured numbers."""
    u = unit_roundoff(dtype)
    kw = dict(lam=lam, causal=causal, quant=quant, q_blocks=q_blocks)
    r_em = so.sparse_attention(q, k, v, mask, pv_dtype=dtype, ref_slack=ref_slack, **kw)
    r_pr = so.sparse_attention(q, k, v, mask, pv_dtype=dtype, ref_slack=0.0, **kw)
    r_un = so.sparse_attention(q, k, v, mask, pv_dtype="none", **kw)
    assert r_em.zero_rows == 0
    pinned = r_un.lam_margin[rows // 128, (rows % 128) // 32] >= LAMBDA_MARGIN
    assert pinned.mean() > 0.9, "too many stage-2 decisions on the threshold for this case to test anything"
    out = {"rows": int(pinned.sum()), "unpinned_rows": int((~pinned).sum())}
    g = got[pinned]
    for name, ref, head_bar, row_bar in (
            ("emul", so.round16(r_em.O[rows], dtype), HEAD_BAR_EMUL, max(ROW_BAR_EMUL_U * u, HEAD_BAR_EMUL)),
            ("printed", so.round16(r_pr.O[rows], dtype), HEAD_BAR_PRINTED_U * u, ROW_BAR_PRINTED_U * u),
            ("unrounded", r_un.O[rows], HEAD_BAR_UNROUNDED_U * u, ROW_BAR_UNROUNDED_U * u)):
        ref = ref[pinned]
        out[name] = so.rel_l1(g, ref)
        out[name + "_row_max"] = float(row_rel_l1(g, ref).max())
        assert out[name] <= head_bar, (label, name, out[name], head_bar)
        assert out[name + "_row_max"] <= row_bar, (label, name, "row", out[name + "_row_max"], row_bar)
    # every element against the loop in exact arithmetic, at the bound derived above
    r_abs = so.sparse_attention(q, k, np.abs(v), mask, pv_dtype="none", **kw)
    exact, weight = r_un.O[rows][pinned], r_abs.O[rows][pinned]
    step = 0.0
    if quant:
        scale = 1.0 / np.sqrt(q.shape[1])
        step = ACC_STEP_FRACTION * float(so.quantize_q(q)[1].max()) * float(so.quantize_k(k)[1].max()) * scale
    out["acc_step"] = step
    bound = ELEMENT_BOUND_FACTOR * ((u + FP32_SLACK + step) * weight + u * np.abs(exact)) + 1e-30
    ratio = np.abs(g - exact) / bound
    out["element_bound_used"] = float(ratio.max())
    assert out["element_bound_used"] <= 1.0, (label, "element", np.unravel_index(ratio.argmax(), ratio.shape),
                                              out["element_bound_used"])
    print(f"  {label}: rel-L1 emul {out['emul']:.2e} (row max {out['emul_row_max']:.2e}), printed "
          f"{out['printed'] / u:.2f}u (row {out['printed_row_max'] / u:.2f}u), unrounded {out['unrounded'] / u:.2f}u "
          f"(row {out['unrounded_row_max'] / u:.2f}u), elements at most {out['element_bound_used']:.2f} of their bound, "
          f"u = {u:.2e}, {out['unpinned_rows']} rows unpinned", flush=True)
    out["ref"] = r_em
    return out
