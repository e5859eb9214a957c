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
