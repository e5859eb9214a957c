"""Seeded synthetic attention inputs shaped like the paper's language / image / video workloads.

The paper measures on Q/K/V captured inside real models (Sec. 4.1); none of those models or
datasets is available here, so these generators stand in for them: smooth random fields on a
(t,h,w) grid flattened along a Hilbert curve (Sec. 3.7) for the visual workloads, and a
low-rank-drift + sink + recency construction for the causal language workload.

This module only *draws inputs*.  It contains no step of the method (no pooling, similarity,
quantization, softmax, ...), so both the CPU oracle's tests and the GPU path's tests may use it.

Every tensor is returned as float32 whose values are exactly representable in the workload's
16-bit dtype (fp16 or bf16), so converting to that dtype anywhere is lossless.
Random streams: numpy Generator(PCG64(SeedSequence([seed, cfg_id, tensor_id, head]))).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Iterable, Optional, Tuple

import numpy as np
import scipy.fft
import scipy.signal

TENSOR_ID = {"q": 0, "k": 1, "v": 2, "aux": 3}
_FFT_WORKERS = -1  # threads scipy.fft may use; pool workers set it to 1


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    H: int
    N: int
    d: int
    dtype: str  # "fp16" | "bf16"
    causal: bool
    tau: float
    theta: float
    lam: float
    kind: str  # "segments" | "field" | "language"
    grid: Optional[Tuple[int, ...]] = None  # (h,w) or (t,h,w)
    length_scale: Optional[Tuple[float, ...]] = None  # Gaussian kernel std per grid axis
    noise: float = 0.0
    seed: int = 0
    B: int = 1
    extra: Dict[str, float] = field(default_factory=dict)


CONFIGS: Dict[str, Workload] = {
    # C1: 16 contiguous 128-token segments, each sharing a centroid ~N(0,I) plus N(0,0.3^2) noise.
    "tiny": Workload("tiny", 1, H=2, N=2048, d=64, dtype="fp16", causal=False,
                     tau=0.9, theta=0.6, lam=-5.0, kind="segments", noise=0.3,
                     extra={"segment": 128}),
    # C2: 64x64 image grid, 2-D Gaussian random field (std 6 cells) + noise, Hilbert order.
    "image": Workload("image", 2, H=24, N=4096, d=128, dtype="bf16", causal=False,
                      tau=0.95, theta=0.5, lam=-8.0, kind="field", grid=(64, 64),
                      length_scale=(6.0, 6.0), noise=0.2),
    # C3: 13x30x45 video grid, 3-D field (std 2 in t, 5 in h,w) + noise, Hilbert order.
    "video": Workload("video", 3, H=48, N=17550, d=64, dtype="bf16", causal=False,
                      tau=0.9, theta=0.5, lam=-6.0, kind="field", grid=(13, 30, 45),
                      length_scale=(2.0, 5.0, 5.0), noise=0.2),
    # C4: causal language-like: noise + rank-8 drifting component + sink token + recency bias; the first
    # 64 tokens (a prompt prefix holding the sink) carry no shared component, so their block is not
    # self-similar and is always computed.
    "language": Workload("language", 4, H=32, N=32768, d=128, dtype="bf16", causal=True,
                         tau=0.95, theta=0.6, lam=-10.0, kind="language",
                         extra={"rank": 8, "corr_len": 4096.0, "drift_gain": 6.0, "pos_gain": 4.0,
                                "min_period": 512.0, "q_bias": 1.0, "sink_gain": 4.0, "prefix": 64}),
    # C5: 20x48x48 long-video grid, 3-D field (std 3 in t, 8 in h,w) + noise, Hilbert order.
    "longvideo": Workload("longvideo", 5, H=24, N=46080, d=128, dtype="bf16", causal=False,
                          tau=0.9, theta=0.5, lam=-5.0, kind="field", grid=(20, 48, 48),
                          length_scale=(3.0, 8.0, 8.0), noise=0.15),
}


# ----------------------------------------------------------------------------------------------
# rounding of generated values to the 16-bit input dtype (input preparation, not method arithmetic)
# ----------------------------------------------------------------------------------------------
def _round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "fp16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        f = np.ascontiguousarray(x, dtype=np.float32)
        u = f.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000  # round to nearest, ties to even
        return u.astype(np.uint32).view(np.float32).reshape(x.shape)
    raise ValueError(f"unknown dtype {dtype}")


def _rng(w: Workload, tensor: str, head: int) -> np.random.Generator:
    ss = np.random.SeedSequence([w.seed, w.cfg_id, TENSOR_ID[tensor], head])
    return np.random.Generator(np.random.PCG64(ss))


# ----------------------------------------------------------------------------------------------
# Hilbert curve (Skilling's axes<->transpose transform), vectorised over points
# ----------------------------------------------------------------------------------------------
def _hilbert_index(coords: np.ndarray, bits: int) -> np.ndarray:
    """Hilbert index of integer points. coords: [P, n] with 0 <= c < 2**bits. Returns uint64 [P]."""
    X = [coords[:, i].astype(np.uint64).copy() for i in range(coords.shape[1])]
    n = len(X)
    M = np.uint64(1 << (bits - 1))
    Q = int(M)
    while Q > 1:
        P = np.uint64(Q - 1)
        Qn = np.uint64(Q)
        for i in range(n):
            hit = (X[i] & Qn) != 0
            if i == 0:
                X[0] = np.where(hit, X[0] ^ P, X[0])  # invert low bits
            else:
                t = (X[0] ^ X[i]) & P  # exchange low bits of X[0] and X[i] where the bit is clear
                X[0], X[i] = np.where(hit, X[0] ^ P, X[0] ^ t), np.where(hit, X[i], X[i] ^ t)
        Q >>= 1
    for i in range(1, n):
        X[i] = X[i] ^ X[i - 1]
    t = np.zeros_like(X[0])
    Q = int(M)
    while Q > 1:
        hit = (X[n - 1] & np.uint64(Q)) != 0
        t = np.where(hit, t ^ np.uint64(Q - 1), t)
        Q >>= 1
    for i in range(n):
        X[i] = X[i] ^ t
    # interleave: most significant bit of X[0] first
    idx = np.zeros_like(X[0])
    for b in range(bits - 1, -1, -1):
        for i in range(n):
            idx = (idx << np.uint64(1)) | ((X[i] >> np.uint64(b)) & np.uint64(1))
    return idx


def hilbert_order(grid: Tuple[int, ...]) -> np.ndarray:
    """Permutation p such that sequence position s holds row-major grid cell p[s].

    Cells of the grid are visited in the order of their Hilbert index on the enclosing
    2^b hyper-cube; cells of the cube outside the grid are simply absent.
    """
    n = len(grid)
    bits = max(1, int(np.ceil(np.log2(max(grid)))))
    axes = np.meshgrid(*[np.arange(g) for g in grid], indexing="ij")
    coords = np.stack([a.reshape(-1) for a in axes], axis=1)
    idx = _hilbert_index(coords, bits)
    return np.argsort(idx, kind="stable")


# ----------------------------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------------------------
def _gaussian_field(rng: np.random.Generator, grid, length_scale, channels: int) -> np.ndarray:
    """Unit-variance smooth random field, [cells(row-major), channels].

    White noise on a box padded by >= 4 kernel std per axis (so the periodic FFT filter cannot
    correlate opposite faces of the cropped grid), multiplied in Fourier space by the Gaussian
    kernel's transfer function, cropped, then renormalised per channel to zero mean / unit variance.
    2-D grids are periodic by construction (no padding), matching the image recipe.
    """
    nd = len(grid)
    if nd == 2:
        box = tuple(grid)
    else:
        box = tuple(int(scipy.fft.next_fast_len(int(g + np.ceil(4 * s)), real=True))
                    for g, s in zip(grid, length_scale))
    white = rng.standard_normal((channels,) + box)
    axes = tuple(range(1, nd + 1))
    F = scipy.fft.rfftn(white, axes=axes, workers=_FFT_WORKERS)
    del white
    shape_f = F.shape[1:]
    tf = np.ones(shape_f, dtype=np.float64)
    for ax, (nbox, s) in enumerate(zip(box, length_scale)):
        if ax == nd - 1:
            freq = np.fft.rfftfreq(nbox)
        else:
            freq = np.fft.fftfreq(nbox)
        g = np.exp(-2.0 * (np.pi * freq * s) ** 2)
        sh = [1] * nd
        sh[ax] = g.shape[0]
        tf = tf * g.reshape(sh)
    F *= tf[None]
    f = scipy.fft.irfftn(F, s=box, axes=axes, workers=_FFT_WORKERS)
    del F
    crop = (slice(None),) + tuple(slice(0, g) for g in grid)
    f = f[crop].reshape(channels, -1)
    f = f - f.mean(axis=1, keepdims=True)
    f = f / f.std(axis=1, keepdims=True)
    return np.ascontiguousarray(f.T)


def _orthonormal_rows(rng: np.random.Generator, r: int, d: int) -> np.ndarray:
    a = rng.standard_normal((d, r))
    q, _ = np.linalg.qr(a)
    return q.T  # [r, d]


def make_head(w: Workload, head: int, tensors: Iterable[str] = ("q", "k", "v"),
              perm: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Generate the requested tensors of one head, each float32 [N, d] (values exact in w.dtype)."""
    out: Dict[str, np.ndarray] = {}
    N, d = w.N, w.d
    tensors = tuple(tensors)
    if "v" in tensors:
        out["v"] = _round_to_dtype(_rng(w, "v", head).standard_normal((N, d)), w.dtype)
    qk = [t for t in tensors if t in ("q", "k")]
    if not qk:
        return out
    if w.kind == "segments":
        seg = int(w.extra["segment"])
        nseg = (N + seg - 1) // seg
        for t in qk:
            rng = _rng(w, t, head)
            cent = rng.standard_normal((nseg, d))
            x = np.repeat(cent, seg, axis=0)[:N] + w.noise * rng.standard_normal((N, d))
            out[t] = _round_to_dtype(x, w.dtype)
    elif w.kind == "field":
        if perm is None:
            perm = hilbert_order(w.grid)
        for t in qk:
            rng = _rng(w, t, head)
            f = _gaussian_field(rng, w.grid, w.length_scale, d)
            x = f[perm] + w.noise * rng.standard_normal((N, d))
            out[t] = _round_to_dtype(x, w.dtype)
    elif w.kind == "language":
        ex = w.extra
        r = int(ex["rank"])
        aux = _rng(w, "aux", head)  # shared between Q and K of this head
        U = _orthonormal_rows(aux, r, d)
        W = _orthonormal_rows(aux, 2 * r, d)
        u0 = aux.standard_normal(d)
        u0 /= np.linalg.norm(u0)
        rho = float(np.exp(-1.0 / ex["corr_len"]))
        eps = aux.standard_normal((N, r))
        eps[0] /= np.sqrt(1.0 - rho * rho)  # stationary start
        z = scipy.signal.lfilter([np.sqrt(1.0 - rho * rho)], [1.0, -rho], eps, axis=0)
        tpos = np.arange(N, dtype=np.float64)[:, None]
        periods = float(ex.get("min_period", 64.0)) * (2.0 ** np.arange(r))[None, :]
        ang = 2.0 * np.pi * tpos / periods
        p = np.concatenate([np.cos(ang), np.sin(ang)], axis=1) / np.sqrt(r)
        shared = ex["drift_gain"] * (z @ U) + ex["pos_gain"] * (p @ W)
        shared[:int(ex.get("prefix", 0))] = 0.0  # prompt-prefix tokens carry no shared component
        for t in qk:
            rng = _rng(w, t, head)
            x = rng.standard_normal((N, d)) + shared
            if t == "q":
                x = x + ex["q_bias"] * u0[None, :]
            else:
                mean_norm = float(np.mean(np.linalg.norm(x, axis=1)))
                x[0] = ex["sink_gain"] * mean_norm * u0
            out[t] = _round_to_dtype(x, w.dtype)
    else:
        raise ValueError(w.kind)
    return out


def _head_job(args):
    w, h, tensors, perm = args
    return make_head(w, h, tensors, perm=perm)


def make_workload(w: Workload, heads: Optional[Iterable[int]] = None,
                  tensors: Iterable[str] = ("q", "k", "v"), workers: int = 1) -> Dict[str, np.ndarray]:
    """All requested heads stacked: each tensor float32 [1, len(heads), N, d].

    workers > 1 generates heads on a thread pool (numpy's generators, FFTs and array arithmetic release
    the GIL).  Every head has its own random stream, so the result does not depend on the worker count.
    """
    global _FFT_WORKERS
    heads = list(range(w.H)) if heads is None else list(heads)
    tensors = tuple(tensors)
    perm = hilbert_order(w.grid) if w.kind == "field" else None
    out = {t: np.empty((1, len(heads), w.N, w.d), dtype=np.float32) for t in tensors}
    jobs = [(w, h, tensors, perm) for h in heads]

    def run(hi_job):
        hi, job = hi_job
        one = _head_job(job)
        for t in tensors:
            out[t][0, hi] = one[t]

    if workers > 1 and len(heads) > 1:
        from concurrent.futures import ThreadPoolExecutor
        saved, _FFT_WORKERS = _FFT_WORKERS, 1
        try:
            with ThreadPoolExecutor(min(workers, len(heads))) as pool:
                list(pool.map(run, enumerate(jobs)))
        finally:
            _FFT_WORKERS = saved
    else:
        for item in enumerate(jobs):
            run(item)
    return out


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (e.g. fewer heads, shorter N for tests)."""
    from dataclasses import replace
    return replace(w, **kw)
