"""ctypes binding for libsparge.so: argument marshalling only.

Every function mirrors the C entry point of the same name (include/sparge.h).  Tensors are torch
tensors on the GPU; outputs and the workspace are allocated here with torch (device memory and
streams are all torch is used for) and every step of the path runs inside the library's kernels.
There is no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple, Union

import torch

WS_QUANTIZE, WS_PREDICT, WS_ATTN, WS_ATTN_QUANTIZED, WS_FORWARD, WS_ATTN_TILED = range(6)
BQ, BK = 128, 64
REF_SLACK_LOG2 = 8      # SPARGE_REF_SLACK_LOG2 of sparge.h
REF_SLACK_LOG2_FP8 = 2  # SPARGE_REF_SLACK_LOG2_FP8

_LIB: Optional[ctypes.CDLL] = None


class SpargeError(RuntimeError):
    pass


class _Desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32), ("d", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64),
                ("stride_n", ctypes.c_int64), ("pv_dtype", ctypes.c_int32), ("qk_dtype", ctypes.c_int32)]


def library_path() -> str:
    """The in-tree library; SPARGE_LIBRARY overrides it (e.g. to load an experimental build)."""
    return os.environ.get("SPARGE_LIBRARY") or os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                            "libsparge.so")


def load_library() -> ctypes.CDLL:
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise SpargeError(f"{path} is missing: build it with `python -m paper_2502_18137_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    vp, f32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(_Desc)
    lib.sparge_last_error.restype = ctypes.c_char_p
    lib.sparge_last_error.argtypes = []
    lib.sparge_version.restype = ctypes.c_int
    lib.sparge_workspace_bytes.argtypes = [dp, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.sparge_quantize.argtypes = [vp, vp, dp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sparge_predict.argtypes = [vp, vp, dp, f32p, f32p, ctypes.c_float, ctypes.c_int, vp, vp, vp, vp,
                                   ctypes.c_size_t, vp]
    lib.sparge_predict_static.argtypes = [vp, vp, dp, f32p, f32p, ctypes.c_float, ctypes.c_int, vp, vp, vp, vp]
    lib.sparge_predict_static.restype = ctypes.c_int
    lib.sparge_attn_quantized.argtypes = [vp, vp, vp, vp, vp, dp, vp, f32p, ctypes.c_float, ctypes.c_int, vp, vp,
                                          vp, ctypes.c_size_t, vp]
    lib.sparge_mask_to_lut.argtypes = [vp, dp, vp, vp, vp]
    lib.sparge_item_order.argtypes = [dp, ctypes.c_int, ctypes.POINTER(ctypes.c_int32)]
    lib.sparge_v_tiles.argtypes = [vp, dp, vp, vp]
    lib.sparge_v_tiles_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t)]
    lib.sparge_attn_tiled.argtypes = [vp, vp, vp, vp, vp, dp, vp, f32p, ctypes.c_float, ctypes.c_int, vp, vp, vp,
                                      ctypes.c_size_t, vp]
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.sparge_rel_l1.argtypes = [vp, vp, dp, vp, vp]
    lib.sparge_tune_workspace_bytes.argtypes = [dp, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.sparge_tune.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.c_int, dp,
                                f32p, ctypes.c_int, f32p, ctypes.c_int, f32p, ctypes.c_int,
                                ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_int,
                                f32p, f32p, f32p, f64p, f64p, f64p, f64p, vp, ctypes.c_size_t, vp]
    lib.sparge_hilbert_order.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int32)]
    lib.sparge_permute_tokens.argtypes = [vp, dp, vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
    lib.sparge_set_timing_events.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.c_int]
    lib.sparge_set_timing_events.restype = ctypes.c_int
    lib.sparge_attn.argtypes = [vp, vp, vp, dp, vp, f32p, ctypes.c_float, ctypes.c_int, vp, vp, vp,
                                ctypes.c_size_t, vp]
    lib.sparge_forward.argtypes = [vp, vp, vp, dp, f32p, f32p, f32p, ctypes.c_float, ctypes.c_int, vp, vp, vp, vp,
                                   ctypes.c_size_t, vp]
    for name in ("sparge_workspace_bytes", "sparge_quantize", "sparge_predict", "sparge_attn_quantized",
                 "sparge_attn", "sparge_forward", "sparge_mask_to_lut", "sparge_item_order", "sparge_v_tiles", "sparge_attn_tiled", "sparge_v_tiles_bytes",
                 "sparge_rel_l1", "sparge_tune_workspace_bytes", "sparge_tune", "sparge_hilbert_order",
                 "sparge_permute_tokens"):
        getattr(lib, name).restype = ctypes.c_int
    _LIB = lib
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise SpargeError(f"libsparge error {rc}: {load_library().sparge_last_error().decode()}")


def _desc(x: torch.Tensor, pv_fp8: bool = False, qk16: bool = False) -> _Desc:
    if x.dim() != 4:
        raise SpargeError("expected a [B, H, N, d] tensor")
    if not x.is_cuda:
        raise SpargeError("tensors must live on the GPU")
    if x.stride(3) != 1:
        raise SpargeError("the head dimension must be contiguous")
    if x.dtype == torch.float16:
        dt = 0
    elif x.dtype == torch.bfloat16:
        dt = 1
    else:
        raise SpargeError(f"dtype {x.dtype} not supported (fp16 or bf16)")
    B, H, N, d = x.shape
    return _Desc(B, H, N, d, dt, x.stride(0), x.stride(1), x.stride(2), 1 if pv_fp8 else 0, 1 if qk16 else 0)


def _same_layout(ref: torch.Tensor, *others: torch.Tensor) -> None:
    for o in others:
        if o.shape != ref.shape or o.stride() != ref.stride() or o.dtype != ref.dtype or o.device != ref.device:
            raise SpargeError("Q, K, V (and O) must share shape, strides, dtype and device")


def _per_head(v: Union[float, Sequence[float]], H: int):
    vals = [float(v)] * H if isinstance(v, (int, float)) else [float(x) for x in v]
    if len(vals) != H:
        raise SpargeError(f"expected {H} per-head values, got {len(vals)}")
    return (ctypes.c_float * H)(*vals)


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def tensor_from_numpy(x, dtype: str, device: str = "cuda") -> torch.Tensor:
    """A float32 numpy array whose values are exact in `dtype` ("fp16" | "bf16") -> GPU tensor of that dtype."""
    import numpy as np
    t = torch.from_numpy(np.ascontiguousarray(x))
    return t.to(device=device, dtype=torch.float16 if dtype == "fp16" else torch.bfloat16)


def sparge_version() -> int:
    return load_library().sparge_version()


def sparge_workspace_bytes(x: torch.Tensor, entry: int, pv_fp8: bool = False) -> int:
    n = ctypes.c_size_t(0)
    d = _desc(x, pv_fp8)
    _check(load_library().sparge_workspace_bytes(ctypes.byref(d), entry, ctypes.byref(n)))
    return int(n.value)


def _workspace(x: torch.Tensor, entry: int, ws: Optional[torch.Tensor], pv_fp8: bool = False) -> torch.Tensor:
    need = sparge_workspace_bytes(x, entry, pv_fp8)
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=x.device)
    return ws


def _blocks(N: int) -> Tuple[int, int]:
    return (N + BQ - 1) // BQ, (N + BK - 1) // BK


def sparge_quantize(Q: torch.Tensor, K: torch.Tensor, ws: Optional[torch.Tensor] = None):
    """-> (Qq int8 [B,H,N,d], Kq int8, q_scale fp32 [B,H,Tm], k_scale fp32 [B,H,Tn], k_mean fp32 [B,H,d])."""
    _same_layout(Q, K)
    d = _desc(Q)
    B, H, N, dim = Q.shape
    Tm, Tn = _blocks(N)
    dev = Q.device
    Qq = torch.empty((B, H, N, dim), dtype=torch.int8, device=dev)
    Kq = torch.empty((B, H, N, dim), dtype=torch.int8, device=dev)
    qs = torch.empty((B, H, Tm), dtype=torch.float32, device=dev)
    ks = torch.empty((B, H, Tn), dtype=torch.float32, device=dev)
    km = torch.empty((B, H, dim), dtype=torch.float32, device=dev)
    ws = _workspace(Q, WS_QUANTIZE, ws)
    _check(load_library().sparge_quantize(_ptr(Q), _ptr(K), ctypes.byref(d), _ptr(Qq), _ptr(Kq), _ptr(qs), _ptr(ks),
                                          _ptr(km), _ptr(ws), ws.numel(), _stream()))
    return Qq, Kq, qs, ks, km


def sparge_predict(Q: torch.Tensor, K: torch.Tensor, tau, theta, causal: bool = False, sm_scale: float = 0.0,
                   return_sims: bool = False, ws: Optional[torch.Tensor] = None):
    """-> mask uint8 [B,H,Tm,Tn] (and sim_q, sim_k fp64 if return_sims)."""
    _same_layout(Q, K)
    d = _desc(Q)
    B, H, N, _ = Q.shape
    Tm, Tn = _blocks(N)
    mask = torch.empty((B, H, Tm, Tn), dtype=torch.uint8, device=Q.device)
    sq = torch.empty((B, H, Tm), dtype=torch.float64, device=Q.device) if return_sims else None
    sk = torch.empty((B, H, Tn), dtype=torch.float64, device=Q.device) if return_sims else None
    ws = _workspace(Q, WS_PREDICT, ws)
    _check(load_library().sparge_predict(_ptr(Q), _ptr(K), ctypes.byref(d), _per_head(tau, H), _per_head(theta, H),
                                         float(sm_scale), int(causal), _ptr(mask), _ptr(sq), _ptr(sk), _ptr(ws),
                                         ws.numel(), _stream()))
    return (mask, sq, sk) if return_sims else mask


STATIC_SCRATCH_BYTES = 4 << 20  # SPARGE_STATIC_SCRATCH_BYTES


def sparge_predict_static(Q: torch.Tensor, K: torch.Tensor, tau, theta, mask: torch.Tensor, causal: bool = False,
                          sm_scale: float = 0.0, sim_q: Optional[torch.Tensor] = None,
                          sim_k: Optional[torch.Tensor] = None) -> None:
    """sparge_predict without a workspace (the library's static scratch).  Nothing is allocated here either:
    the caller passes `mask` (uint8 [B,H,Tm,Tn]) and, optionally, sim_q / sim_k (fp64)."""
    _same_layout(Q, K)
    d = _desc(Q)
    _check(load_library().sparge_predict_static(_ptr(Q), _ptr(K), ctypes.byref(d), _per_head(tau, Q.shape[1]),
                                                _per_head(theta, Q.shape[1]), float(sm_scale), int(causal),
                                                _ptr(mask), _ptr(sim_q), _ptr(sim_k), _stream()))


def sparge_attn_quantized(Qq, Kq, q_scale, k_scale, V: torch.Tensor, mask: Optional[torch.Tensor], lam,
                          causal: bool = False, sm_scale: float = 0.0, return_stats: bool = False,
                          ws: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                          pv_fp8: bool = False):
    """-> O (same layout as V) (and stats uint64-as-int64 [B,H,4] if return_stats).
    pv_fp8: the P~V product in FP8 (E4M3) instead of V's 16-bit type."""
    d = _desc(V, pv_fp8)
    B, H, N, dim = V.shape
    Tm, Tn = _blocks(N)
    for t, shape, dt in ((Qq, (B, H, N, dim), torch.int8), (Kq, (B, H, N, dim), torch.int8),
                         (q_scale, (B, H, Tm), torch.float32), (k_scale, (B, H, Tn), torch.float32)):
        if tuple(t.shape) != shape or t.dtype != dt or not t.is_contiguous() or t.device != V.device:
            raise SpargeError("quantized operands must be contiguous outputs of sparge_quantize for this shape")
    if mask is not None and (tuple(mask.shape) != (B, H, Tm, Tn) or mask.dtype != torch.uint8
                             or not mask.is_contiguous() or mask.device != V.device):
        raise SpargeError("mask must be a contiguous uint8 [B,H,Tm,Tn] tensor")
    O = torch.empty_like(V) if out is None else out
    _same_layout(V, O)
    stats = torch.zeros((B, H, 4), dtype=torch.int64, device=V.device) if return_stats else None
    ws = _workspace(V, WS_ATTN_QUANTIZED, ws, pv_fp8)
    _check(load_library().sparge_attn_quantized(_ptr(Qq), _ptr(Kq), _ptr(q_scale), _ptr(k_scale), _ptr(V),
                                                ctypes.byref(d), _ptr(mask), _per_head(lam, H), float(sm_scale),
                                                int(causal), _ptr(O), _ptr(stats), _ptr(ws), ws.numel(), _stream()))
    return (O, stats) if return_stats else O


def sparge_mask_to_lut(mask: torch.Tensor, like: torch.Tensor):
    """-> (lut int32 [B,H,Tm,Tn]: kept key blocks of each row ascending, then -1; count int32 [B,H,Tm]).
    `like`: a tensor of the attention shape [B,H,N,d] the mask belongs to."""
    d = _desc(like)
    B, H, N, _ = like.shape
    Tm, Tn = _blocks(N)
    if tuple(mask.shape) != (B, H, Tm, Tn) or mask.dtype != torch.uint8 or not mask.is_contiguous() or mask.device != like.device:
        raise SpargeError("mask must be a contiguous uint8 [B,H,Tm,Tn] tensor")
    lut = torch.empty((B, H, Tm, Tn), dtype=torch.int32, device=mask.device)
    count = torch.empty((B, H, Tm), dtype=torch.int32, device=mask.device)
    _check(load_library().sparge_mask_to_lut(_ptr(mask), ctypes.byref(d), _ptr(lut), _ptr(count), _stream()))
    return lut, count


def sparge_v_tiles(V: torch.Tensor, pv_fp8: bool = False) -> torch.Tensor:
    """-> V re-tiled for the P~V product: [B,H,Tn,d,64] in V's dtype, or (pv_fp8) a flat uint8 buffer holding
    the E4M3 tiles, the channel scales and the channel maxima (layout: sparge.h)."""
    d = _desc(V, pv_fp8)
    B, H, N, dim = V.shape
    if pv_fp8:
        n = ctypes.c_size_t(0)
        _check(load_library().sparge_v_tiles_bytes(ctypes.byref(d), ctypes.byref(n)))
        tiles = torch.empty(n.value, dtype=torch.uint8, device=V.device)
    else:
        tiles = torch.empty((B, H, _blocks(N)[1], dim, BK), dtype=V.dtype, device=V.device)
    _check(load_library().sparge_v_tiles(_ptr(V), ctypes.byref(d), _ptr(tiles), _stream()))
    return tiles


def sparge_attn_tiled(Qq, Kq, q_scale, k_scale, v_tiles: torch.Tensor, like: torch.Tensor,
                      mask: Optional[torch.Tensor], lam, causal: bool = False, sm_scale: float = 0.0,
                      stats: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                      pv_fp8: bool = False, ws: Optional[torch.Tensor] = None):
    """The sparse flash loop alone.  `like` gives O's shape/strides/dtype (the V it was tiled from)."""
    d = _desc(like, pv_fp8)
    B, H, N, dim = like.shape
    if pv_fp8:
        n = ctypes.c_size_t(0)
        _check(load_library().sparge_v_tiles_bytes(ctypes.byref(d), ctypes.byref(n)))
        ok = v_tiles.dtype == torch.uint8 and v_tiles.numel() == n.value
    else:
        ok = tuple(v_tiles.shape) == (B, H, _blocks(N)[1], dim, BK)
    if not ok or not v_tiles.is_contiguous():
        raise SpargeError("v_tiles must come from sparge_v_tiles for this shape and pv_fp8 setting")
    O = torch.empty_like(like) if out is None else out
    _same_layout(like, O)
    ws = _workspace(like, WS_ATTN_TILED, ws, pv_fp8)
    _check(load_library().sparge_attn_tiled(_ptr(Qq), _ptr(Kq), _ptr(q_scale), _ptr(k_scale), _ptr(v_tiles),
                                            ctypes.byref(d), _ptr(mask), _per_head(lam, H), float(sm_scale),
                                            int(causal), _ptr(O), _ptr(stats), _ptr(ws), ws.numel(), _stream()))
    return O


def sparge_attn(Q, K, V, mask: Optional[torch.Tensor], lam, causal: bool = False, sm_scale: float = 0.0,
                return_stats: bool = False, ws: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                pv_fp8: bool = False, qk16: bool = False):
    """Quantize + sparse attention.  -> O (and stats).  qk16: the Q K^T product on the 16-bit tensors
    themselves instead of their INT8 quantization."""
    _same_layout(Q, K, V)
    d = _desc(Q, pv_fp8, qk16)
    B, H, N, _ = Q.shape
    Tm, Tn = _blocks(N)
    if mask is not None and (tuple(mask.shape) != (B, H, Tm, Tn) or mask.dtype != torch.uint8
                             or not mask.is_contiguous() or mask.device != Q.device):
        raise SpargeError("mask must be a contiguous uint8 [B,H,Tm,Tn] tensor")
    O = torch.empty_like(V) if out is None else out
    _same_layout(V, O)
    stats = torch.zeros((B, H, 4), dtype=torch.int64, device=Q.device) if return_stats else None
    ws = _workspace(Q, WS_ATTN, ws, pv_fp8)
    _check(load_library().sparge_attn(_ptr(Q), _ptr(K), _ptr(V), ctypes.byref(d), _ptr(mask), _per_head(lam, H),
                                      float(sm_scale), int(causal), _ptr(O), _ptr(stats), _ptr(ws), ws.numel(),
                                      _stream()))
    return (O, stats) if return_stats else O


def sparge_forward(Q, K, V, tau, theta, lam, causal: bool = False, sm_scale: float = 0.0,
                   return_mask: bool = False, return_stats: bool = False, ws: Optional[torch.Tensor] = None,
                   out: Optional[torch.Tensor] = None, pv_fp8: bool = False, qk16: bool = False):
    """All of Algorithm 1.  -> O (and mask, stats when requested, in that order)."""
    _same_layout(Q, K, V)
    d = _desc(Q, pv_fp8, qk16)
    B, H, N, _ = Q.shape
    Tm, Tn = _blocks(N)
    O = torch.empty_like(V) if out is None else out
    _same_layout(V, O)
    mask = torch.empty((B, H, Tm, Tn), dtype=torch.uint8, device=Q.device) if return_mask else None
    stats = torch.zeros((B, H, 4), dtype=torch.int64, device=Q.device) if return_stats else None
    ws = _workspace(Q, WS_FORWARD, ws, pv_fp8)
    _check(load_library().sparge_forward(_ptr(Q), _ptr(K), _ptr(V), ctypes.byref(d), _per_head(tau, H),
                                         _per_head(theta, H), _per_head(lam, H), float(sm_scale), int(causal),
                                         _ptr(O), _ptr(mask), _ptr(stats), _ptr(ws), ws.numel(), _stream()))
    res = [O]
    if return_mask:
        res.append(mask)
    if return_stats:
        res.append(stats)
    return res[0] if len(res) == 1 else tuple(res)


def sparge_rel_l1(O: torch.Tensor, O_ref: torch.Tensor) -> torch.Tensor:
    """-> fp64 [B,H,2] = {sum|O_ref - O|, sum|O_ref|} (Sec. 3.6); divide to get the relative L1 distance."""
    _same_layout(O_ref, O)
    d = _desc(O)
    out = torch.empty((O.shape[0], O.shape[1], 2), dtype=torch.float64, device=O.device)
    _check(load_library().sparge_rel_l1(_ptr(O), _ptr(O_ref), ctypes.byref(d), _ptr(out), _stream()))
    return out


def sparge_tune(inputs, tau_grid, theta_grid, lambda_grid, l1: float, l2: float, causal: bool = False,
                sm_scale: float = 0.0, pv_fp8: bool = False):
    """Sec. 3.6 per head.  inputs: list of (Q, K, V) of one shape and layout.
    -> dict(tau, theta, lam [H] lists; sparsity, l1 [H]; stage1 [n_tau,n_theta,H,2], stage2 [n_lambda,H,2] as
    nested lists of {mean sparsity, worst relative L1}).  Blocks until done."""
    import numpy as np
    Q0 = inputs[0][0]
    for q, k, v in inputs:
        _same_layout(Q0, q, k, v)
    d = _desc(Q0, pv_fp8)
    H, n = Q0.shape[1], len(inputs)
    need = ctypes.c_size_t(0)
    _check(load_library().sparge_tune_workspace_bytes(ctypes.byref(d), n, ctypes.byref(need)))
    ws = torch.empty(need.value, dtype=torch.uint8, device=Q0.device)
    arr = lambda k: (ctypes.c_void_p * n)(*[t[k].data_ptr() for t in inputs])
    fl = lambda xs: (ctypes.c_float * len(xs))(*[float(x) for x in xs])
    tau, theta, lam = (ctypes.c_float * H)(), (ctypes.c_float * H)(), (ctypes.c_float * H)()
    sp, err = (ctypes.c_double * H)(), (ctypes.c_double * H)()
    n1, n2 = len(tau_grid) * len(theta_grid), len(lambda_grid)
    s1, s2 = (ctypes.c_double * (n1 * H * 2))(), (ctypes.c_double * max(n2 * H * 2, 1))()
    _check(load_library().sparge_tune(arr(0), arr(1), arr(2), n, ctypes.byref(d), fl(tau_grid), len(tau_grid),
                                      fl(theta_grid), len(theta_grid), fl(lambda_grid), n2, float(l1), float(l2),
                                      float(sm_scale), int(causal), tau, theta, lam, sp, err, s1, s2, _ptr(ws),
                                      ws.numel(), _stream()))
    return {"tau": list(tau), "theta": list(theta), "lam": list(lam), "sparsity": list(sp), "l1": list(err),
            "stage1": np.array(s1[:]).reshape(len(tau_grid), len(theta_grid), H, 2),
            "stage2": np.array(s2[:n2 * H * 2]).reshape(n2, H, 2)}


def sparge_item_order(B: int, H: int, N: int, d: int = 128, causal: bool = False) -> torch.Tensor:
    """-> int32 [B*H*Tm] (CPU tensor): the attention kernel's items (b*H + h)*Tm + i in hand-out order, the eight
    ranges one after the other (diagnostic; runs on the host)."""
    desc = _Desc(B, H, N, d, 1, H * N * d, N * d, d, 0, 0)
    n = B * H * _blocks(N)[0]
    buf = (ctypes.c_int32 * max(n, 1))()
    _check(load_library().sparge_item_order(ctypes.byref(desc), int(causal), buf))
    return torch.frombuffer(buf, dtype=torch.int32)[:n].clone()


def sparge_hilbert_order(T: int, H: int, W: int) -> torch.Tensor:
    """-> int32 [T*H*W] (CPU tensor): the row-major grid cell at every position along the Hilbert curve (Sec. 3.7)."""
    n = T * H * W
    buf = (ctypes.c_int32 * n)()
    _check(load_library().sparge_hilbert_order(T, H, W, buf))
    return torch.frombuffer(buf, dtype=torch.int32).clone()


def sparge_permute_tokens(x: torch.Tensor, perm: torch.Tensor, offset: int = 0, inverse: bool = False,
                          out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Gathers tokens [offset, offset + len(perm)) of a [B,H,N,d] tensor by `perm` (device int32), or scatters
    them back (inverse); the other tokens are copied."""
    if perm.dtype != torch.int32 or not perm.is_cuda or not perm.is_contiguous() or perm.dim() != 1:
        raise SpargeError("perm must be a contiguous int32 vector on the GPU")
    d = _desc(x)
    y = torch.empty_like(x) if out is None else out
    _same_layout(x, y)
    _check(load_library().sparge_permute_tokens(_ptr(x), ctypes.byref(d), _ptr(perm), perm.numel(), int(offset),
                                                int(inverse), _ptr(y), _stream()))
    return y


class AttnKernelTimer:
    """Brackets the next `n` launches of the attention kernel with HIP events (profiling aid).

    Events are created with the HIP runtime directly; elapsed_ms() synchronises on the last stop event
    and returns the per-launch durations of the launches that actually happened.
    """

    def __init__(self, n: int):
        self.n = n
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventQuery.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.starts = (ctypes.c_void_p * n)()
        self.stops = (ctypes.c_void_p * n)()
        for arr in (self.starts, self.stops):
            for k in range(n):
                ev = ctypes.c_void_p()
                if self.hip.hipEventCreate(ctypes.byref(ev)) != 0:
                    raise SpargeError("hipEventCreate failed")
                arr[k] = ev

    def __enter__(self):
        _check(load_library().sparge_set_timing_events(self.starts, self.stops, self.n))
        return self

    def __exit__(self, *exc):
        _check(load_library().sparge_set_timing_events(None, None, 0))

    def elapsed_ms(self):
        out = []
        for k in range(self.n):
            if self.hip.hipEventSynchronize(self.stops[k]) != 0:
                break
            ms = ctypes.c_float(0)
            if self.hip.hipEventElapsedTime(ctypes.byref(ms), self.starts[k], self.stops[k]) != 0:
                break  # this pair was never recorded
            out.append(ms.value)
        return out

    def close(self):
        for arr in (self.starts, self.stops):
            for k in range(self.n):
                self.hip.hipEventDestroy(arr[k])
