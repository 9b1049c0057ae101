"""Thin ctypes binding of ``libciar.so``: argument marshalling only.

Every step of the pass runs in the HIP kernels behind the C ABI (``include/ciar.h``); this module
turns torch tensors into device pointers, allocates output tensors and checks the status code.
There is no CPU fallback: if the library has not been built, importing a function raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libciar.so")

CIAR_F32, CIAR_BF16 = 0, 1
STATUS = {0: "CIAR_OK", -1: "CIAR_EINVAL", -2: "CIAR_EALIGN", -3: "CIAR_EWORKSPACE",
          -4: "CIAR_EUNSUPPORTED", -5: "CIAR_EHIP"}


class CiarParams(ctypes.Structure):
    """Mirror of ``struct ciar_params``."""
    _fields_ = [("struct_size", ctypes.c_uint32), ("vocab", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("window", ctypes.c_int32), ("row_stride", ctypes.c_int64),
                ("confidence", ctypes.c_float), ("radius_scale", ctypes.c_float),
                ("radius_max", ctypes.c_float), ("tau", ctypes.c_float),
                ("lower_cap", ctypes.c_float), ("upper_cap", ctypes.c_float),
                ("normalize", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class CiarError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (``python -m paper_2603_25463_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
        pp = ctypes.POINTER(CiarParams)
        L.ciar_params_default.restype = None
        L.ciar_params_default.argtypes = [pp]
        L.ciar_workspace_bytes.restype = sz
        L.ciar_workspace_bytes.argtypes = [i64, pp]
        L.ciar_quantify.restype = ctypes.c_int
        L.ciar_quantify.argtypes = [vp, vp, vp, i64, pp] + [vp] * 7 + [vp, sz, vp]
        L.ciar_verify.restype = ctypes.c_int
        L.ciar_verify.argtypes = [vp, vp, vp, vp, vp, i64, pp] + [vp] * 4 + [vp, sz, vp]
        L.ciar_quantify_verify.restype = ctypes.c_int
        L.ciar_quantify_verify.argtypes = [vp, vp, vp, vp, vp, vp, i64, pp] + [vp] * 11 + [vp, sz, vp]
        L.ciar_quantify_verify_static.restype = ctypes.c_int
        L.ciar_quantify_verify_static.argtypes = [vp, vp, vp, vp, vp, vp, i64, pp] + [vp] * 11 + [vp]
        L.ciar_stream_rows.restype = ctypes.c_int
        L.ciar_stream_rows.argtypes = [vp, vp, vp, vp, vp, vp, i64, pp] + [vp] * 11 + [vp, sz, vp]
        L.ciar_stream_rows_timed.restype = ctypes.c_int
        L.ciar_stream_rows_timed.argtypes = [vp, vp, vp, vp, vp, vp, i64, pp] + [vp] * 11 + [vp, sz, vp, vp, vp]
        L.ciar_finish_rows.restype = ctypes.c_int
        L.ciar_finish_rows.argtypes = [vp, vp, vp, vp, vp, vp, i64, pp] + [vp] * 11 + [vp, sz, vp]
        L.ciar_window_epilogue.restype = ctypes.c_int
        L.ciar_window_epilogue.argtypes = [vp, vp, i64, pp, vp, vp, vp]
        L.ciar_dense_intervals.restype = ctypes.c_int
        L.ciar_dense_intervals.argtypes = [vp, vp, i64, pp, vp, vp, vp, vp]
        L.ciar_multihead_workspace_bytes.restype = sz
        L.ciar_multihead_workspace_bytes.argtypes = [i64, ctypes.c_int32, pp]
        L.ciar_quantify_multihead.restype = ctypes.c_int
        L.ciar_quantify_multihead.argtypes = [vp, vp, ctypes.c_int32, i64, vp, i64, pp, ctypes.c_int32] + \
            [vp] * 8 + [vp, sz, vp]
        L.ciar_interdro_loss.restype = ctypes.c_int
        L.ciar_interdro_loss.argtypes = [vp, vp, vp, i64, pp] + [ctypes.c_float] * 4 + [vp, vp, vp, vp]
        L.ciar_read_rows.restype = ctypes.c_int
        L.ciar_read_rows.argtypes = [vp, vp, i64, pp, vp, vp]
        L.ciar_read_rows_timed.restype = ctypes.c_int
        L.ciar_read_rows_timed.argtypes = [vp, vp, i64, pp, vp, vp, vp, vp]
        L.ciar_interhead_workspace_bytes.restype = sz
        L.ciar_interhead_workspace_bytes.argtypes = [i64, pp]
        L.ciar_interhead_logits.restype = ctypes.c_int
        L.ciar_interhead_logits.argtypes = [vp, vp, vp, ctypes.c_int32, i64, pp, vp, vp, vp]
        L.ciar_interhead_logits_timed.restype = ctypes.c_int
        L.ciar_interhead_logits_timed.argtypes = [vp, vp, vp, ctypes.c_int32, i64, pp, vp, vp, vp, vp, vp]
        L.ciar_interhead_quantify.restype = ctypes.c_int
        L.ciar_interhead_quantify.argtypes = [vp, vp, vp, ctypes.c_int32, vp, i64, pp] + [vp] * 7 + [vp, sz, vp]
        L.ciar_width_polynomial.restype = ctypes.c_int
        L.ciar_width_polynomial.argtypes = [pp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
        L.ciar_last_error.restype = ctypes.c_char_p
        L.ciar_last_error.argtypes = []
        L.ciar_version.restype = ctypes.c_char_p
        L.ciar_version.argtypes = []
        _lib = L
    return _lib


def version() -> str:
    return lib().ciar_version().decode()


def last_error() -> str:
    return lib().ciar_last_error().decode()


@dataclass
class Params:
    """Python-side parameters; ``radius_scale < 0`` derives the radius from ``confidence``."""
    confidence: float = 0.9
    radius_scale: float = -1.0
    radius_max: float = 10.0
    tau: float = 0.30
    lower_cap: float = 0.99
    upper_cap: float = 1.01
    normalize: bool = True
    window: int = 8

    def to_c(self, logits: torch.Tensor, vocab: int | None = None) -> CiarParams:
        p = CiarParams()
        lib().ciar_params_default(ctypes.byref(p))
        if logits.dtype == torch.float32:
            p.dtype = CIAR_F32
        elif logits.dtype == torch.bfloat16:
            p.dtype = CIAR_BF16
        else:
            raise TypeError(f"logits must be float32 or bfloat16, got {logits.dtype}")
        if logits.dim() != 2 or logits.stride(1) != 1:
            raise ValueError("logits must be a 2-D tensor with unit stride along the vocabulary")
        p.vocab = int(logits.shape[1] if vocab is None else vocab)
        p.row_stride = int(logits.stride(0)) if logits.shape[0] > 1 else max(int(logits.stride(0)), p.vocab)
        p.window = int(self.window)
        p.confidence = float(self.confidence)
        p.radius_scale = float(self.radius_scale)
        p.radius_max = float(self.radius_max)
        p.tau = float(self.tau)
        p.lower_cap = float(self.lower_cap)
        p.upper_cap = float(self.upper_cap)
        p.normalize = int(bool(self.normalize))
        return p


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(rc: int):
    if rc != 0:
        raise CiarError(rc, last_error())


# public names of the marshalling helpers (bench.py and the tests call the C ABI directly through them)
ptr, stream_handle, check = _ptr, _stream, _check


def _need_cuda(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("all tensors must live on the GPU")


def _like_draft(t, draft, name: str):
    """``target`` / ``radius`` tensors share the layout of the draft logits."""
    if t is not None and (t.dtype != draft.dtype or t.shape != draft.shape or t.stride() != draft.stride()):
        raise ValueError(f"{name} must match draft in dtype, shape and strides")


def width_polynomial(cparams: CiarParams):
    """``ciar_width_polynomial`` (host only): (four coefficients, x_max) for the call's scalar radius."""
    coef = (ctypes.c_float * 4)()
    xmax = ctypes.c_float()
    _check(lib().ciar_width_polynomial(ctypes.byref(cparams), coef, ctypes.byref(xmax)))
    return [float(v) for v in coef], float(xmax.value)


def workspace_bytes(N: int, cparams: CiarParams) -> int:
    return int(lib().ciar_workspace_bytes(int(N), ctypes.byref(cparams)))


def _workspace(N: int, cp: CiarParams, dev, workspace):
    """The caller's workspace, or a fresh one of the size the library asks for."""
    if workspace is None:
        workspace = torch.empty(max(workspace_bytes(N, cp), 16), dtype=torch.uint8, device=dev)
    return workspace, workspace.numel() * workspace.element_size()


def quantify(draft: torch.Tensor, ids: torch.Tensor | None, params: Params, vocab: int | None = None,
             stream=None, out: dict | None = None, workspace: torch.Tensor | None = None,
             radius: torch.Tensor | None = None) -> dict:
    """``ciar_quantify``.  Returns dict of [N] tensors: p_lo, p_mid, p_hi, omega, sigma, score (float32)
    and flags (uint8).  ``out`` may carry preallocated tensors under the same names.  ``radius``: the raw
    radius tensor (tensor mode), laid out like ``draft``."""
    _need_cuda(draft, ids, radius)
    _like_draft(radius, draft, "radius")
    N, dev = draft.shape[0], draft.device
    cp = params.to_c(draft, vocab)
    workspace, wsb = _workspace(N, cp, dev, workspace)
    o = dict(out) if out else {}
    for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score"):
        o.setdefault(k, torch.empty(N, dtype=torch.float32, device=dev))
    o.setdefault("flags", torch.empty(N, dtype=torch.uint8, device=dev))
    _check(lib().ciar_quantify(_ptr(draft), _ptr(radius), _ptr(ids), N, ctypes.byref(cp),
                               _ptr(o["p_lo"]), _ptr(o["p_mid"]), _ptr(o["p_hi"]), _ptr(o["omega"]),
                               _ptr(o["sigma"]), _ptr(o["score"]), _ptr(o["flags"]), _ptr(workspace), wsb,
                               _stream(stream)))
    return o


def _verify_outputs(N: int, K: int, dev, out: dict | None) -> dict:
    W = (N + K - 1) // K
    o = dict(out) if out else {}
    o.setdefault("accept", torch.empty(N, dtype=torch.uint8, device=dev))
    o.setdefault("row_id", torch.empty(N, dtype=torch.int32, device=dev))
    o.setdefault("accept_len", torch.empty(W, dtype=torch.int32, device=dev))
    o.setdefault("resampled_id", torch.empty(W, dtype=torch.int32, device=dev))
    return o


def verify(draft, target, ids, u_accept, u_resample, params: Params, vocab: int | None = None,
           stream=None, out: dict | None = None, workspace: torch.Tensor | None = None) -> dict:
    """``ciar_verify``.  Returns accept uint8 [N], row_id int32 [N], accept_len / resampled_id int32 [W]."""
    _need_cuda(draft, target, ids, u_accept, u_resample)
    N, dev = draft.shape[0], draft.device
    cp = params.to_c(draft, vocab)
    _like_draft(target, draft, "target")
    o = _verify_outputs(N, cp.window, dev, out)
    workspace, wsb = _workspace(N, cp, dev, workspace)
    _check(lib().ciar_verify(_ptr(draft), _ptr(target), _ptr(ids), _ptr(u_accept), _ptr(u_resample), N,
                             ctypes.byref(cp), _ptr(o["accept"]), _ptr(o["row_id"]), _ptr(o["accept_len"]),
                             _ptr(o["resampled_id"]), _ptr(workspace), wsb, _stream(stream)))
    return o


def quantify_verify(draft, target, ids, u_accept, u_resample, params: Params, vocab: int | None = None,
                    stream=None, out: dict | None = None, workspace: torch.Tensor | None = None,
                    radius: torch.Tensor | None = None) -> dict:
    """``ciar_quantify_verify``: the fused pass; union of the outputs of quantify and verify."""
    _need_cuda(draft, target, ids, u_accept, u_resample, radius)
    N, dev = draft.shape[0], draft.device
    cp = params.to_c(draft, vocab)
    _like_draft(target, draft, "target")
    _like_draft(radius, draft, "radius")
    o = _verify_outputs(N, cp.window, dev, out)
    for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score"):
        o.setdefault(k, torch.empty(N, dtype=torch.float32, device=dev))
    o.setdefault("flags", torch.empty(N, dtype=torch.uint8, device=dev))
    workspace, wsb = _workspace(N, cp, dev, workspace)
    _check(lib().ciar_quantify_verify(
        _ptr(draft), _ptr(radius), _ptr(target), _ptr(ids), _ptr(u_accept), _ptr(u_resample), N, ctypes.byref(cp),
        _ptr(o["p_lo"]), _ptr(o["p_mid"]), _ptr(o["p_hi"]), _ptr(o["omega"]), _ptr(o["sigma"]),
        _ptr(o["score"]), _ptr(o["flags"]), _ptr(o["accept"]), _ptr(o["row_id"]), _ptr(o["accept_len"]),
        _ptr(o["resampled_id"]), _ptr(workspace), wsb, _stream(stream)))
    return o


STATIC_MAX_ROWS = 32768


def quantify_verify_static(draft, target, ids, u_accept, u_resample, params: Params, out: dict,
                           vocab: int | None = None, stream=None, radius: torch.Tensor | None = None) -> dict:
    """``ciar_quantify_verify_static``: the fused pass on the library's built-in scratch buffer.  Nothing is
    allocated here either: ``out`` must carry every output tensor (names as ``quantify_verify``)."""
    _need_cuda(draft, target, ids, u_accept, u_resample, radius)
    _like_draft(target, draft, "target")
    _like_draft(radius, draft, "radius")
    cp = params.to_c(draft, vocab)
    g = lambda k: _ptr(out.get(k))
    _check(lib().ciar_quantify_verify_static(
        _ptr(draft), _ptr(radius), _ptr(target), _ptr(ids), _ptr(u_accept), _ptr(u_resample), draft.shape[0],
        ctypes.byref(cp), g("p_lo"), g("p_mid"), g("p_hi"), g("omega"), g("sigma"), g("score"), g("flags"),
        g("accept"), g("row_id"), g("accept_len"), g("resampled_id"), _stream(stream)))
    return out


def _staged(entry, draft, target, ids, u_accept, u_resample, params: Params, workspace: torch.Tensor,
            with_intervals: bool, vocab, stream, out, radius) -> dict:
    _need_cuda(draft, target, ids, u_accept, u_resample, workspace, radius)
    _like_draft(radius, draft, "radius")
    N, dev = draft.shape[0], draft.device
    cp = params.to_c(draft, vocab)
    o = dict(out) if out else {}
    if target is not None:
        o = _verify_outputs(N, cp.window, dev, o)
    if with_intervals:
        for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score"):
            o.setdefault(k, torch.empty(N, dtype=torch.float32, device=dev))
        o.setdefault("flags", torch.empty(N, dtype=torch.uint8, device=dev))
    g = lambda k: _ptr(o.get(k))
    _check(entry(
        _ptr(draft), _ptr(radius), _ptr(target), _ptr(ids), _ptr(u_accept), _ptr(u_resample), N, ctypes.byref(cp),
        g("p_lo"), g("p_mid"), g("p_hi"), g("omega"), g("sigma"), g("score"), g("flags"), g("accept"),
        g("row_id"), g("accept_len"), g("resampled_id"), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))
    return o


def stream_rows(draft, target, ids, u_accept, u_resample, params: Params, workspace: torch.Tensor,
                with_intervals: bool = True, vocab: int | None = None, stream=None, out: dict | None = None,
                radius: torch.Tensor | None = None, events=None) -> dict:
    """``ciar_stream_rows``: stage 1, the streaming kernel (a quantify-only call also finishes its rows where the
    launch shape allows).  Returns the output tensors (allocated here unless passed in ``out``); hand the same dict
    and the same arguments to ``finish_rows``.  ``events`` = (start, stop), two ``torch.cuda.Event`` objects with
    timing enabled that have been recorded at least once (which creates the HIP events behind them):
    ``ciar_stream_rows_timed``, the kernel's dispatch records them at its start and end."""
    if events is None:
        return _staged(lib().ciar_stream_rows, draft, target, ids, u_accept, u_resample, params, workspace,
                       with_intervals, vocab, stream, out, radius)
    start, stop = events
    entry = lambda *a: lib().ciar_stream_rows_timed(*a, start.cuda_event, stop.cuda_event)
    return _staged(entry, draft, target, ids, u_accept, u_resample, params, workspace, with_intervals, vocab, stream,
                   out, radius)


def finish_rows(draft, target, ids, u_accept, u_resample, params: Params, workspace: torch.Tensor,
                with_intervals: bool = True, vocab: int | None = None, stream=None, out: dict | None = None,
                radius: torch.Tensor | None = None) -> dict:
    """``ciar_finish_rows``: stage 2 on a workspace filled by ``stream_rows`` (same arguments, same ``out``):
    whatever per-row finishing is left, the residual draws and the window outputs."""
    return _staged(lib().ciar_finish_rows, draft, target, ids, u_accept, u_resample, params, workspace,
                   with_intervals, vocab, stream, out, radius)


def window_epilogue(accept: torch.Tensor, row_id: torch.Tensor, params: Params, stream=None,
                    out: dict | None = None) -> dict:
    """``ciar_window_epilogue``: accept_len / resampled_id int32 [W] from per-row accept / row_id."""
    _need_cuda(accept, row_id)
    N, K = accept.shape[0], int(params.window)
    cp = CiarParams()
    lib().ciar_params_default(ctypes.byref(cp))
    cp.window = K
    W = (N + K - 1) // K
    o = dict(out) if out else {}
    o.setdefault("accept_len", torch.empty(W, dtype=torch.int32, device=accept.device))
    o.setdefault("resampled_id", torch.empty(W, dtype=torch.int32, device=accept.device))
    _check(lib().ciar_window_epilogue(_ptr(accept), _ptr(row_id), N, ctypes.byref(cp), _ptr(o["accept_len"]),
                                      _ptr(o["resampled_id"]), _stream(stream)))
    return o


def dense_intervals(draft: torch.Tensor, params: Params, vocab: int | None = None, stream=None,
                    radius: torch.Tensor | None = None):
    """``ciar_dense_intervals`` (test export): (p_lo, p_mid, p_hi), float32 [N, V]."""
    _need_cuda(draft, radius)
    _like_draft(radius, draft, "radius")
    N, dev = draft.shape[0], draft.device
    cp = params.to_c(draft, vocab)
    lo, mid, hi = (torch.empty((N, cp.vocab), dtype=torch.float32, device=dev) for _ in range(3))
    _check(lib().ciar_dense_intervals(_ptr(draft), _ptr(radius), N, ctypes.byref(cp), _ptr(lo), _ptr(mid), _ptr(hi),
                                      _stream(stream)))
    return lo, mid, hi


def read_rows(draft: torch.Tensor, target: torch.Tensor | None, params: Params, vocab: int | None = None,
              out: torch.Tensor | None = None, stream=None):
    """``ciar_read_rows`` (measurement aid): the sum of every row's logits, float32 [N]."""
    _need_cuda(draft)
    N, dev = draft.shape[0], draft.device
    cp = params.to_c(draft, vocab)
    if out is None:
        out = torch.empty(N, dtype=torch.float32, device=dev)
    _check(lib().ciar_read_rows(_ptr(draft), _ptr(target), N, ctypes.byref(cp), _ptr(out), _stream(stream)))
    return out


VOTING, ENSEMBLE = 0, 1


def quantify_multihead(draft_heads: torch.Tensor, ids: torch.Tensor | None, params: Params, strategy: int,
                       vocab: int | None = None, stream=None, radius_heads: torch.Tensor | None = None,
                       workspace: torch.Tensor | None = None) -> dict:
    """``ciar_quantify_multihead``.  ``draft_heads`` (and ``radius_heads``): [H, N, stride].  VOTING: per-head
    float outputs [H, N], ``head_flags`` [H, N] and the voted ``flags`` [N]; ENSEMBLE: all outputs [N]."""
    _need_cuda(draft_heads, ids, radius_heads)
    if draft_heads.dim() != 3 or draft_heads.stride(2) != 1:
        raise ValueError("draft_heads must be [H, N, stride] with unit stride along the vocabulary")
    if radius_heads is not None and (radius_heads.dtype != draft_heads.dtype or radius_heads.shape != draft_heads.shape
                                     or radius_heads.stride() != draft_heads.stride()):
        raise ValueError("radius_heads must match draft_heads in dtype, shape and strides")
    H, N, dev = draft_heads.shape[0], draft_heads.shape[1], draft_heads.device
    cp = params.to_c(draft_heads[0], vocab)
    head_stride = int(draft_heads.stride(0)) if H > 1 else N * int(cp.row_stride)
    shape = (H, N) if strategy == VOTING else (N,)
    o = {k: torch.empty(shape, dtype=torch.float32, device=dev)
         for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score")}
    o["flags"] = torch.empty(N, dtype=torch.uint8, device=dev)
    if strategy == VOTING:
        o["head_flags"] = torch.empty((H, N), dtype=torch.uint8, device=dev)
    if workspace is None:
        nbytes = int(lib().ciar_multihead_workspace_bytes(N, H, ctypes.byref(cp)))
        workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=dev)
    _check(lib().ciar_quantify_multihead(
        _ptr(draft_heads), _ptr(radius_heads), H, head_stride, _ptr(ids), N, ctypes.byref(cp), int(strategy),
        _ptr(o["p_lo"]), _ptr(o["p_mid"]), _ptr(o["p_hi"]), _ptr(o["omega"]), _ptr(o["sigma"]), _ptr(o["score"]),
        _ptr(o["flags"]), _ptr(o.get("head_flags")), _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream(stream)))
    return o


DRO_TERMS = ("l1_mid", "l1_up", "l1_lo", "ce_mid", "ce_up", "ce_lo", "kl")
DRO_LOSSES = ("center", "upper", "lower", "dro", "total")


def interdro_loss(center: torch.Tensor, radius: torch.Tensor | None, cloud: torch.Tensor, params: Params,
                  lambda_v: float, lambda_p: float, lambda_beta: float, alpha: float, vocab: int | None = None,
                  stream=None) -> dict:
    """``ciar_interdro_loss`` (forward only).  Returns ``terms`` float32 [7, N] (rows named by DRO_TERMS),
    ``weights`` float32 [N] and ``losses`` float32 [5] (named by DRO_LOSSES), all on the GPU."""
    _need_cuda(center, radius, cloud)
    _like_draft(cloud, center, "cloud")
    _like_draft(radius, center, "radius")
    N, dev = center.shape[0], center.device
    cp = params.to_c(center, vocab)
    o = {"terms": torch.empty((7, N), dtype=torch.float32, device=dev),
         "weights": torch.empty(N, dtype=torch.float32, device=dev),
         "losses": torch.empty(5, dtype=torch.float32, device=dev)}
    _check(lib().ciar_interdro_loss(_ptr(center), _ptr(radius), _ptr(cloud), N, ctypes.byref(cp), float(lambda_v),
                                    float(lambda_p), float(lambda_beta), float(alpha), _ptr(o["terms"]),
                                    _ptr(o["weights"]), _ptr(o["losses"]), _stream(stream)))
    return o


def _head_params(hidden: torch.Tensor, weight: torch.Tensor, bias, params: Params, row_stride: int | None):
    """Checks the Interval Head operands and returns (N, D, V, ciar_params) for fp32 logits of the given stride."""
    _need_cuda(hidden, weight, bias)
    if hidden.dtype != torch.bfloat16 or weight.dtype != torch.bfloat16:
        raise TypeError("hidden and weight must be bfloat16")
    if hidden.dim() != 2 or weight.dim() != 2 or not hidden.is_contiguous() or not weight.is_contiguous():
        raise ValueError("hidden [N, D] and weight [2V, D] must be contiguous 2-D tensors")
    if weight.shape[1] != hidden.shape[1] or weight.shape[0] % 2:
        raise ValueError("weight must be [2V, D] with D = hidden.shape[1]")
    N, D, V = hidden.shape[0], hidden.shape[1], weight.shape[0] // 2
    if bias is not None and (bias.dtype != torch.float32 or bias.shape != (2 * V,) or not bias.is_contiguous()):
        raise ValueError("bias must be a contiguous float32 tensor of 2V entries")
    stride = V if row_stride is None else int(row_stride)
    cp = params.to_c(torch.empty((0, stride), dtype=torch.float32), V)
    cp.row_stride = stride
    return N, D, V, cp


head_params = _head_params


def interhead_logits(hidden: torch.Tensor, weight: torch.Tensor, bias: torch.Tensor | None, params: Params,
                     row_stride: int | None = None, stream=None, out: tuple | None = None, events: tuple | None = None):
    """``ciar_interhead_logits``: (centre, raw radius), float32 [N, row_stride] each (only the first V columns
    of a row are written).  ``events`` = (start, stop) torch events recorded by the kernel's own dispatch
    (``ciar_interhead_logits_timed``)."""
    N, D, V, cp = _head_params(hidden, weight, bias, params, row_stride)
    if out is None:
        out = (torch.empty((N, cp.row_stride), dtype=torch.float32, device=hidden.device),
               torch.empty((N, cp.row_stride), dtype=torch.float32, device=hidden.device))
    _need_cuda(*out)
    if events is None:
        _check(lib().ciar_interhead_logits(_ptr(hidden), _ptr(weight), _ptr(bias), D, N, ctypes.byref(cp),
                                           _ptr(out[0]), _ptr(out[1]), _stream(stream)))
    else:
        _check(lib().ciar_interhead_logits_timed(_ptr(hidden), _ptr(weight), _ptr(bias), D, N, ctypes.byref(cp),
                                                 _ptr(out[0]), _ptr(out[1]), _stream(stream),
                                                 events[0].cuda_event, events[1].cuda_event))
    return out


def interhead_workspace_bytes(N: int, cparams: CiarParams) -> int:
    return int(lib().ciar_interhead_workspace_bytes(int(N), ctypes.byref(cparams)))


def interhead_quantify(hidden: torch.Tensor, weight: torch.Tensor, bias: torch.Tensor | None,
                       ids: torch.Tensor | None, params: Params, row_stride: int | None = None, stream=None,
                       out: dict | None = None, workspace: torch.Tensor | None = None) -> dict:
    """``ciar_interhead_quantify``: the Interval Head's contraction, then the tensor-radius quantifier on its
    logits.  Outputs as ``quantify``."""
    N, D, V, cp = _head_params(hidden, weight, bias, params, row_stride)
    _need_cuda(ids)
    dev = hidden.device
    need = interhead_workspace_bytes(N, cp)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    _need_cuda(workspace)
    o = dict(out) if out else {}
    for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score"):
        o.setdefault(k, torch.empty(N, dtype=torch.float32, device=dev))
    o.setdefault("flags", torch.empty(N, dtype=torch.uint8, device=dev))
    _check(lib().ciar_interhead_quantify(_ptr(hidden), _ptr(weight), _ptr(bias), D, _ptr(ids), N, ctypes.byref(cp),
                                         _ptr(o["p_lo"]), _ptr(o["p_mid"]), _ptr(o["p_hi"]), _ptr(o["omega"]),
                                         _ptr(o["sigma"]), _ptr(o["score"]), _ptr(o["flags"]), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)))
    return o
