"""ctypes front end of the fp64 CPU oracle in ``ciar_oracle.c`` (TEST INFRASTRUCTURE).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It shares nothing with the HIP library: it compiles its own C file with
gcc and talks to it through numpy arrays.

Logit arrays are ``numpy.float32`` (dtype code 0), ``numpy.uint16`` holding raw bfloat16 bits
(dtype code 1) or ``numpy.float64`` (dtype code 2: logits that the oracle itself produced in double
precision), shape [N, row_stride] or [N, V], C-contiguous.

The Interval Head's two linear maps (``interhead_logits``: Sec. 3.2.1, "Interval Head Architecture") are
numpy's fp64 matrix product of the exactly widened bf16 operands plus the bias; ``interhead_quantify`` feeds
those fp64 logits to the quantifier.  Pins: ``tests/test_interhead_oracle_pins.py``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ciar_oracle.c")
_LIB = os.path.join(_HERE, "libciar_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (OpenMP only spreads rows over threads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _CParams(ctypes.Structure):
    _fields_ = [("vocab", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("row_stride", ctypes.c_int64), ("kappa", ctypes.c_double),
                ("confidence", ctypes.c_double), ("radius_max", ctypes.c_double),
                ("tau", ctypes.c_double), ("lower_cap", ctypes.c_double),
                ("upper_cap", ctypes.c_double), ("normalize", ctypes.c_int32),
                ("window", ctypes.c_int32)]


@dataclass
class Params:
    """Parameters of the pass.  ``kappa < 0`` derives the radius from ``confidence``."""
    confidence: float = 0.9
    kappa: float = -1.0
    radius_max: float = 10.0
    tau: float = 0.30
    lower_cap: float = 0.99
    upper_cap: float = 1.01
    normalize: bool = True
    window: int = 8


_lib = None


def _load():
    global _lib
    if _lib is None:
        # (CIAR_ORACLE_LIB: a library built elsewhere from a copy of the source -- the mutation test plants mistakes in
        # such copies and checks that the pins catch them)
        lib = ctypes.CDLL(os.environ.get("CIAR_ORACLE_LIB") or build())
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        pp = ctypes.POINTER(_CParams)
        lib.ciar_oracle_kappa.restype = ctypes.c_double
        lib.ciar_oracle_kappa.argtypes = [ctypes.c_double]
        lib.ciar_oracle_quantify.restype = i32
        lib.ciar_oracle_quantify.argtypes = [vp, vp, vp, i64, pp] + [vp] * 7 + [i32]
        lib.ciar_oracle_dense_intervals.restype = i32
        lib.ciar_oracle_dense_intervals.argtypes = [vp, vp, i64, pp, vp, vp, vp]
        lib.ciar_oracle_quantify_multihead.restype = i32
        lib.ciar_oracle_quantify_multihead.argtypes = [vp, vp, ctypes.c_int32, i64, vp, i64, pp, ctypes.c_int32] + \
            [vp] * 8 + [i32]
        lib.ciar_oracle_interdro_loss.restype = i32
        lib.ciar_oracle_interdro_loss.argtypes = [vp, vp, vp, i64, pp] + [ctypes.c_double] * 4 + [vp, vp, vp, i32]
        lib.ciar_oracle_residual_cdf.restype = ctypes.c_double
        lib.ciar_oracle_residual_cdf.argtypes = [vp, vp, i64, pp, vp]
        lib.ciar_oracle_verify.restype = i32
        lib.ciar_oracle_verify.argtypes = [vp, vp, vp, vp, vp, i64, pp] + [vp] * 6 + [i32]
        _lib = lib
    return _lib


def _logits(a) -> np.ndarray:
    """Accept numpy float32 / uint16(bf16 bits) or a CPU torch tensor (float32 / bfloat16)."""
    if not isinstance(a, np.ndarray):
        import torch
        assert isinstance(a, torch.Tensor) and a.device.type == "cpu"
        if a.dtype == torch.bfloat16:
            a = a.contiguous().view(torch.int16).numpy().view(np.uint16)
        else:
            a = a.contiguous().numpy()
    assert a.dtype in (np.float32, np.uint16, np.float64), a.dtype
    assert a.ndim == 2 and a.flags.c_contiguous
    return a


def _cparams(p: Params, logits: np.ndarray, vocab: int | None) -> _CParams:
    V = int(vocab if vocab is not None else logits.shape[1])
    assert 1 <= V <= logits.shape[1]
    return _CParams(V, {np.dtype(np.float32): 0, np.dtype(np.uint16): 1, np.dtype(np.float64): 2}[logits.dtype], logits.shape[1],
                    float(p.kappa), float(p.confidence), float(p.radius_max), float(p.tau),
                    float(p.lower_cap), float(p.upper_cap), int(bool(p.normalize)), int(p.window))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def kappa(confidence: float) -> float:
    return float(_load().ciar_oracle_kappa(float(confidence)))


def default_threads() -> int:
    return max(1, min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "1024"))))


def _radius(radius, c: np.ndarray):
    """The raw radius tensor (None: scalar mode): same dtype, shape and stride as the logits."""
    if radius is None:
        return None
    r = _logits(radius)
    assert r.shape == c.shape and r.dtype == c.dtype
    return r


def quantify(draft, ids, params: Params, vocab: int | None = None, threads: int | None = None, radius=None):
    """Returns dict of fp64 arrays p_lo, p_mid, p_hi, omega, sigma, score and uint8 flags, each [N].
    ``radius``: raw radius tensor like ``draft`` (r_i = min(kappa * Softplus(raw_i), radius_max)), or None
    for the scalar radius r = min(kappa, radius_max)."""
    c = _logits(draft)
    N = c.shape[0]
    cp = _cparams(params, c, vocab)
    rad = _radius(radius, c)
    ids32 = None if ids is None else np.ascontiguousarray(np.asarray(ids), dtype=np.int32)
    if ids32 is not None:
        assert ids32.shape == (N,) and (N == 0 or (ids32.min() >= 0 and ids32.max() < cp.vocab))
    out = {k: np.empty(N, dtype=np.float64) for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score")}
    out["flags"] = np.empty(N, dtype=np.uint8)
    rc = _load().ciar_oracle_quantify(_ptr(c), _ptr(rad), _ptr(ids32), N, ctypes.byref(cp),
                                      _ptr(out["p_lo"]), _ptr(out["p_mid"]), _ptr(out["p_hi"]),
                                      _ptr(out["omega"]), _ptr(out["sigma"]), _ptr(out["score"]),
                                      _ptr(out["flags"]), threads or default_threads())
    assert rc == 0
    return out


def _bf16_to_f64(a) -> np.ndarray:
    """bf16 values (torch CPU bfloat16 tensor, or numpy uint16 bit patterns) widened exactly to float64."""
    if not isinstance(a, np.ndarray):
        import torch
        assert isinstance(a, torch.Tensor) and a.device.type == "cpu" and a.dtype == torch.bfloat16
        a = a.contiguous().view(torch.int16).numpy().view(np.uint16)
    assert a.dtype == np.uint16
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def interhead_logits(hidden, weight, bias=None):
    """The Interval Head's two linear maps (Sec. 3.2.1, "Interval Head Architecture": output dimension 2|V|,
    c_t = Linear_center(h_t), raw radius = Linear_radius(h_t)) in fp64: hidden [N, D] and weight [2V, D] are bf16
    (widened exactly), bias [2V] or None.  Returns (centre, raw_radius), each [N, V] float64:
    centre[n, j] = sum_k hidden[n, k] weight[j, k] + bias[j], raw_radius[n, j] likewise with weight row V + j."""
    h = _bf16_to_f64(hidden)
    w = _bf16_to_f64(weight)
    assert h.ndim == 2 and w.ndim == 2 and w.shape[1] == h.shape[1] and w.shape[0] % 2 == 0
    V = w.shape[0] // 2
    out = h @ w.T                                                  # numpy's fp64 matrix product is the step
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64)
        assert b.shape == (2 * V,)
        out = out + b[None, :]
    return np.ascontiguousarray(out[:, :V]), np.ascontiguousarray(out[:, V:])


def interhead_quantify(hidden, weight, bias, ids, params: Params, threads: int | None = None):
    """quantify() on the Interval Head's own fp64 logits: r_i = min(kappa * Softplus(raw_i), radius_max)."""
    centre, raw = interhead_logits(hidden, weight, bias)
    return quantify(centre, ids, params, radius=raw, threads=threads)


DRO_TERMS = ("l1_mid", "l1_up", "l1_lo", "ce_mid", "ce_up", "ce_lo", "kl")
DRO_LOSSES = ("center", "upper", "lower", "dro", "total")


def interdro_loss(center, radius, cloud, params: Params, lambda_v: float, lambda_p: float, lambda_beta: float,
                  alpha: float, vocab: int | None = None, threads: int | None = None):
    """Forward value of the Inter-DRO loss.  Returns dict: the seven per-row terms (fp64 [N] each, names in
    DRO_TERMS), ``weights`` [N] and the five scalars of DRO_LOSSES."""
    c, t = _logits(center), _logits(cloud)
    assert c.shape == t.shape and c.dtype == t.dtype
    rad = _radius(radius, c)
    N = c.shape[0]
    cp = _cparams(params, c, vocab)
    rows = np.empty((7, N), dtype=np.float64)
    w = np.empty(N, dtype=np.float64)
    losses = np.empty(5, dtype=np.float64)
    rc = _load().ciar_oracle_interdro_loss(_ptr(c), _ptr(rad), _ptr(t), N, ctypes.byref(cp), float(lambda_v),
                                           float(lambda_p), float(lambda_beta), float(alpha), _ptr(rows), _ptr(w),
                                           _ptr(losses), threads or default_threads())
    assert rc == 0
    out = {k: rows[i] for i, k in enumerate(DRO_TERMS)}
    out["weights"] = w
    out.update({k: float(losses[i]) for i, k in enumerate(DRO_LOSSES)})
    return out


VOTING, ENSEMBLE = 0, 1


def _heads(a) -> np.ndarray:
    """[H, N, stride] logits of H heads as one C-contiguous array (float32, or uint16 bfloat16 bits)."""
    if not isinstance(a, np.ndarray):
        import torch
        assert isinstance(a, torch.Tensor) and a.device.type == "cpu" and a.dim() == 3
        if a.dtype == torch.bfloat16:
            a = a.contiguous().view(torch.int16).numpy().view(np.uint16)
        else:
            a = a.contiguous().numpy()
    assert a.dtype in (np.float32, np.uint16) and a.ndim == 3 and a.flags.c_contiguous
    return a


def quantify_multihead(draft_heads, ids, params: Params, strategy: int, vocab: int | None = None,
                       threads: int | None = None, radius_heads=None):
    """Quantifier over H heads ([H, N, stride]).  VOTING: per-head fp64 arrays [H, N], head_flags [H, N] and the
    voted flags [N].  ENSEMBLE: arrays [N] from the token-wise average of the heads' curves."""
    c = _heads(draft_heads)
    H, N = c.shape[0], c.shape[1]
    cp = _cparams(params, c[0], vocab)
    rad = None
    if radius_heads is not None:
        rad = _heads(radius_heads)
        assert rad.shape == c.shape and rad.dtype == c.dtype
    ids32 = None if ids is None else np.ascontiguousarray(np.asarray(ids), dtype=np.int32)
    if ids32 is not None:
        assert ids32.shape == (N,) and (N == 0 or (ids32.min() >= 0 and ids32.max() < cp.vocab))
    shape = (H, N) if strategy == VOTING else (N,)
    out = {k: np.empty(shape, dtype=np.float64) for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score")}
    out["flags"] = np.empty(N, dtype=np.uint8)
    if strategy == VOTING:
        out["head_flags"] = np.empty((H, N), dtype=np.uint8)
    rc = _load().ciar_oracle_quantify_multihead(
        _ptr(c), _ptr(rad), H, c.shape[1] * c.shape[2], _ptr(ids32), N, ctypes.byref(cp), int(strategy),
        _ptr(out["p_lo"]), _ptr(out["p_mid"]), _ptr(out["p_hi"]), _ptr(out["omega"]), _ptr(out["sigma"]),
        _ptr(out["score"]), _ptr(out["flags"]), _ptr(out.get("head_flags")), threads or default_threads())
    assert rc == 0
    return out


def dense_intervals(draft, params: Params, vocab: int | None = None, radius=None):
    """Returns (p_lo, p_mid, p_hi), fp64 [N, V].  ``radius`` as for :func:`quantify`."""
    c = _logits(draft)
    cp = _cparams(params, c, vocab)
    rad = _radius(radius, c)
    N, V = c.shape[0], cp.vocab
    lo, mid, hi = (np.empty((N, V), dtype=np.float64) for _ in range(3))
    rc = _load().ciar_oracle_dense_intervals(_ptr(c), _ptr(rad), N, ctypes.byref(cp), _ptr(lo), _ptr(mid),
                                             _ptr(hi))
    assert rc == 0
    return lo, mid, hi


def residual_cdf(draft, target, row: int, params: Params, vocab: int | None = None):
    """Inclusive running sum of max(0, q - p) over the vocabulary of one row, and its total R."""
    c, t = _logits(draft), _logits(target)
    assert c.shape == t.shape and c.dtype == t.dtype
    cp = _cparams(params, c, vocab)
    cdf = np.empty(cp.vocab, dtype=np.float64)
    R = _load().ciar_oracle_residual_cdf(_ptr(c), _ptr(t), int(row), ctypes.byref(cp), _ptr(cdf))
    return cdf, float(R)


def verify(draft, target, ids, u_accept, u_resample, params: Params, vocab: int | None = None,
           threads: int | None = None):
    """Returns dict: accept uint8 [N], row_id int32 [N], accept_len / resampled_id int32 [W],
    log_ratio / res_margin fp64 [N] (diagnostics for the margin rule)."""
    c, t = _logits(draft), _logits(target)
    assert c.shape == t.shape and c.dtype == t.dtype
    N = c.shape[0]
    cp = _cparams(params, c, vocab)
    ids32 = np.ascontiguousarray(np.asarray(ids), dtype=np.int32)
    ua = np.ascontiguousarray(np.asarray(u_accept), dtype=np.float32)
    ur = np.ascontiguousarray(np.asarray(u_resample), dtype=np.float32)
    assert ids32.shape == (N,) and ua.shape == (N,) and ur.shape == (N,)
    assert N == 0 or (ids32.min() >= 0 and ids32.max() < cp.vocab)
    W = (N + cp.window - 1) // cp.window
    out = {"accept": np.empty(N, dtype=np.uint8), "row_id": np.empty(N, dtype=np.int32),
           "accept_len": np.empty(W, dtype=np.int32), "resampled_id": np.empty(W, dtype=np.int32),
           "log_ratio": np.empty(N, dtype=np.float64), "res_margin": np.empty(N, dtype=np.float64)}
    rc = _load().ciar_oracle_verify(_ptr(c), _ptr(t), _ptr(ids32), _ptr(ua), _ptr(ur), N, ctypes.byref(cp),
                                    _ptr(out["accept"]), _ptr(out["row_id"]), _ptr(out["accept_len"]),
                                    _ptr(out["resampled_id"]), _ptr(out["log_ratio"]),
                                    _ptr(out["res_margin"]), threads or default_threads())
    assert rc == 0
    return out
