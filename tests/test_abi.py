"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function that
include/ciar.h declares, and rejects bad arguments with the documented status codes before any
launch.  Pointers passed here are fake device addresses; they are validated, never dereferenced."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ciar.h")


@pytest.fixture(scope="module")
def L():
    from paper_2603_25463_amd import build as _build
    from paper_2603_25463_amd import binding
    _build.build(force=False)
    return binding.lib()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ciar_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = _declared_functions()
    for n in ("ciar_quantify", "ciar_verify", "ciar_quantify_verify", "ciar_dense_intervals",
              "ciar_stream_rows", "ciar_stream_rows_timed", "ciar_finish_rows", "ciar_window_epilogue", "ciar_read_rows", "ciar_read_rows_timed", "ciar_interdro_loss", "ciar_quantify_multihead", "ciar_multihead_workspace_bytes",
              "ciar_workspace_bytes", "ciar_width_polynomial", "ciar_params_default", "ciar_last_error", "ciar_version"):
        assert n in names


def test_library_exports_every_declared_symbol(L):
    for n in _declared_functions():
        assert hasattr(L, n), n


def test_struct_layout_matches_the_binding(L):
    from paper_2603_25463_amd.binding import CiarParams
    p = CiarParams()
    L.ciar_params_default(ctypes.byref(p))
    assert p.struct_size == ctypes.sizeof(CiarParams) == 56
    assert (p.dtype, p.window, p.normalize, p.reserved) == (0, 8, 1, 0)
    assert abs(p.confidence - 0.9) < 1e-7 and p.radius_scale < 0 and p.radius_max == 10.0
    assert abs(p.tau - 0.30) < 1e-7 and abs(p.lower_cap - 0.99) < 1e-7 and abs(p.upper_cap - 1.01) < 1e-7


def _params(L, **kw):
    from paper_2603_25463_amd.binding import CiarParams
    p = CiarParams()
    L.ciar_params_default(ctypes.byref(p))
    p.vocab, p.row_stride = 1024, 1024
    for k, v in kw.items():
        setattr(p, k, v)
    return p


FAKE = 0x7f0000000000          # 16-byte aligned, never dereferenced on an error path


def _quantify(L, p, draft=FAKE, N=4, out=FAKE + 4096, ws=FAKE + 8192, wsb=1 << 20):
    return L.ciar_quantify(draft, None, None, N, ctypes.byref(p), out, None, None, None, None, None, None,
                           ws, wsb, None)


def test_argument_errors_are_reported_before_any_launch(L):
    from paper_2603_25463_amd.binding import last_error
    EINVAL, EALIGN, EWORK, EUNSUP = -1, -2, -3, -4
    assert _quantify(L, _params(L, struct_size=8)) == EINVAL and "struct_size" in last_error()
    assert _quantify(L, _params(L, vocab=0)) == EINVAL
    assert _quantify(L, _params(L, vocab=40000)) == EUNSUP and "maximum" in last_error()
    assert _quantify(L, _params(L, vocab=70000, row_stride=70000, dtype=1)) == EUNSUP
    assert _quantify(L, _params(L, dtype=7)) == EUNSUP
    assert _quantify(L, _params(L, row_stride=1000)) == EINVAL            # stride < vocab
    assert _quantify(L, _params(L, vocab=1001, row_stride=1001)) == EALIGN  # 4004 bytes per row
    assert _quantify(L, _params(L, window=0)) == EINVAL
    assert _quantify(L, _params(L, confidence=1.0)) == EINVAL
    assert _quantify(L, _params(L, confidence=1.0, radius_scale=0.5), N=0) == 0   # override: gamma unused
    assert _quantify(L, _params(L, radius_max=-1.0)) == EINVAL
    assert _quantify(L, _params(L, tau=float("nan"))) == EINVAL
    assert _quantify(L, _params(L, lower_cap=1.5)) == EINVAL
    assert _quantify(L, _params(L, reserved=1)) == EINVAL
    assert _quantify(L, _params(L), draft=None) == EINVAL and "draft_logits" in last_error()
    assert _quantify(L, _params(L), draft=FAKE + 4) == EALIGN
    assert _quantify(L, _params(L), N=-1) == EINVAL
    assert _quantify(L, _params(L), out=None) == EINVAL and "output" in last_error()
    assert L.ciar_quantify(FAKE, None, None, 4, None, FAKE, None, None, None, None, None, None, FAKE, 4096, None) == EINVAL
    # the workspace carries the per-row statistics between the two kernels: always required
    assert _quantify(L, _params(L), ws=None, wsb=0) == EWORK and "workspace" in last_error()
    assert _quantify(L, _params(L), wsb=64) == EWORK
    assert _quantify(L, _params(L), ws=FAKE + 8) == EALIGN
    # verify: required inputs, workspace rules
    p = _params(L)
    a = ctypes.byref(p)
    assert L.ciar_verify(FAKE, None, FAKE, FAKE, FAKE, 4, a, FAKE, FAKE, None, None, None, 0, None) == EINVAL
    assert L.ciar_verify(FAKE, FAKE, None, FAKE, FAKE, 4, a, FAKE, FAKE, None, None, None, 0, None) == EINVAL
    assert L.ciar_verify(FAKE, FAKE, FAKE, None, FAKE, 4, a, FAKE, FAKE, None, None, None, 0, None) == EINVAL
    assert L.ciar_verify(FAKE, FAKE, FAKE, FAKE, None, 4, a, FAKE, FAKE, None, None, None, 0, None) == EINVAL
    assert L.ciar_verify(FAKE, FAKE, FAKE, FAKE, FAKE, 4, a, None, None, None, None, None, 0, None) == EINVAL
    assert L.ciar_verify(FAKE, FAKE, FAKE, FAKE, FAKE, 4, a, FAKE, FAKE, None, None, None, 0, None) == EWORK
    assert L.ciar_verify(FAKE, FAKE, FAKE, FAKE, FAKE, 4, a, None, None, FAKE, FAKE, None, 0, None) == EWORK
    assert L.ciar_verify(FAKE, FAKE, FAKE, FAKE, FAKE, 4, a, None, None, FAKE, FAKE, FAKE, 8, None) == EWORK
    assert L.ciar_verify(FAKE, FAKE, FAKE, FAKE, FAKE, 4, a, None, None, FAKE, FAKE, FAKE + 8, 4096, None) == EALIGN
    assert L.ciar_quantify_verify(FAKE, None, FAKE, FAKE, FAKE, FAKE, 4, a, *([None] * 11), None, 0, None) == EINVAL
    assert L.ciar_dense_intervals(FAKE, None, 4, a, None, None, None, None) == EINVAL
    assert L.ciar_dense_intervals(FAKE, FAKE + 8, 4, a, FAKE, None, None, None) == EALIGN     # radius alignment
    # the stages on their own
    assert L.ciar_stream_rows_timed(FAKE, None, None, None, None, None, 4, a, FAKE, *([None] * 10), FAKE, 4096, None,
                                    None, FAKE) == EINVAL                            # an event is missing
    for stage in (L.ciar_stream_rows, L.ciar_finish_rows):
        assert stage(FAKE, None, None, None, None, None, 4, a, *([None] * 11), FAKE, 4096, None) == EINVAL   # no output
        assert stage(FAKE, None, None, None, None, None, 4, a, FAKE, *([None] * 10), None, 0, None) == EWORK
        assert stage(None, None, None, None, None, None, 4, a, FAKE, *([None] * 10), FAKE, 4096, None) == EINVAL
        assert stage(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, a, *([None] * 7), FAKE, None, None, None, FAKE, 4096,
                     None) == EINVAL                                                 # radius without intervals
        assert stage(FAKE, FAKE + 4, None, None, None, None, 4, a, FAKE, *([None] * 10), FAKE, 4096,
                     None) == EALIGN                                                 # radius alignment
    assert L.ciar_finish_rows(FAKE, None, None, FAKE, FAKE, FAKE, 4, a, *([None] * 7), FAKE, FAKE, None, None,
                              FAKE, 4096, None) == EINVAL                            # verify outputs, no target
    assert L.ciar_finish_rows(FAKE, None, FAKE, FAKE, FAKE, FAKE, 4, a, FAKE, *([None] * 10), FAKE, 4096,
                              None) == EINVAL                                        # target, no verify output
    # Inter-DRO loss
    f4 = [ctypes.c_float(1.0)] * 4
    assert L.ciar_interdro_loss(FAKE, None, FAKE, 4, a, *f4, None, None, None, None) == EINVAL      # no row_terms
    assert L.ciar_interdro_loss(None, None, FAKE, 4, a, *f4, FAKE, None, None, None) == EINVAL
    assert L.ciar_interdro_loss(FAKE, None, None, 4, a, *f4, FAKE, None, None, None) == EINVAL
    assert L.ciar_interdro_loss(FAKE, FAKE + 2, FAKE, 4, a, *f4, FAKE, None, None, None) == EALIGN
    assert L.ciar_interdro_loss(FAKE, None, FAKE, 4, a, ctypes.c_float(float("nan")), *f4[:3], FAKE, None, None,
                                None) == EINVAL
    assert L.ciar_interdro_loss(FAKE, None, FAKE, 0, a, *f4, FAKE, None, None, None) == 0
    # several heads
    def mh(heads=2, hs=4096, strategy=1, out=FAKE, ws=FAKE, wsb=1 << 20, draft=FAKE, radius=None, hf=None):
        return L.ciar_quantify_multihead(draft, radius, heads, hs, None, 4, a, strategy, out, None, None, None,
                                         None, None, None, hf, ws, wsb, None)
    assert mh(heads=0) == EUNSUP and mh(heads=9) == EUNSUP
    assert mh(strategy=2) == EINVAL
    assert mh(hs=100) == EINVAL                      # heads overlap
    assert mh(hs=4097) == EALIGN
    assert mh(draft=None) == EINVAL and mh(radius=FAKE + 4) == EALIGN
    assert mh(out=None) == EINVAL
    assert mh(ws=None, wsb=0) == EWORK and mh(wsb=64) == EWORK
    assert L.ciar_multihead_workspace_bytes(0, 2, a) == 0 and L.ciar_multihead_workspace_bytes(4, 0, a) == 0
    assert L.ciar_multihead_workspace_bytes(2048, 3, a) >= 3 * 77 * 2048
    assert L.ciar_read_rows(FAKE, FAKE, 4, a, None, None) == EINVAL
    assert L.ciar_read_rows(None, FAKE, 4, a, FAKE, None) == EINVAL
    assert L.ciar_read_rows(FAKE, FAKE + 4, 4, a, FAKE, None) == EALIGN
    assert L.ciar_read_rows(FAKE, None, 0, a, FAKE, None) == 0
    assert L.ciar_read_rows_timed(FAKE, None, 4, a, FAKE, None, None, None) == EINVAL
    assert L.ciar_window_epilogue(None, FAKE, 4, a, FAKE, FAKE, None) == EINVAL
    assert L.ciar_window_epilogue(FAKE, None, 4, a, FAKE, FAKE, None) == EINVAL
    assert L.ciar_window_epilogue(FAKE, FAKE, 4, a, None, None, None) == EINVAL


def test_empty_batch_is_ok_and_launches_nothing(L):
    p = _params(L)
    a = ctypes.byref(p)
    assert _quantify(L, p, N=0) == 0
    assert L.ciar_verify(FAKE, FAKE, FAKE, FAKE, FAKE, 0, a, FAKE, FAKE, FAKE, FAKE, None, 0, None) == 0
    assert L.ciar_dense_intervals(FAKE, None, 0, a, FAKE, None, None, None) == 0


def test_workspace_size(L):
    p = _params(L)
    f = L.ciar_workspace_bytes
    assert f(0, ctypes.byref(p)) == 0 and f(-5, ctypes.byref(p)) == 0
    for N in (1, 7, 256, 2048, 32768):
        b = f(N, ctypes.byref(p))
        assert b % 256 == 0 and b >= 113 * N


def test_version_and_error_strings(L):
    from paper_2603_25463_amd import binding
    assert re.fullmatch(r"\d+\.\d+\.\d+", binding.version())
    assert isinstance(binding.last_error(), str)


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2603_25463_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "absent.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.lib()


# ---- host logic: the fitted width polynomial ---------------------------------------------------------

def _width_poly(L, **kw):
    coef = (ctypes.c_float * 4)()
    xmax = ctypes.c_float()
    p = _params(L, **kw)
    assert L.ciar_width_polynomial(ctypes.byref(p), coef, ctypes.byref(xmax)) == 0
    return [float(v) for v in coef], float(xmax.value)


@pytest.mark.parametrize("radius", [1e-3, 0.1, 0.5, 1.0, 1.2816, 1.6449, 1.96, 3.0, 5.0, 8.0])
def test_width_polynomial_matches_the_interval_width(L, radius):
    """The polynomial the kernels use for small probabilities against the InterFuse width itself
    (App. "Proof of Interval Validity": p^u = a x / (1 + (a-1) x), p^l = b x / (1 - (1-b) x)), in 40-digit
    decimal arithmetic: (p^u - p^l) / ((a - b) x) = 1 + x P(x) within 2.5e-8 on (0, x_max], with the float32
    coefficients the kernels receive; and within 1.5e-7 when the polynomial itself is evaluated in float32."""
    import decimal
    import numpy as np
    D = decimal.Decimal
    decimal.getcontext().prec = 40
    coef, xmax = _width_poly(L, radius_scale=radius)
    assert xmax > 0
    r = D(float(np.float32(radius)))
    a, b = r.exp(), (-r).exp()
    worst = worst32 = D(0)
    f32 = np.float32
    for i in range(1, 1501):
        xf = f32(xmax * i / 1500.0)
        x = D(float(xf))
        width = a * x / (1 + (a - 1) * x) - b * x / (1 - (1 - b) * x)
        G = width / ((a - b) * x)
        P = sum(D(c) * x ** j for j, c in enumerate(coef))
        worst = max(worst, abs(1 + x * P - G) / G)
        h = f32(coef[3])
        for c in (coef[2], coef[1], coef[0], 1.0):
            h = f32(f32(h * xf) + f32(c))                            # two roundings per step: an upper bound on the FMA
        worst32 = max(worst32, abs(D(float(h)) - G) / G)
    assert worst <= D("2.5e-8"), worst
    assert worst32 <= D("1.5e-7"), worst32


def test_width_polynomial_range_shrinks_with_the_radius_and_ends(L):
    xs = [_width_poly(L, radius_scale=r)[1] for r in (0.5, 1.0, 2.0, 4.0, 8.0)]
    assert all(x > 0 for x in xs) and all(x1 > x2 for x1, x2 in zip(xs, xs[1:]))
    assert 0.015 < _width_poly(L, confidence=0.9)[1] < 0.025          # the benchmark's radius, kappa(0.9) = 1.645
    assert _width_poly(L, radius_scale=12.0, radius_max=16.0)[1] < 0  # no useful range left: the kernels skip it
    # the clamp is part of the radius
    assert _width_poly(L, radius_scale=50.0, radius_max=1.0) == _width_poly(L, radius_scale=1.0)
    p = _params(L)
    assert L.ciar_width_polynomial(ctypes.byref(p), None, None) == -1    # CIAR_EINVAL


def test_interhead_argument_errors_and_workspace(L):
    """The Interval Head entry points: every argument error returns before any launch; the workspace is the two
    fp32 logit tensors plus the quantifier's."""
    from paper_2603_25463_amd.binding import last_error
    EINVAL, EALIGN, EWORK, EUNSUP = -1, -2, -3, -4
    p = _params(L)                                                  # V = 1024, stride 1024, fp32
    a = ctypes.byref(p)

    def logits(params, D=128, N=4, hidden=FAKE, weight=FAKE + 4096, centre=FAKE + 8192, radius=FAKE + 12288):
        return L.ciar_interhead_logits(hidden, weight, None, D, N, ctypes.byref(params), centre, radius, None)

    def quantify(params, D=128, N=4, out=FAKE + 8192, ws=FAKE + 16384, wsb=1 << 30):
        return L.ciar_interhead_quantify(FAKE, FAKE + 4096, None, D, None, N, ctypes.byref(params), out, None, None, None,
                                         None, None, None, ws, wsb, None)

    assert logits(_params(L, dtype=1)) == EUNSUP and "fp32" in last_error()
    assert logits(p, D=96) == EUNSUP and "hidden_dim" in last_error()
    assert logits(p, D=0) == EUNSUP
    assert logits(_params(L, vocab=1000, row_stride=1000)) == EUNSUP and "multiple of 128" in last_error()
    assert logits(p, N=-1) == EINVAL
    assert logits(p, hidden=None) == EINVAL and "hidden" in last_error()
    assert logits(p, weight=FAKE + 4) == EALIGN
    assert logits(p, centre=None) == EINVAL
    assert logits(p, radius=FAKE + 12292) == EALIGN
    assert logits(p, N=0, hidden=None, weight=None, centre=None, radius=None) == 0     # an empty batch reads nothing
    assert quantify(p, out=None) == EINVAL and "output" in last_error()
    assert quantify(p, ws=None) == EWORK
    assert quantify(p, wsb=1024) == EWORK and "needed" in last_error()
    assert quantify(p, D=100) == EUNSUP
    assert quantify(p, N=0, ws=None, wsb=0) == 0
    f = L.ciar_interhead_workspace_bytes
    assert f(0, a) == 0
    for N in (1, 130, 2048):
        assert f(N, a) == 2 * ((N * 1024 * 4 + 255) // 256 * 256) + L.ciar_workspace_bytes(N, a)
    # the timed form needs both events
    assert L.ciar_interhead_logits_timed(FAKE, FAKE + 4096, None, 128, 4, a, FAKE + 8192, FAKE + 12288, None, None,
                                         None) == EINVAL
