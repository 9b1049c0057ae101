"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on identical bytes.

Every test prints what it is about to run (and flushes) before the first GPU call.
"""
import dataclasses
import math
import os

import numpy as np
import pytest
import torch

import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ciar():
    import paper_2603_25463_amd as m
    m.lib()                      # raises if libciar.so has not been built: no fallback
    assert torch.cuda.is_available()
    return m


def _sweep_seeds(count_var, default):
    """Seeds of a random sweep: `default` of them from 0, or as many as `count_var` says, from CIAR_RANDOM_FIRST on."""
    first = int(os.environ.get("CIAR_RANDOM_FIRST", "0"))
    return [first + k for k in range(int(os.environ.get(count_var, str(default))))]


def say(*a):
    print(*a, flush=True)


def _OP(oracle, **kw):
    """Oracle parameters with every real number rounded to float32 first: the C ABI carries them as floats, and
    the oracle has to see the numbers the library sees (near gamma = 1 the radius scale reacts to the eighth digit
    of the confidence: float32(0.999) moves kappa by 1.1e-6 and a = e^r at r = 14 by 1.5e-5)."""
    o = oracle.Params(**kw)
    return dataclasses.replace(o, **{f.name: float(np.float32(getattr(o, f.name))) for f in dataclasses.fields(o)
                                     if isinstance(getattr(o, f.name), float)})


def _oparams(oracle, p):
    return _OP(oracle, confidence=float(p.confidence), kappa=float(p.radius_scale), radius_max=float(p.radius_max),
               tau=float(p.tau), lower_cap=float(p.lower_cap), upper_cap=float(p.upper_cap),
               normalize=p.normalize, window=p.window)


def _run_case(ciar, oracle, draft, target, ids, ua, ur, P, vocab=None, tag="", host=None, radius=None):
    """Fused, quantify-only and verify-only entry points against the oracle.  Tensors are on the GPU.
    ``radius``: raw radius tensor (tensor-radius mode) or None (scalar radius)."""
    say(f"[case {tag}] N={draft.shape[0]} V={vocab or draft.shape[1]} dtype={draft.dtype} "
        f"K={P.window} conf={P.confidence} kappa={P.radius_scale} tau={P.tau} norm={P.normalize} "
        f"radius={'tensor' if radius is not None else 'scalar'}")
    N = draft.shape[0]
    ws = torch.empty(ciar.workspace_bytes(N, P.to_c(draft, vocab)) or 16, dtype=torch.uint8, device=draft.device)
    fused = ciar.quantify_verify(draft, target, ids, ua, ur, P, vocab=vocab, workspace=ws, radius=radius)
    qonly = ciar.quantify(draft, ids, P, vocab=vocab, workspace=ws, radius=radius)
    vonly = ciar.verify(draft, target, ids, ua, ur, P, vocab=vocab, workspace=ws)
    # the launch configuration the benchmark times: the two stages called one after the other
    ws2 = torch.empty_like(ws)
    staged = ciar.stream_rows(draft, target, ids, ua, ur, P, ws2, with_intervals=True, vocab=vocab, radius=radius)
    staged = ciar.finish_rows(draft, target, ids, ua, ur, P, ws2, with_intervals=True, vocab=vocab, radius=radius,
                              out=staged)
    torch.cuda.synchronize()
    # the entry points run the same arithmetic: floats equal up to the freedom the compiler has in contracting
    # multiply-adds differently in the fused and the single-purpose kernels (seen only where Sigma is rounding
    # noise, ~1e-25); the two stages launch the fused call's own kernels: identical outputs
    for k in parity.FLOAT_KEYS:
        d = (fused[k].double() - qonly[k].double()).abs()
        assert bool((d <= 1e-6 * qonly[k].double().abs() + 1e-12).all()), \
            (k, int(d.argmax()), fused[k][d.argmax()].item(), qonly[k][d.argmax()].item())
    assert torch.equal(fused["flags"], qonly["flags"])
    for k in fused:
        assert torch.equal(fused[k], staged[k]), k

    OP = _oparams(oracle, P)
    dh, th = host if host is not None else (draft.cpu(), target.cpu())
    idh, uah, urh = ids.cpu().numpy(), ua.cpu().numpy(), ur.cpu().numpy()
    oq = oracle.quantify(dh, idh, OP, vocab=vocab, radius=None if radius is None else radius.cpu())
    ov = oracle.verify(dh, th, idh, uah, urh, OP, vocab=vocab)
    worst = parity.check_floats(fused, oq)
    ex_flag = parity.check_flags(fused["flags"], oq, float(np.float32(P.tau)))
    cdf = lambda r: oracle.residual_cdf(dh, th, r, OP, vocab=vocab)
    st = parity.check_verify(fused, ov, uah, urh, P.window, residual_cdf=cdf)
    # The verify-only call runs other kernel instances than the fused call, and not always the same route to a draw
    # (in the streaming kernel from fp32 residuals, or in resample_kernel): it is held to the oracle like the fused
    # call, and to the fused call's decisions row by row wherever the oracle's margin to the decision is not below
    # the exemption's -- a threshold within 1e-7 R of a token boundary may fall to either side in either of them.
    parity.check_verify(vonly, ov, uah, urh, P.window, residual_cdf=cdf)
    with np.errstate(divide="ignore", invalid="ignore"):
        close = np.abs(np.log(uah.astype(np.float64)) - np.minimum(0.0, ov["log_ratio"])) < parity.MARGIN
    close |= (ov["accept"] == 0) & (ov["res_margin"] < parity.MARGIN)
    far = torch.from_numpy(~close).to(fused["accept"].device)
    for k in ("accept", "row_id"):
        assert torch.equal(fused[k][far], vonly[k][far]), k
    K = P.window
    far_w = torch.from_numpy(np.array([not close[w * K:(w + 1) * K].any() for w in range(-(-N // K))], bool)).to(far.device)
    for k in ("accept_len", "resampled_id"):
        assert torch.equal(fused[k][far_w], vonly[k][far_w]), k
    say(f"   worst err/bound {max(worst.values()):.3f}; flagged {int(oq['flags'].sum())}/{N}; "
        f"exempt flag/accept/resample = {ex_flag}/{st['exempt_accept']}/{st['exempt_resample']}; "
        f"rejected {st['rejected']}")
    return oq, ov, ex_flag, st


# ---- the five workloads, full size, every row -------------------------------------------------------

@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_workload_full_size(ciar, oracle, cfg):
    from paper_2603_25463_amd import workloads as wl
    say(f"[workload {cfg}] generating on the GPU")
    w = wl.make(cfg, device="cuda")
    spec = w.spec
    N = w.rows
    host = (w.draft.cpu(), w.target.cpu())
    for gi, gamma in enumerate(spec.confidences):
        # tau = 0.30 is the paper's value (nothing is flagged on these synthetic rows: U ~ 1e-2);
        # tau* = the oracle's median U splits the rows ~50/50 and exercises the margin rule.
        P = ciar.Params(confidence=gamma, tau=0.30, window=spec.window)
        if gi == 0:
            oq, ov, exf, st = _run_case(ciar, oracle, w.draft, w.target, w.ids, w.u_accept, w.u_resample, P,
                                        tag=f"cfg{cfg} tau=0.30", host=host)
            assert int(oq["flags"].sum()) == 0
            assert st["exempt_accept"] <= 2 and st["exempt_resample"] <= max(4, 0.3 * st["rejected"])
            acc = float(ov["accept"].mean())
            say(f"   acceptance rate {acc:.3f}")
            if cfg == 4:
                # identical rows always accept; only redrawn rows can reject
                same = ~w.meta["redraw"]
                assert ov["accept"][same].all()
            else:
                expect = 2 * 0.5 * math.erfc(spec.sigma / 2 / math.sqrt(2))     # 2 Phi(-sigma/2)
                assert abs(acc - expect) < 0.06
        else:
            oq = oracle.quantify(host[0], w.ids.cpu().numpy(), _oparams(oracle, P))
        tau_star = float(np.float32(np.median(oq["score"])))
        P2 = ciar.Params(confidence=gamma, tau=tau_star, window=spec.window)
        say(f"[workload {cfg}] gamma={gamma} tau*={tau_star:.6g}")
        g = ciar.quantify(w.draft, w.ids, P2)
        torch.cuda.synchronize()
        oq2 = dict(oq)
        oq2["flags"] = (oq["score"] > float(np.float32(tau_star))).astype(np.uint8)
        parity.check_floats(g, oq2)
        ex = parity.check_flags(g["flags"], oq2, float(np.float32(tau_star)))
        frac = float(oq2["flags"].mean())
        say(f"   flagged fraction {frac:.3f}, exempt {ex}")
        assert 0.4 < frac < 0.6 and ex <= 3


def test_nested_intervals_across_confidences_on_the_gpu(ciar):
    """Raw InterFuse on the large-vocabulary workload: the drafted token's interval widens with gamma
    and Omega grows (a property that holds at any size; checked on the GPU outputs themselves)."""
    from paper_2603_25463_amd import workloads as wl
    say("[nested] cfg5 first 2048 rows, normalize=0, gamma in 0.8/0.9/0.95")
    w = wl.make(5, device="cuda", rows=2048)
    prev = None
    for gamma in (0.8, 0.9, 0.95):
        g = ciar.quantify(w.draft, w.ids, ciar.Params(confidence=gamma, normalize=False, window=8))
        torch.cuda.synchronize()
        if prev is not None:
            assert torch.all(g["p_lo"] <= prev["p_lo"]) and torch.all(g["p_hi"] >= prev["p_hi"])
            assert torch.all(g["omega"] > prev["omega"])
            assert torch.equal(g["p_mid"], prev["p_mid"])
        prev = g


# ---- shapes: every tile configuration, ragged vocabularies, strides, ragged last window ---------------

SHAPES = [
    # (V, stride, N, K, dtype)
    (2, 4, 37, 4, torch.float32),
    (5, 8, 19, 3, torch.float32),
    (1000, 1000, 65, 8, torch.float32),
    (1023, 1024, 33, 5, torch.float32),
    (1024, 1024, 64, 8, torch.float32),
    (1025, 1028, 31, 8, torch.float32),
    (3000, 3000, 40, 7, torch.float32),
    (4096, 4100, 40, 8, torch.float32),
    (8191, 8192, 21, 8, torch.float32),
    (8192, 8192, 48, 16, torch.float32),
    (12345, 12348, 35, 8, torch.float32),
    (16384, 16384, 70, 8, torch.float32),
    (16385, 16388, 9, 4, torch.float32),
    (32768, 32768, 12, 4, torch.float32),
    (3, 8, 37, 4, torch.bfloat16),
    (1001, 1008, 65, 8, torch.bfloat16),
    (2048, 2048, 64, 8, torch.bfloat16),
    (5000, 5000, 40, 6, torch.bfloat16),
    (8192, 8192, 40, 8, torch.bfloat16),
    (16383, 16384, 33, 8, torch.bfloat16),
    (16384, 16384, 64, 8, torch.bfloat16),
    (20000, 20000, 17, 8, torch.bfloat16),
    (32768, 32776, 20, 8, torch.bfloat16),
    (65535, 65536, 9, 4, torch.bfloat16),
    (65536, 65536, 16, 8, torch.bfloat16),
]


def _random_case(V, stride, N, K, dtype, seed, sigma=0.5):
    g = torch.Generator(device="cuda").manual_seed(seed)
    scale = torch.rand((N, 1), generator=g, device="cuda") * 2.5 + 0.5
    c = torch.randn((N, stride), generator=g, device="cuda") * scale
    peak = torch.randint(0, V, (N,), generator=g, device="cuda")
    c[torch.arange(N, device="cuda")[::2], peak[::2]] += 8.0
    t = c + sigma * torch.randn((N, stride), generator=g, device="cuda")
    # poison the padding: it must never be read as a token
    if stride > V:
        c[:, V:] = 1e30
        t[:, V:] = -1e30
    c, t = c.to(dtype), t.to(dtype)
    gum = -torch.log(-torch.log(torch.rand((N, V), generator=g, device="cuda").clamp_(1e-30, 1 - 1e-7)))
    ids = torch.argmax(c[:, :V].float() + gum, dim=1).to(torch.int32)
    ua = torch.randint(0, 1 << 24, (N,), generator=g, device="cuda").float() / (1 << 24)
    ur = torch.randint(0, 1 << 24, (N,), generator=g, device="cuda").float() / (1 << 24)
    return c, t, ids, ua, ur


@pytest.mark.parametrize("V,stride,N,K,dtype", SHAPES)
def test_shapes_and_ragged_tails(ciar, oracle, V, stride, N, K, dtype):
    c, t, ids, ua, ur = _random_case(V, stride, N, K, dtype, seed=1000 + V)
    for norm, kap in ((True, -1.0), (False, 0.7)):
        P = ciar.Params(confidence=0.9, radius_scale=kap, normalize=norm, window=K, tau=0.01)
        _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=V, tag=f"V={V} stride={stride}")


# ---- tensor-radius mode: r_i = min(kappa Softplus(raw_i), r_max)  (Sec. 3.2.3, Interval Head) ----------------

def _raw_radius(N, stride, V, dtype, seed, mu_lo=-1.0, mu_hi=1.0, sd=1.0):
    g = torch.Generator(device="cuda").manual_seed(seed)
    mu = torch.rand((N, 1), generator=g, device="cuda") * (mu_hi - mu_lo) + mu_lo
    raw = torch.randn((N, stride), generator=g, device="cuda") * sd + mu
    if stride > V:
        raw[:, V:] = float("nan")          # poison the padding: it must never reach a result
    return raw.to(dtype)


RADIUS_SHAPES = [
    (2, 4, 37, 4, torch.float32), (5, 8, 19, 3, torch.float32), (1023, 1024, 33, 5, torch.float32),
    (3000, 3000, 40, 7, torch.float32), (8192, 8192, 48, 16, torch.float32), (12345, 12348, 35, 8, torch.float32),
    (16384, 16384, 70, 8, torch.float32), (32768, 32768, 12, 4, torch.float32),
    (3, 8, 37, 4, torch.bfloat16), (1001, 1008, 65, 8, torch.bfloat16), (5000, 5000, 40, 6, torch.bfloat16),
    (16384, 16384, 64, 8, torch.bfloat16), (20000, 20000, 17, 8, torch.bfloat16), (65535, 65536, 9, 4, torch.bfloat16),
]


@pytest.mark.parametrize("V,stride,N,K,dtype", RADIUS_SHAPES)
def test_tensor_radius_shapes(ciar, oracle, V, stride, N, K, dtype):
    c, t, ids, ua, ur = _random_case(V, stride, N, K, dtype, seed=2000 + V)
    raw = _raw_radius(N, stride, V, dtype, seed=3000 + V)
    for norm, kap in ((True, 1.0), (False, 0.6)):
        P = ciar.Params(radius_scale=kap, normalize=norm, window=K, tau=0.01)
        _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=V, tag=f"tensor radius V={V} stride={stride}",
                  radius=raw)


def test_tensor_radius_extremes_and_clamp(ciar, oracle):
    """Raw radii from -60 (radius ~ 1e-26) to +60 (clamped), a small clamp, rows of constant raw radius (which
    must reproduce the scalar mode bit for bit in the flags and to tolerance in the floats)."""
    V, N, K = 4096, 24, 4
    c, t, ids, ua, ur = _random_case(V, V, N, K, torch.float32, seed=61)
    raw = _raw_radius(N, V, V, torch.float32, seed=62, mu_lo=-3.0, mu_hi=3.0, sd=8.0)
    raw[0] = -60.0
    raw[1] = 60.0
    raw[2, ::2] = -30.0
    for rmax in (10.0, 1.5):
        P = ciar.Params(radius_scale=1.0, radius_max=rmax, window=K, tau=0.01)
        _run_case(ciar, oracle, c, t, ids, ua, ur, P, tag=f"tensor radius extremes rmax={rmax}", radius=raw)
    const = torch.full_like(c, 0.75)
    kap = 1.3
    r = kap * math.log1p(math.exp(0.75))
    say("[tensor radius] constant raw radius against the scalar mode")
    a = ciar.quantify(c, ids, ciar.Params(radius_scale=kap, tau=0.01), radius=const)
    b = ciar.quantify(c, ids, ciar.Params(radius_scale=r, tau=0.01))
    torch.cuda.synchronize()
    for k in parity.FLOAT_KEYS:
        assert torch.allclose(a[k], b[k], rtol=2e-5, atol=1e-7), k


def test_tensor_radius_argmax_token_and_dense(ciar, oracle):
    """Without drafted ids the reported token is the lowest-index arg-max and its own radius applies; the dense
    curves match the oracle's."""
    for V, dtype in ((1000, torch.float32), (16384, torch.bfloat16)):
        c, *_ = _random_case(V, V, 9, 4, dtype, seed=71)
        c[3, 5] = c[3].max() + 1
        c[3, 400] = c[3, 5]                                           # a tie: the lower index wins
        raw = _raw_radius(9, V, V, dtype, seed=72)
        say(f"[tensor radius] arg-max report and dense export V={V} {dtype}")
        P = ciar.Params(radius_scale=1.0)
        g = ciar.quantify(c, None, P, radius=raw)
        lo, mid, hi = ciar.dense_intervals(c, P, radius=raw)
        torch.cuda.synchronize()
        OP = _OP(oracle, kappa=1.0)
        o = oracle.quantify(c.cpu(), None, OP, radius=raw.cpu())
        parity.check_floats(g, o)
        olo, omid, ohi = oracle.dense_intervals(c.cpu(), OP, radius=raw.cpu())
        for gg, oo in ((lo, olo), (mid, omid), (hi, ohi)):
            gg = gg.cpu().numpy().astype(np.float64)
            assert np.all(np.abs(gg - oo) <= parity.ATOL + parity.RTOL * np.abs(oo))


# ---- flat rows with wide intervals: widths that agree to 1e-6 while Omega ~ V multiplies their spread ----------------

def _flat_rows(V, stride, N, dtype, seed):
    """Rows that are flat in the centre logits (largest probability <= 2 / V) with raw radii around ln(4 V) (e^r ~ 4 V:
    every width ~ 0.8) in the variants that leave the least spread: constant centre row with a constant, a nearly
    constant (noise 1e-6 ... 1e-3) or a slowly varying radius; centre rows flat to 1e-6 / 1e-4 / 1e-2 with the same
    radii; a row of smaller radii (e^r ~ V / 4)."""
    g = torch.Generator(device="cuda").manual_seed(seed)
    c = torch.empty((N, stride), device="cuda")
    raw = torch.empty((N, stride), device="cuda")
    tok = torch.arange(stride, device="cuda", dtype=torch.float32)
    centre = math.log(4.0 * V)
    for r in range(N):
        cs = (0.0, 0.0, 0.0, 1e-6, 1e-4, 1e-2)[r % 6]
        rs = (0.0, 1e-6, 1e-5, 1e-4, 1e-3)[(r // 6) % 5]
        slow = (r // 30) % 2 == 1
        rc = centre if (r // 60) % 2 == 0 else math.log(0.25 * V)
        c[r] = 1.5 + cs * torch.randn(stride, generator=g, device="cuda")
        if slow:
            raw[r] = rc + rs * torch.sin(tok * (2 * math.pi / V))
        else:
            raw[r] = rc + rs * torch.randn(stride, generator=g, device="cuda")
    t = c + 0.3 * torch.randn((N, stride), generator=g, device="cuda")
    if stride > V:
        c[:, V:] = 1e30
        t[:, V:] = -1e30
        raw[:, V:] = float("nan")
    ids = torch.randint(0, V, (N,), generator=g, device="cuda").to(torch.int32)
    ua = torch.randint(0, 1 << 24, (N,), generator=g, device="cuda").float() / (1 << 24)
    ur = torch.randint(0, 1 << 24, (N,), generator=g, device="cuda").float() / (1 << 24)
    return c.to(dtype), t.to(dtype), raw.to(dtype), ids, ua, ur


FLAT_SHAPES = [   # every tile of the streaming kernel, both dtypes, ragged vocabularies and padded strides
    (1000, 1000, 120, torch.float32), (2048, 2048, 60, torch.float32), (4000, 4000, 60, torch.float32),
    (8192, 8192, 120, torch.float32), (16384, 16384, 120, torch.float32), (12345, 12348, 3100, torch.float32),
    (32768, 32768, 36, torch.float32),
    (2000, 2000, 60, torch.bfloat16), (4096, 4096, 60, torch.bfloat16), (8192, 8192, 60, torch.bfloat16),
    (16384, 16384, 120, torch.bfloat16), (30000, 30000, 36, torch.bfloat16), (65535, 65536, 36, torch.bfloat16),
]


@pytest.mark.parametrize("V,stride,N,dtype", FLAT_SHAPES)
def test_flat_rows_with_wide_intervals(ciar, oracle, V, stride, N, dtype):
    """The regime in which fp32 token arithmetic cannot hold the score's tolerance: all widths of a row O(1) and
    equal to 1e-6 and better, so that U = Omega * Sigma with Omega ~ 0.8 V needs Sigma to ~1e-11.  The library redoes
    such rows in fp64 (flatrow_kernel); fused, quantify-only, verify-only and staged calls, tensor and scalar radius."""
    c, t, raw, ids, ua, ur = _flat_rows(V, stride, N, dtype, seed=7000 + V)
    for rmax in (16.0, 10.0):
        P = ciar.Params(radius_scale=1.0, radius_max=rmax, window=8, tau=1e-3)
        _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=V, tag=f"flat rows, tensor radius, V={V} rmax={rmax}",
                  radius=raw)
    # the same centre rows under a scalar radius of that size
    P = ciar.Params(radius_scale=math.log(4.0 * V), radius_max=16.0, window=8, tau=1e-3)
    _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=V, tag=f"flat rows, scalar radius ln(4V), V={V}")
    P = ciar.Params(radius_scale=math.log(0.25 * V), radius_max=16.0, window=8, tau=1e-3)
    _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=V, tag=f"flat rows, scalar radius ln(V/4), V={V}")


def test_flat_rows_take_the_fp64_pass(ciar):
    """White box: the streaming kernel marks the flat rows of such a call and flatrow_kernel rewrites their
    statistics (RowStats::mode, the float at byte 84 of each 88-byte record at the start of the workspace, reads 3);
    rows that are not flat, and calls whose widths are small, keep the streaming kernel's sums (mode 0 ... 2)."""
    V, N = 4096, 60
    c, t, raw, ids, ua, ur = _flat_rows(V, V, N, torch.float32, seed=11)
    c[1] = torch.randn(V, device="cuda") * 2.0                     # an ordinary row among them
    P = ciar.Params(radius_scale=1.0, radius_max=10.0, window=8, tau=1e-3)
    ws = torch.zeros(ciar.workspace_bytes(N, P.to_c(c)), dtype=torch.uint8, device="cuda")
    say("[flat rows] RowStats::mode after a tensor-radius call and after a default scalar call")
    ciar.quantify(c, ids, P, workspace=ws, radius=raw)
    torch.cuda.synchronize()
    mode = ws[:N * 88].view(N, 88)[:, 84:88].contiguous().view(torch.float32).flatten().cpu()
    assert mode[1] < 3.0 and bool((mode[torch.arange(N) != 1] == 3.0).all()), mode
    ciar.quantify(c, ids, ciar.Params(confidence=0.9, tau=1e-3), workspace=ws)
    torch.cuda.synchronize()
    mode = ws[:N * 88].view(N, 88)[:, 84:88].contiguous().view(torch.float32).flatten().cpu()
    assert bool((mode < 3.0).all()), mode


@pytest.mark.parametrize("V,dtype", [(1000, torch.float32), (16384, torch.float32), (16384, torch.bfloat16)])
def test_flat_rows_with_wide_intervals_ensemble(ciar, oracle, V, dtype):
    """The same regime through the Ensemble sweep (rows flat in every head take its fp64 branch) and Voting."""
    H, N = 3, 60
    heads = [_flat_rows(V, V, N, dtype, seed=7100 + V + h) for h in range(H)]
    c = torch.stack([x[0] for x in heads])
    raw = torch.stack([x[2] for x in heads])
    ids = heads[0][3]
    for rad in (raw, None):
        P = ciar.Params(radius_scale=1.0 if rad is not None else math.log(4.0 * V), radius_max=16.0, tau=1e-3)
        OP = _oparams(oracle, P)
        for strat, ostrat in ((ciar.ENSEMBLE, oracle.ENSEMBLE), (ciar.VOTING, oracle.VOTING)):
            say(f"[flat rows, heads] V={V} {dtype} strategy={strat} radius={'tensor' if rad is not None else 'scalar'}")
            g = ciar.quantify_multihead(c, ids, P, strat, radius_heads=rad)
            torch.cuda.synchronize()
            o = oracle.quantify_multihead(c.cpu(), ids.cpu().numpy(), OP, ostrat,
                                          radius_heads=None if rad is None else rad.cpu())
            if strat == ciar.VOTING:
                o2 = {k: o[k].reshape(-1) for k in parity.FLOAT_KEYS}
                parity.check_floats({k: g[k].reshape(-1) for k in parity.FLOAT_KEYS}, o2)
            else:
                parity.check_floats(g, o)


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_tensor_radius_workloads(ciar, oracle, cfg):
    """Workloads 1-3 at full size with the synthetic radius head (raw ~ N(mu_row, 1), kappa = 1), at tau = 0.30
    and at the oracle's median U."""
    from paper_2603_25463_amd import workloads as wl
    say(f"[tensor radius workload {cfg}] generating on the GPU")
    w = wl.make(cfg, device="cuda")
    raw = wl.make_radius(w)
    P = ciar.Params(radius_scale=1.0, tau=0.30, window=w.spec.window)
    oq, ov, exf, st = _run_case(ciar, oracle, w.draft, w.target, w.ids, w.u_accept, w.u_resample, P,
                                tag=f"cfg{cfg} tensor radius", radius=raw)
    tau_star = float(np.float32(np.median(oq["score"])))
    g = ciar.quantify(w.draft, w.ids, ciar.Params(radius_scale=1.0, tau=tau_star, window=w.spec.window), radius=raw)
    torch.cuda.synchronize()
    oq2 = dict(oq)
    oq2["flags"] = (oq["score"] > float(np.float32(tau_star))).astype(np.uint8)
    parity.check_floats(g, oq2)
    ex = parity.check_flags(g["flags"], oq2, float(np.float32(tau_star)))
    frac = float(oq2["flags"].mean())
    say(f"   tau*={tau_star:.6g} flagged fraction {frac:.3f}, exempt {ex}")
    assert 0.4 < frac < 0.6 and ex <= 3


# ---- several heads: Voting and Ensemble (Sec. 4, ablation on the Inter-Head) ---------------------------------

def _head_stack(H, V, stride, N, dtype, seed):
    """H heads that agree on the gist of every row and differ in detail: one shared row plus per-head noise."""
    c, *_ = _random_case(V, stride, N, 4, torch.float32, seed=seed)
    g = torch.Generator(device="cuda").manual_seed(seed + 1)
    heads = torch.stack([c + 0.4 * torch.randn((N, stride), generator=g, device="cuda") for _ in range(H)])
    if stride > V:
        heads[:, :, V:] = 1e30
    return heads.to(dtype).contiguous()


MULTIHEAD_CASES = [
    (2, 2, 4, 21, torch.float32), (3, 1000, 1000, 33, torch.float32), (3, 16384, 16384, 40, torch.float32),
    (5, 4099, 4100, 17, torch.float32), (2, 16385, 16388, 9, torch.float32), (8, 777, 780, 12, torch.float32),
    (3, 1001, 1008, 30, torch.bfloat16), (2, 65536, 65536, 6, torch.bfloat16), (1, 512, 512, 20, torch.float32),
]


@pytest.mark.parametrize("H,V,stride,N,dtype", MULTIHEAD_CASES)
@pytest.mark.parametrize("tensor_radius", [False, True])
def test_multihead_ensemble_and_voting(ciar, oracle, H, V, stride, N, dtype, tensor_radius):
    heads = _head_stack(H, V, stride, N, dtype, seed=4000 + V + H)
    raw = None
    if tensor_radius:
        raw = torch.stack([_raw_radius(N, stride, V, dtype, seed=5000 + V + h) for h in range(H)]).contiguous()
    g = torch.Generator(device="cuda").manual_seed(9)
    ids = torch.randint(0, V, (N,), generator=g, device="cuda").to(torch.int32)
    say(f"[multihead] H={H} V={V} stride={stride} N={N} {dtype} radius={'tensor' if tensor_radius else 'scalar'}")
    kw = dict(radius_scale=1.0) if tensor_radius else dict(confidence=0.9)
    okw = dict(kappa=1.0) if tensor_radius else dict(confidence=0.9)
    hh, rh = heads.cpu(), None if raw is None else raw.cpu()
    # a threshold in the middle of the scores so that flags and votes go both ways
    o0 = oracle.quantify_multihead(hh, ids.cpu().numpy(), _OP(oracle, **okw), oracle.ENSEMBLE, vocab=V,
                                   radius_heads=rh)
    tau = float(np.float32(np.median(o0["score"])))
    P, OP = ciar.Params(tau=tau, **kw), _OP(oracle, tau=tau, **okw)
    for with_ids in (True, False):
        i_gpu = ids if with_ids else None
        i_cpu = ids.cpu().numpy() if with_ids else None
        ge = ciar.quantify_multihead(heads, i_gpu, P, ciar.ENSEMBLE, vocab=V, radius_heads=raw)
        gv = ciar.quantify_multihead(heads, i_gpu, P, ciar.VOTING, vocab=V, radius_heads=raw)
        torch.cuda.synchronize()
        oe = oracle.quantify_multihead(hh, i_cpu, OP, oracle.ENSEMBLE, vocab=V, radius_heads=rh)
        ov = oracle.quantify_multihead(hh, i_cpu, OP, oracle.VOTING, vocab=V, radius_heads=rh)
        parity.check_floats(ge, oe)
        parity.check_flags(ge["flags"], oe, float(np.float32(tau)))
        # voting: every head against the oracle's head, the vote recomputed from the GPU's own head flags, and
        # the vote against the oracle's wherever no head sits inside the threshold margin
        near = np.zeros(N, dtype=bool)
        for h in range(H):
            gh = {k: gv[k][h] for k in parity.FLOAT_KEYS}
            oh = {k: ov[k][h] for k in parity.FLOAT_KEYS}
            oh["flags"] = ov["head_flags"][h]
            parity.check_floats(gh, oh)
            parity.check_flags(gv["head_flags"][h], oh, float(np.float32(tau)))
            near |= np.abs(ov["score"][h] - float(np.float32(tau))) < parity.MARGIN
        votes = gv["head_flags"].sum(0, dtype=torch.int32)
        assert torch.equal(gv["flags"], (2 * votes > H).to(torch.uint8))
        same = gv["flags"].cpu().numpy() == ov["flags"]
        assert np.all(same | near)


ONE_SWEEP_CASES = [  # H, V, stride, N, dtype: every tile of the one-sweep Ensemble kernel, ragged vocabularies, N above its grid
    (1, 4097, 4100, 40, torch.float32), (2, 8192, 8192, 70, torch.float32), (3, 8200, 8200, 33, torch.float32),
    (2, 16384, 16384, 1100, torch.float32), (3, 16381, 16384, 25, torch.float32), (3, 130, 132, 700, torch.float32),
    (3, 16384, 16384, 30, torch.bfloat16), (2, 9000, 9000, 30, torch.bfloat16), (1, 16384, 16384, 600, torch.bfloat16),
    (3, 4099, 4104, 41, torch.bfloat16),
]


@pytest.mark.parametrize("H,V,stride,N,dtype", ONE_SWEEP_CASES)
def test_ensemble_one_sweep_special_rows(ciar, oracle, H, V, stride, N, dtype):
    """The one-sweep Ensemble kernel (a few heads, scalar radius) on the rows its branches are for: nearly one-hot
    rows in one head or in all (active caps, probabilities above 1/2), rows with masked tokens, ordinary rows whose
    tokens are all small (the width polynomial) next to peaked ones, with and without drafted ids, three radii."""
    heads = _head_stack(H, V, stride, N, torch.float32, seed=7000 + V + H)
    g = torch.Generator(device="cuda").manual_seed(11)
    rows = torch.arange(N, device="cuda")
    tok = torch.randint(0, V, (N,), generator=g, device="cuda")
    heads[0, rows[1::5], tok[1::5]] += 25.0                 # one head nearly one-hot
    heads[:, rows[2::5], tok[2::5]] += 30.0                 # every head nearly one-hot, the same token
    heads[H - 1, rows[3::5], tok[3::5]] += 12.0             # a strong peak in the last head only
    heads[:, rows[4::10], : max(1, V // 3)] = float("-inf")  # masked tokens
    if stride > V:
        heads[:, :, V:] = 1e30
    heads = heads.to(dtype).contiguous()
    ids = torch.randint(0, V, (N,), generator=g, device="cuda").to(torch.int32)
    ids[2::5] = tok[2::5].to(torch.int32)                    # the reported token is the dominant one there
    hh = heads.cpu()
    for kw in (dict(confidence=0.9), dict(radius_scale=0.3), dict(radius_scale=2.5, normalize=False)):
        say(f"[one-sweep ensemble] H={H} V={V} stride={stride} N={N} {dtype} {kw}")
        o0 = oracle.quantify_multihead(hh, ids.cpu().numpy(), _oparams(oracle, ciar.Params(**kw)), oracle.ENSEMBLE, vocab=V)
        tau = float(np.float32(np.median(o0["score"])))
        P = ciar.Params(tau=tau, **kw)
        OP = _oparams(oracle, P)
        for with_ids in (True, False):
            ge = ciar.quantify_multihead(heads, ids if with_ids else None, P, ciar.ENSEMBLE, vocab=V)
            torch.cuda.synchronize()
            oe = oracle.quantify_multihead(hh, ids.cpu().numpy() if with_ids else None, OP, oracle.ENSEMBLE, vocab=V)
            parity.check_floats(ge, oe)
            parity.check_flags(ge["flags"], oe, float(np.float32(tau)))


# ---- Inter-DRO loss, forward (Sec. 3.2.3) -------------------------------------------------------------------

def _check_dro(g, o, N):
    """Per-row terms, batch weights and the five scalars against the oracle: 1e-5 relative, 1e-7 absolute
    (the weights sum to one, so their absolute floor is scaled by 1/N)."""
    terms = g["terms"].cpu().numpy().astype(np.float64)
    for i, k in enumerate(("l1_mid", "l1_up", "l1_lo", "ce_mid", "ce_up", "ce_lo", "kl")):
        assert np.all(np.isfinite(terms[i])), k
        err = np.abs(terms[i] - o[k])
        bound = parity.ATOL + parity.RTOL * np.abs(o[k])
        assert np.all(err <= bound), (k, int(np.argmax(err / bound)), float(np.max(err / bound)))
    w = g["weights"].cpu().numpy().astype(np.float64)
    # a weight is exp(alpha CE): an error of 1e-5 relative in CE of ~10 with alpha ~2 moves it by ~2e-4 relative
    assert np.all(np.abs(w - o["weights"]) <= parity.ATOL / max(N, 1) + 5e-4 * o["weights"])
    assert abs(w.sum() - 1.0) < 1e-5
    L = g["losses"].cpu().numpy().astype(np.float64)
    for i, k in enumerate(("center", "upper", "lower", "dro", "total")):
        assert abs(L[i] - o[k]) <= parity.ATOL + parity.RTOL * abs(o[k]), (k, L[i], o[k])


DRO_SHAPES = [
    (2, 4, 21, torch.float32), (193, 196, 33, torch.float32), (4096, 4096, 40, torch.float32),
    (4100, 4100, 9, torch.float32), (16384, 16384, 64, torch.float32), (16385, 16388, 5, torch.float32),
    (32768, 32768, 6, torch.float32), (1001, 1008, 30, torch.bfloat16), (16384, 16384, 40, torch.bfloat16),
    (65536, 65536, 6, torch.bfloat16),
]


@pytest.mark.parametrize("V,stride,N,dtype", DRO_SHAPES)
@pytest.mark.parametrize("tensor_radius", [True, False])
def test_interdro_loss(ciar, oracle, V, stride, N, dtype, tensor_radius):
    c, t, *_ = _random_case(V, stride, N, 4, dtype, seed=6000 + V)
    if stride > V:                                                   # _random_case poisons target padding with -1e30
        t[:, V:] = 1e30
    raw = _raw_radius(N, stride, V, dtype, seed=6100 + V) if tensor_radius else None
    if V > 8:
        t[0, 3] = float("-inf")                                      # a token the cloud rules out
    say(f"[interdro] V={V} stride={stride} N={N} {dtype} radius={'tensor' if tensor_radius else 'scalar'}")
    lam = (0.7, 1.3, 0.4, 2.0)
    P = ciar.Params(radius_scale=1.0 if tensor_radius else 0.8)
    g = ciar.interdro_loss(c, raw, t, P, *lam, vocab=V)
    torch.cuda.synchronize()
    o = oracle.interdro_loss(c.cpu(), None if raw is None else raw.cpu(), t.cpu(),
                             _OP(oracle, kappa=P.radius_scale), *lam, vocab=V)
    _check_dro(g, o, N)


# More rows than the chip has compute units: the loss then runs in its persistent row kernel (rows strided over the
# workgroups, the next row fetched while one is summed).  N = 16700 is above 64 rows per workgroup on 256 units, where
# the grid grows instead; 257 leaves all but one workgroup a single row; the vocabularies cover each vector count, a
# ragged tail and padded strides.
DRO_MANY_ROWS = [
    (70, 72, 16700, torch.float32), (1000, 1000, 257, torch.float32), (4100, 4104, 300, torch.float32),
    (8192, 8192, 513, torch.float32), (16381, 16384, 290, torch.float32), (520, 520, 3000, torch.bfloat16),
    (8200, 8200, 300, torch.bfloat16), (16384, 16384, 261, torch.bfloat16), (32768, 32768, 259, torch.bfloat16),
]


@pytest.mark.parametrize("V,stride,N,dtype", DRO_MANY_ROWS)
@pytest.mark.parametrize("tensor_radius", [True, False])
def test_interdro_loss_many_rows(ciar, oracle, V, stride, N, dtype, tensor_radius):
    c, t, *_ = _random_case(V, stride, N, 4, dtype, seed=6500 + V)
    if stride > V:
        t[:, V:] = 1e30
    raw = _raw_radius(N, stride, V, dtype, seed=6600 + V) if tensor_radius else None
    gen = torch.Generator(device="cpu").manual_seed(6700 + V)
    rows = torch.randint(0, N, (7,), generator=gen)
    cols = torch.randint(0, V, (7,), generator=gen)
    t[rows.cuda(), cols.cuda()] = float("-inf")                      # tokens the cloud rules out, in scattered rows
    t[N - 1, V - 1] = float("-inf")
    say(f"[interdro many rows] V={V} stride={stride} N={N} {dtype} radius={'tensor' if tensor_radius else 'scalar'}")
    lam = (0.9, 0.6, 1.1, 1.5)
    P = ciar.Params(radius_scale=1.0 if tensor_radius else 0.6)
    g = ciar.interdro_loss(c, raw, t, P, *lam, vocab=V)
    torch.cuda.synchronize()
    o = oracle.interdro_loss(c.cpu(), None if raw is None else raw.cpu(), t.cpu(),
                             _OP(oracle, kappa=P.radius_scale), *lam, vocab=V)
    _check_dro(g, o, N)


@pytest.mark.parametrize("V,N,dtype", [(1000, 40, torch.float32), (4100, 300, torch.float32), (16384, 270, torch.float32),
                                       (16384, 300, torch.bfloat16), (40000, 7, torch.bfloat16)])
def test_interdro_tokens_the_device_rules_out(ciar, oracle, V, N, dtype):
    """Centre logits of -inf.  Where the cloud rules the same tokens out the terms stay finite and match; a row in which
    the cloud keeps such a token has infinite cross-entropies and KL (its L1 distances stay finite)."""
    c, t, *_ = _random_case(V, V, N, 4, dtype, seed=6900 + V)
    raw = _raw_radius(N, V, V, dtype, seed=6950 + V)
    gen = torch.Generator(device="cpu").manual_seed(6990 + V)
    dead = torch.randint(0, V, (N, 9), generator=gen).cuda()
    rows = torch.arange(N, device="cuda")[:, None]
    c[rows, dead] = float("-inf")
    t[rows, dead] = float("-inf")
    c[:, V - 3:] = float("-inf")                                     # a masked tail, as a padded vocabulary has
    t[:, V - 3:] = float("-inf")
    infinite = torch.arange(N) % 5 == 2
    t[infinite.cuda(), dead[infinite.cuda(), 0]] = 0.5               # the cloud keeps one of them
    say(f"[interdro ruled out] V={V} N={N} {dtype}")
    lam = (1.0, 1.0, 1.0, 1.0)
    P = ciar.Params(radius_scale=1.0)
    g = ciar.interdro_loss(c, raw, t, P, *lam, vocab=V)
    torch.cuda.synchronize()
    o = oracle.interdro_loss(c.cpu(), raw.cpu(), t.cpu(), _OP(oracle, kappa=1.0), *lam, vocab=V)
    terms = g["terms"].cpu().numpy().astype(np.float64)
    inf = infinite.numpy()
    for i, k in enumerate(("l1_mid", "l1_up", "l1_lo", "ce_mid", "ce_up", "ce_lo", "kl")):
        ok = np.ones(N, bool) if i < 3 else ~inf
        assert np.all(np.isfinite(o[k][ok])) and np.all(np.isfinite(terms[i][ok])), k
        err = np.abs(terms[i][ok] - o[k][ok])
        assert np.all(err <= parity.ATOL + parity.RTOL * np.abs(o[k][ok])), (k, float(err.max()))
        if i >= 3:
            assert np.all(np.isposinf(o[k][inf])) and np.all(np.isposinf(terms[i][inf])), k


def test_interdro_loss_on_a_workload(ciar, oracle):
    """The benchmark workload's rows as (centre, cloud) pairs with the synthetic radius head, every row."""
    from paper_2603_25463_amd import workloads as wl
    say("[interdro] workload 2, full size")
    w = wl.make(2, device="cuda")
    raw = wl.make_radius(w)
    lam = (1.0, 1.0, 0.5, 1.0)
    g = ciar.interdro_loss(w.draft, raw, w.target, ciar.Params(radius_scale=1.0), *lam)
    torch.cuda.synchronize()
    o = oracle.interdro_loss(w.draft.cpu(), raw.cpu(), w.target.cpu(), _OP(oracle, kappa=1.0), *lam)
    _check_dro(g, o, w.rows)
    say(f"   total loss {o['total']:.6f} (centre {o['center']:.4f}, upper {o['upper']:.4f}, lower {o['lower']:.4f}, "
        f"DRO {o['dro']:.4f})")


@pytest.mark.parametrize("K", [1, 3, 8, 100, 128, 255, 256, 257, 300, 1000])
def test_window_lengths(ciar, oracle, K):
    """Windows that divide, straddle and exceed the finishing kernel's 256-row workgroups; N = 700 leaves a
    ragged last window for most K."""
    c, t, ids, ua, ur = _random_case(1024, 1024, 700, K, torch.float32, seed=500 + K, sigma=0.25)
    P = ciar.Params(confidence=0.9, window=K, tau=0.01)
    _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=1024, tag=f"window K={K}")


# ---- degenerate rows ----------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_degenerate_rows(ciar, oracle, dtype):
    """Uniform, one-hot, extreme-magnitude, masked (-inf) and identical draft/target rows."""
    V, K = 16384, 4
    g = torch.Generator(device="cuda").manual_seed(7)
    torch.manual_seed(77)                                              # the rows below come from the global CPU generator
    rows = []
    rows.append(torch.zeros(V))                                        # uniform
    rows.append(torch.full((V,), 3.25))                                # uniform, shifted
    r = torch.zeros(V); r[77] = 80.0; rows.append(r)                   # one-hot
    r = torch.zeros(V); r[V - 1] = 30.0; rows.append(r)                # one-hot at the last token
    r = torch.randn(V) * 2 + 80.0; rows.append(r)                      # large positive logits
    r = torch.randn(V) * 2 - 80.0; rows.append(r)                      # large negative logits
    r = torch.randn(V) * 2; r[::3] = -float("inf"); rows.append(r)     # a third of the tokens masked
    r = torch.full((V,), -float("inf")); r[5] = 1.0; r[9000] = 0.5; rows.append(r)   # two live tokens
    r = torch.randn(V) * 0.01; rows.append(r)                          # nearly flat
    r = torch.randn(V) * 10; rows.append(r)                            # very spread
    r = torch.randn(V) * 10; r[0] = r.max() + 3.0; rows.append(r)      # very spread, the first token the largest
    r = torch.randn(V) * 0.5; r[0] = 6.0; rows.append(r)               # flat but for a large first token
    c = torch.stack(rows).cuda()
    N = c.shape[0]
    t = c.clone()
    t[4] = c[4] + 0.5 * torch.randn(V, device="cuda", generator=g)
    t[9] = c[9] + 1.0 * torch.randn(V, device="cuda", generator=g)
    t[2] = torch.full((V,), -30.0, device="cuda"); t[2, 100] = 5.0     # target disagrees with a one-hot draft
    c, t = c.to(dtype), t.to(dtype)
    ids = torch.tensor([0, 5, 77, V - 1, 3, 4, 1, 5, 6, 7, 0, 0], dtype=torch.int32, device="cuda")
    ids[4] = int(torch.argmax(c[4].float())); ids[9] = int(torch.argmax(c[9].float()))
    ua = torch.tensor([0.0, 0.999, 0.5, 0.3, 0.99, 0.2, 0.7, 0.1, 0.6, 0.999, 0.4, 0.8], device="cuda")
    ur = torch.tensor([0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1 - 2.0 ** -24, 0.35, 0.65], device="cuda")
    for norm in (True, False):
        for kap in (-1.0, 0.0, 3.0):
            P = ciar.Params(confidence=0.9, radius_scale=kap, normalize=norm, window=K, tau=1e-3)
            oq, ov, _, _ = _run_case(ciar, oracle, c, t, ids, ua, ur, P, tag=f"degenerate {dtype} norm={norm}")
            assert list(ov["accept"][[0, 1, 3, 5, 6, 7, 8]]) == [1] * 7      # identical rows accept
            assert ov["accept"][2] == 0 and ov["row_id"][2] == 100            # the only residual mass
    # closed forms straight from the GPU (uniform row: Omega = V (p^u - p^l), U = 0; one-hot with caps)
    gq = ciar.quantify(c, ids, ciar.Params(confidence=0.9, window=K))
    torch.cuda.synchronize()
    kappa = math.sqrt(2) * 1.1630871536766743      # erfinv(0.9)
    a, b = math.exp(kappa), math.exp(-kappa)
    assert abs(gq["omega"][0].item() - V * (a / (V - 1 + a) - b / (V - 1 + b))) < 1e-4
    assert gq["score"][0].item() < 1e-7 and gq["flags"][0].item() == 0
    assert abs(gq["omega"][2].item() - 0.02) < 1e-6
    assert abs(gq["score"][2].item() - 0.02 ** 2 * math.sqrt(V - 1) / V) < 1e-9


def test_quantify_without_ids_reports_the_argmax_token(ciar, oracle):
    c, t, ids, ua, ur = _random_case(4096, 4096, 50, 8, torch.float32, seed=5)
    say("[argmax] V=4096 N=50")
    g = ciar.quantify(c, None, ciar.Params())
    torch.cuda.synchronize()
    o = oracle.quantify(c.cpu(), None, _OP(oracle))
    parity.check_floats(g, o)


def test_null_outputs_and_workspace_paths(ciar, oracle):
    """Window outputs only (per-row results go to the workspace), and single outputs."""
    import ctypes
    from paper_2603_25463_amd.binding import _ptr, _stream
    c, t, ids, ua, ur = _random_case(2048, 2048, 43, 5, torch.float32, seed=11)
    say("[null outputs] V=2048 N=43 K=5")
    P = ciar.Params(window=5)
    cp = P.to_c(c)
    L = ciar.lib()
    ref = ciar.verify(c, t, ids, ua, ur, P, workspace=None)
    W = ref["accept_len"].numel()
    al = torch.full((W,), -7, dtype=torch.int32, device="cuda")
    ri = torch.full((W,), -7, dtype=torch.int32, device="cuda")
    ws = torch.empty(ciar.workspace_bytes(43, cp), dtype=torch.uint8, device="cuda")
    rc = L.ciar_verify(_ptr(c), _ptr(t), _ptr(ids), _ptr(ua), _ptr(ur), 43, ctypes.byref(cp),
                       None, None, _ptr(al), _ptr(ri), _ptr(ws), ws.numel(), _stream(None))
    assert rc == 0, ciar.last_error()
    torch.cuda.synchronize()
    assert torch.equal(al, ref["accept_len"]) and torch.equal(ri, ref["resampled_id"])
    # accept_len alone: no residual draw is needed
    al2 = torch.full((W,), -7, dtype=torch.int32, device="cuda")
    rc = L.ciar_verify(_ptr(c), _ptr(t), _ptr(ids), _ptr(ua), _ptr(ur), 43, ctypes.byref(cp),
                       None, None, _ptr(al2), None, _ptr(ws), ws.numel(), _stream(None))
    assert rc == 0, ciar.last_error()
    torch.cuda.synchronize()
    assert torch.equal(al2, ref["accept_len"])
    # a single quantify output
    sc = torch.empty(43, dtype=torch.float32, device="cuda")
    rc = L.ciar_quantify(_ptr(c), None, None, 43, ctypes.byref(cp), None, None, None, None, None, _ptr(sc), None,
                         _ptr(ws), ws.numel(), _stream(None))
    assert rc == 0, ciar.last_error()
    torch.cuda.synchronize()
    assert torch.equal(sc, ciar.quantify(c, ids, P)["score"])


def test_dense_export_matches_the_oracle_curves(ciar, oracle):
    for V, dtype in ((1000, torch.float32), (16384, torch.bfloat16)):
        c, *_ = _random_case(V, V, 6, 4, dtype, seed=21)
        say(f"[dense] V={V} {dtype}")
        for norm in (True, False):
            P = ciar.Params(confidence=0.95, normalize=norm)
            lo, mid, hi = ciar.dense_intervals(c, P)
            torch.cuda.synchronize()
            olo, omid, ohi = oracle.dense_intervals(c.cpu(), _OP(oracle, confidence=0.95, normalize=norm))
            for g, o in ((lo, olo), (mid, omid), (hi, ohi)):
                g = g.cpu().numpy().astype(np.float64)
                assert np.all(np.abs(g - o) <= parity.ATOL + parity.RTOL * np.abs(o))


@pytest.mark.parametrize("V,stride,N,dtype", [(1000, 1000, 9, torch.float32), (16384, 16384, 33, torch.float32),
                                              (16385, 16388, 5, torch.float32), (5000, 5008, 7, torch.bfloat16),
                                              (65536, 65536, 3, torch.bfloat16)])
def test_read_rows_sums_every_logit_once(ciar, V, stride, N, dtype):
    """The bandwidth-ceiling kernel is not part of the method; its row sums are checked against a plain
    fp64 sum of the same bits so that the benchmark's ceiling provably reads every logit."""
    c, t, *_ = _random_case(V, stride, N, 4, dtype, seed=77 + V)
    say(f"[read_rows] V={V} stride={stride} N={N} {dtype}")
    both = ciar.read_rows(c, t, ciar.Params(), vocab=V)
    one = ciar.read_rows(c, None, ciar.Params(), vocab=V)
    torch.cuda.synchronize()
    cs, ts = c[:, :V].double().sum(1), t[:, :V].double().sum(1)
    scale = c[:, :V].double().abs().sum(1) + t[:, :V].double().abs().sum(1)
    assert torch.all((both.double() - (cs + ts)).abs() <= 1e-5 * scale)
    assert torch.all((one.double() - cs).abs() <= 1e-5 * scale)


def test_results_are_deterministic_and_stream_ordered(ciar):
    c, t, ids, ua, ur = _random_case(16384, 16384, 300, 8, torch.float32, seed=31)
    say("[determinism] V=16384 N=300, two runs, second on a side stream")
    P = ciar.Params(tau=0.01)
    a = ciar.quantify_verify(c, t, ids, ua, ur, P)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        b = ciar.quantify_verify(c, t, ids, ua, ur, P, stream=s)
    s.synchronize()
    for k in a:
        assert torch.equal(a[k], b[k]), k


@pytest.mark.parametrize("dtype,V", [(torch.float32, 16384), (torch.bfloat16, 8192)])
def test_calls_overlap_on_two_streams(ciar, dtype, V):
    """Consecutive batches are independent: calls on two streams, each with its own outputs and workspace, may be in
    flight together (bench.py's two-stream figure).  Every call must reproduce what the same batch gives on its own,
    bit for bit -- windows that span workgroups meet in words of the call's own workspace, tagged per launch."""
    N, K = 1024, 8
    P = ciar.Params(confidence=0.9, window=K, tau=0.01)
    batches = [_random_case(V, V, N, K, dtype, seed=900 + b, sigma=0.4) for b in range(2)]
    refs = [ciar.quantify_verify(*b, P) for b in batches]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    wss = [torch.empty(ciar.workspace_bytes(N, P.to_c(batches[0][0])), dtype=torch.uint8, device="cuda") for _ in range(2)]
    outs = [{k: torch.empty_like(v) for k, v in refs[0].items()} for _ in range(2)]
    for rep in range(12):
        for o in outs:
            for v in o.values():
                v.fill_(0)
        torch.cuda.synchronize()
        for lane in (0, 1):
            b = (lane + rep) % 2                                   # the batches swap streams from round to round
            ciar.quantify_verify(*batches[b], P, out=outs[lane], workspace=wss[lane], stream=streams[lane])
        torch.cuda.synchronize()
        for lane in (0, 1):
            ref = refs[(lane + rep) % 2]
            for k in ref:
                assert torch.equal(outs[lane][k], ref[k]), (rep, lane, k)


@pytest.mark.parametrize("N", [1, 2, 7, 255, 256, 257, 511, 513, 1025])
def test_row_counts_around_the_block_sizes(ciar, oracle, N):
    """Row counts below, at and just above the finishing kernels' 256-row workgroups and the streaming
    kernel's resident grid, with a window length that does not divide them."""
    c, t, ids, ua, ur = _random_case(1024, 1024, N, 5, torch.float32, seed=700 + N, sigma=0.4)
    _run_case(ciar, oracle, c, t, ids, ua, ur, ciar.Params(confidence=0.9, window=5, tau=0.01), vocab=1024,
              tag=f"row count N={N}")


@pytest.mark.parametrize("dtype,N,K", [(torch.float32, 300, 8), (torch.bfloat16, 300, 8), (torch.float32, 3000, 8),
                                       (torch.bfloat16, 37, 5)])
def test_calls_replay_from_a_captured_graph(ciar, dtype, N, K):
    """The library allocates nothing, records no memset and never synchronises, so a call can be captured into
    a HIP graph.  Replays (with eager work and synchronisation between them, and the inputs changed between
    replays) must reproduce the eager results bit for bit.  A replay repeats the launch with the same arguments, the
    tag of its counters in the workspace included: windows that span workgroups (few rows, fp32), the list of pending
    draws (bf16) and windows inside workgroups (many rows) all have to start afresh on every replay."""
    c, t, ids, ua, ur = _random_case(16384, 16384, N, K, dtype, seed=41)
    c2, t2, *_ = _random_case(16384, 16384, N, K, dtype, seed=42)
    say(f"[graph] V=16384 N={N} K={K} {dtype}: capture ciar_quantify_verify, replay 4 times on alternating inputs")
    P = ciar.Params(tau=0.01, window=K)
    ref1 = ciar.quantify_verify(c, t, ids, ua, ur, P)
    ref2 = ciar.quantify_verify(c2, t2, ids, ua, ur, P)
    torch.cuda.synchronize()
    cin, tin = c.clone(), t.clone()
    ws = torch.empty(ciar.workspace_bytes(N, P.to_c(c)), dtype=torch.uint8, device="cuda")
    out = {k: torch.empty_like(v) for k, v in ref1.items()}
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        ciar.quantify_verify(cin, tin, ids, ua, ur, P, out=out, workspace=ws, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for i in range(4):
        src_c, src_t, ref = (c, t, ref1) if i % 2 == 0 else (c2, t2, ref2)
        cin.copy_(src_c)
        tin.copy_(src_t)
        for k in out:
            out[k].fill_(0)                      # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in ref:
            assert torch.equal(out[k], ref[k]), (i, k)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_radius_extremes_scalar_mode(ciar, oracle, dtype):
    """Zero radius (the interval collapses onto the softmax; with the caps Omega = 0.02) and the largest radius the
    library accepts, reached by the scale and by the clamp; both normalisation modes."""
    c, t, ids, ua, ur = _random_case(4096, 4096, 48, 8, dtype, seed=81)
    for kap, rmax in ((0.0, 10.0), (1e-3, 10.0), (16.0, 16.0), (200.0, 16.0)):
        for norm in (True, False):
            P = ciar.Params(radius_scale=kap, radius_max=rmax, normalize=norm, tau=0.01)
            _run_case(ciar, oracle, c, t, ids, ua, ur, P, tag=f"radius kappa={kap} rmax={rmax}")


@pytest.mark.parametrize("V,stride,dtype", [(40, 40, torch.float32), (3000, 3008, torch.float32),
                                            (16384, 16384, torch.float32), (16384, 16384, torch.bfloat16),
                                            (65536, 65536, torch.bfloat16)])
def test_verifier_rows_far_from_their_centre_rows(ciar, oracle, V, stride, dtype):
    """The kernel sums the verifier row about the reference of the centre row's tokens and falls back to the
    verifier row's own maximum when that sum leaves the safe range.  Verifier rows that sit hundreds of nats above
    or below their centre rows, that are much sharper or flatter, and rows where only one stretch of the
    vocabulary is far off (some waves fall back, others do not) must give the same decisions and draws."""
    N, K = 24, 4
    c, t, ids, ua, ur = _random_case(V, stride, N, K, dtype, seed=7000 + V)
    t = t.float()
    t[0, :V] += 300.0
    t[1, :V] -= 300.0
    t[2, :V] *= 40.0
    t[3, :V] *= 0.01
    t[4, :V] = t[4, :V] * 30.0 + 500.0
    t[5, :V] = t[5, :V] * 30.0 - 500.0
    lo, hi = V // 3, V // 2
    t[6, lo:hi] += 120.0                                               # one stretch far above ...
    t[7, lo:hi] -= 250.0                                               # ... far below its centre tokens
    t[8, :lo] -= 400.0
    t[9, 0] += 200.0                                                   # a single verifier token holds the mass
    t[10, V - 1] += 90.0
    c = c.float()
    c[11, :V] += 250.0                                                 # the centre row is the one far off
    c[12, :V] -= 250.0
    c[13, lo:hi] += 150.0
    c, t = c.to(dtype), t.to(dtype)
    for P in (ciar.Params(window=K, tau=0.01), ciar.Params(radius_scale=0.7, normalize=False, window=K, tau=0.01)):
        oq, ov, exf, st = _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=V, tag="verifier far from centre")
    assert st["rejected"] >= 4                                         # draws were compared as well


@pytest.mark.parametrize("V,stride,dtype", [(3000, 3008, torch.float32), (16384, 16384, torch.float32),
                                            (16384, 16384, torch.bfloat16), (65536, 65536, torch.bfloat16)])
def test_probabilities_around_the_small_probability_bound(ciar, oracle, V, stride, dtype):
    """Scalar radius: the kernel evaluates the widths of tokens with small probabilities by a polynomial and the
    others by the rational form, deciding per 16-byte vector of 64 lanes against a bound that depends on the
    radius (about 0.02 at confidence 0.9, 0.1 at radius 0.5, 5e-4 at radius 5).  Rows whose probabilities are
    spread log-uniformly from 1e-5 to 0.3 put tokens on both sides of the bound at every radius, in varying
    numbers per vector; the background is flat so that the rest of the mass is far below it."""
    N, K = 24, 4
    g = torch.Generator().manual_seed(9000 + V)
    c = 0.05 * torch.randn((N, stride), generator=g)
    for r in range(N):
        k = 4 + 9 * r                                                  # tokens lifted out of the background
        near = k // 2 if r % 3 == 0 else 0                             # ... some of them next to each other
        pos = torch.cat([torch.arange(near), near + torch.randperm(V - near, generator=g)[: k - near]])
        p = torch.exp(torch.empty(k).uniform_(float(np.log(1e-5)), float(np.log(0.3)), generator=g))
        p = p * min(1.0, 0.9 / float(p.sum()))
        rest = (1.0 - float(p.sum())) / (V - k)                        # probability of a background token
        c[r, pos] = torch.log(p / rest)
    c = c.to(dtype).cuda()
    t = (c.float() + 0.3 * torch.randn(c.shape, generator=torch.Generator(device="cuda").manual_seed(5),
                                       device="cuda")).to(dtype)
    ids = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).cuda()
    ua, ur = torch.rand(N, generator=g).cuda(), torch.rand(N, generator=g).cuda()
    for kap in (0.1, 0.5, 1.0, 1.645, 2.5, 5.0, 8.0):
        for norm in (True, False):
            P = ciar.Params(radius_scale=kap, normalize=norm, window=K, tau=0.01)
            _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=V, tag=f"small-probability bound r={kap}")


@pytest.mark.parametrize("V,stride,dtype", [(2, 4, torch.float32), (50, 56, torch.float32), (1000, 1000, torch.float32),
                                            (3000, 3008, torch.float32), (8192, 8192, torch.float32),
                                            (16384, 16384, torch.float32), (32768, 32768, torch.float32),
                                            (40, 40, torch.bfloat16), (16384, 16384, torch.bfloat16),
                                            (65536, 65536, torch.bfloat16)])
def test_wide_radius(ciar, oracle, V, stride, dtype):
    """Radii from 6 to the accepted maximum of 16: towards the upper end every width approaches 1 and Sigma, the
    spread of numbers that differ in the fifth digit and beyond, falls to 1e-5 while Omega ~ V.  The score must
    still meet the tolerance: every vocabulary tile, flat and peaked rows, rows with tokens at probability 0, both
    radius modes."""
    N, K = 20, 4
    c, t, ids, ua, ur = _random_case(V, stride, N, K, dtype, seed=300 + V)
    c[:5] *= 0.2                                                       # flat rows: widths crowd together earliest
    c[5:8] *= 4.0                                                      # peaked rows
    if V > 8:
        c[8, : V // 2] = -200.0                                        # half the tokens at probability 0: widths 0 and ~1
    c[9, 0] = 60.0                                                     # one token holds the mass
    for r in (6.0, 10.0, 13.0, 15.0, 16.0):
        P = ciar.Params(radius_scale=r, radius_max=16.0, window=K, tau=1e-4)
        oq, *_ = _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=V, tag=f"wide radius r={r}")
    assert float(np.min(oq["sigma"])) < 1e-3 or V <= 64                # the regime was reached
    raw = _raw_radius(N, stride, V, dtype, seed=400 + V, mu_lo=2.0, mu_hi=30.0, sd=0.5)
    for kap, rmax in ((1.0, 16.0), (3.0, 12.0)):
        P = ciar.Params(radius_scale=kap, radius_max=rmax, window=K, tau=1e-4)
        _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=V, tag=f"wide tensor radius kappa={kap} rmax={rmax}",
                  radius=raw)


@pytest.mark.parametrize("V,dtype", [(48, torch.float32), (4096, torch.float32), (16384, torch.bfloat16)])
def test_wide_radius_multihead(ciar, oracle, V, dtype):
    H, N = 3, 12
    heads = _head_stack(H, V, V, N, dtype, seed=4500 + V)
    heads[:, :4] *= 0.2
    ids = torch.arange(N, device="cuda", dtype=torch.int32) % V
    hh = heads.cpu()
    raw = torch.stack([_raw_radius(N, V, V, dtype, seed=5500 + V + h, mu_lo=5.0, mu_hi=30.0, sd=0.5)
                       for h in range(H)]).contiguous()
    for kw, okw, rh in ((dict(radius_scale=13.0, radius_max=16.0), dict(kappa=13.0, radius_max=16.0), None),
                        (dict(radius_scale=30.0, radius_max=16.0), dict(kappa=30.0, radius_max=16.0), None),
                        (dict(radius_scale=1.0, radius_max=16.0), dict(kappa=1.0, radius_max=16.0), raw)):
        say(f"[multihead wide] V={V} {dtype} {kw} radius={'tensor' if rh is not None else 'scalar'}")
        P, OP = ciar.Params(tau=1e-4, **kw), _OP(oracle, tau=1e-4, **okw)
        for strategy, ostrategy in ((ciar.ENSEMBLE, oracle.ENSEMBLE), (ciar.VOTING, oracle.VOTING)):
            g = ciar.quantify_multihead(heads, ids, P, strategy, vocab=V, radius_heads=rh)
            torch.cuda.synchronize()
            o = oracle.quantify_multihead(hh, ids.cpu().numpy(), OP, ostrategy, vocab=V,
                                          radius_heads=None if rh is None else rh.cpu())
            if strategy == ciar.ENSEMBLE:
                parity.check_floats(g, o)
                parity.check_flags(g["flags"], o, float(np.float32(1e-4)))
            else:
                for h in range(H):
                    parity.check_floats({k: g[k][h] for k in parity.FLOAT_KEYS}, {k: o[k][h] for k in parity.FLOAT_KEYS})


# ---- seeded random walk over the parameter space -------------------------------------------------------------

def _archetype_rows(N, V, stride, dtype, rng, dev_gen):
    """Rows of mixed character: Gaussian logits of a random scale, a planted peak of random height, a block of
    masked (-inf) tokens, ties for the maximum, constant rows."""
    c = torch.randn((N, stride), generator=dev_gen, device="cuda")
    for i in range(N):
        kind = rng.integers(0, 7)
        c[i] *= float(10.0 ** rng.uniform(-2.0, 1.3))
        if kind == 1:
            c[i, int(rng.integers(0, V))] += float(rng.uniform(5.0, 90.0))
        elif kind == 2 and V > 4:
            lo = int(rng.integers(0, V - 2)); hi = int(rng.integers(lo + 1, V))
            c[i, lo:hi] = float("-inf")
            if hi - lo >= V - 1:
                c[i, 0] = 0.0
        elif kind == 3:
            m = c[i, :V].max()
            for j in rng.integers(0, V, size=3):
                c[i, int(j)] = m
        elif kind == 4:
            c[i] = float(rng.uniform(-50.0, 50.0))
        elif kind == 5:
            c[i] += float(rng.uniform(-100.0, 100.0))
    return c


@pytest.mark.parametrize("seed", [511620])
def test_random_parameters_found_cases(ciar, oracle, seed):
    """A case that a long run of the sweep below found.  511620 (V = 101, bf16, scalar radius 1.75): a nearly one-hot row
    with both caps active, Omega = cap_hi - cap_lo = 0.01; the fp32 lower bound of the token above 1/2 left S_l 2e-7
    off, which the cap then no longer absorbed: Omega 2.04e-7 off against a bound of 2.00e-7.  The finishing lane now
    exchanges that token's fp32 values for fp64 ones."""
    test_random_parameters(ciar, oracle, seed)


@pytest.mark.parametrize("seed", _sweep_seeds("CIAR_RANDOM_CASES", 32))
def test_random_parameters(ciar, oracle, seed):
    """Vocabulary, stride, dtype, window, radius mode, scale, clamp, caps and normalisation drawn at random (seeded),
    rows of mixed character; the threshold sits at the oracle's median score."""
    rng = np.random.default_rng(9000 + seed)
    dtype = (torch.float32, torch.bfloat16)[int(rng.integers(0, 2))]
    epv = 4 if dtype == torch.float32 else 8
    vmax = 32768 if dtype == torch.float32 else 65536
    V = int(min(vmax, max(2, round(2.0 ** rng.uniform(1.0, 16.0)))))
    stride = -(-V // epv) * epv + epv * int(rng.integers(0, 3))
    if stride > vmax:
        stride = -(-V // epv) * epv
    K = int(rng.integers(1, 12))
    N = K * int(rng.integers(1, 5)) + int(rng.integers(0, K))
    gen = torch.Generator(device="cuda").manual_seed(9100 + seed)
    c = _archetype_rows(N, V, stride, dtype, rng, gen)
    t = c + float(10.0 ** rng.uniform(-2.0, 0.5)) * torch.randn((N, stride), generator=gen, device="cuda")
    t = torch.where(torch.isfinite(t), t, c)                          # masked tokens stay masked on both sides
    if stride > V:
        c[:, V:] = 1e30
        t[:, V:] = -1e30
    c, t = c.to(dtype), t.to(dtype)
    gum = -torch.log(-torch.log(torch.rand((N, V), generator=gen, device="cuda").clamp_(1e-30, 1 - 1e-7)))
    ids = torch.argmax(c[:, :V].float() + gum, dim=1).to(torch.int32)  # drafted from the centre distribution
    ua = torch.randint(0, 1 << 24, (N,), generator=gen, device="cuda").float() / (1 << 24)
    ur = torch.randint(0, 1 << 24, (N,), generator=gen, device="cuda").float() / (1 << 24)
    tensor_mode = bool(rng.integers(0, 2))
    raw = None
    if tensor_mode:
        raw = _raw_radius(N, stride, V, dtype, seed=9200 + seed, mu_lo=float(rng.uniform(-20.0, 0.0)),
                          mu_hi=float(rng.uniform(0.0, 20.0)), sd=float(10.0 ** rng.uniform(-1.0, 1.0)))
    kw = dict(radius_scale=float(10.0 ** rng.uniform(-3.0, 1.3)), radius_max=float(rng.uniform(0.3, 16.0)),
              normalize=bool(rng.integers(0, 4)), window=K,
              lower_cap=float(rng.choice([0.99, 0.9, 0.5, 1.0])), upper_cap=float(rng.choice([1.01, 1.1, 2.0, 1.0])))
    if rng.integers(0, 3) == 0:
        kw["radius_scale"] = -1.0
        kw["confidence"] = float(rng.choice([0.5, 0.8, 0.9, 0.95, 0.999]))
    say(f"[random {seed}] V={V} stride={stride} N={N} {dtype} {kw} radius={'tensor' if tensor_mode else 'scalar'}")
    o0 = oracle.quantify(c.cpu(), ids.cpu().numpy(), _oparams(oracle, ciar.Params(**kw)), vocab=V,
                         radius=None if raw is None else raw.cpu())
    # between the two middle scores, not on one of them: float32(U) of a large U is further than the 1e-6 margin
    # from U itself, and no arithmetic could then be asked to reproduce the flag
    sc = np.sort(np.asarray(o0["score"], dtype=np.float64))
    lo, hi = sc[(N - 1) // 2], sc[min(N - 1, (N - 1) // 2 + 1)]
    tau = float(np.float32(0.5 * (lo + hi) if hi - lo > 1e-3 * hi else 0.5 * lo))
    P = ciar.Params(tau=tau, **kw)
    _run_case(ciar, oracle, c, t, ids, ua, ur, P, vocab=V, tag=f"random {seed}", radius=raw)
    # the same rows without drafted ids (the arg-max token is reported; rows with a tie for the maximum are left
    # out: which of the tied tokens is lowest is covered elsewhere, here their radii may differ) and as dense curves
    OP = _oparams(oracle, P)
    rh = None if raw is None else raw.cpu()
    g = ciar.quantify(c, None, P, vocab=V, radius=raw)
    lo, mid, hi = ciar.dense_intervals(c, P, vocab=V, radius=raw)
    torch.cuda.synchronize()
    o = oracle.quantify(c.cpu(), None, OP, vocab=V, radius=rh)
    cf = c[:, :V].float()
    untied = ((cf == cf.max(dim=1, keepdim=True).values).sum(dim=1) == 1).cpu().numpy()
    parity.check_floats({k: g[k][torch.from_numpy(untied).cuda()] for k in parity.FLOAT_KEYS},
                        {k: np.asarray(o[k])[untied] for k in parity.FLOAT_KEYS})
    olo, omid, ohi = oracle.dense_intervals(c.cpu(), OP, vocab=V, radius=rh)
    for gd, od, name in ((lo, olo, "p_lo"), (mid, omid, "p_mid"), (hi, ohi, "p_hi")):
        gd = gd.cpu().numpy().astype(np.float64)
        bad = np.abs(gd - od) > parity.ATOL + parity.RTOL * np.abs(od)
        assert not bad.any(), (name, np.argwhere(bad)[0], gd[bad][0], od[bad][0])


@pytest.mark.parametrize("seed", list(range(6)))
def test_random_parameters_many_rows(ciar, oracle, seed):
    """Thousands of rows of mixed character and a small vocabulary: every workgroup of the streaming kernel walks
    over several rows, windows straddle workgroups, and the finishing kernels see long lists of rejected rows."""
    rng = np.random.default_rng(39000 + seed)
    dtype = (torch.float32, torch.bfloat16)[seed % 2]
    epv = 4 if dtype == torch.float32 else 8
    V = int(rng.integers(40, 2100))
    stride = -(-V // epv) * epv + epv * int(rng.integers(0, 2))
    K = int(rng.integers(1, 20))
    N = int(rng.integers(1500, 9000))
    gen = torch.Generator(device="cuda").manual_seed(39100 + seed)
    c = torch.randn((N, stride), generator=gen, device="cuda") * (torch.rand((N, 1), generator=gen, device="cuda") * 3 + 0.05)
    kinds = torch.randint(0, 6, (N,), generator=gen, device="cuda")
    peak = torch.randint(0, V, (N,), generator=gen, device="cuda")
    rows = torch.arange(N, device="cuda")
    c[rows[kinds == 1], peak[kinds == 1]] += 12.0                       # peaked rows
    c[kinds == 2, : V // 3] = float("-inf")                             # a third of the tokens masked
    c[kinds == 3] = 1.5                                                 # constant rows
    c[kinds == 4] += 70.0                                               # large common offset
    t = c + float(10.0 ** rng.uniform(-1.5, 0.3)) * torch.randn((N, stride), generator=gen, device="cuda")
    t = torch.where(torch.isfinite(t), t, c)
    if stride > V:
        c[:, V:] = 1e30
        t[:, V:] = -1e30
    c, t = c.to(dtype), t.to(dtype)
    gum = -torch.log(-torch.log(torch.rand((N, V), generator=gen, device="cuda").clamp_(1e-30, 1 - 1e-7)))
    ids = torch.argmax(c[:, :V].float() + gum, dim=1).to(torch.int32)
    ua = torch.randint(0, 1 << 24, (N,), generator=gen, device="cuda").float() / (1 << 24)
    ur = torch.randint(0, 1 << 24, (N,), generator=gen, device="cuda").float() / (1 << 24)
    raw = _raw_radius(N, stride, V, dtype, seed=39200 + seed) if seed % 3 == 2 else None
    kw = dict(radius_scale=float(10.0 ** rng.uniform(-1.0, 0.9)), radius_max=float(rng.uniform(1.0, 12.0)),
              normalize=bool(seed % 4 != 3), window=K)
    say(f"[random many rows {seed}] V={V} stride={stride} N={N} K={K} {dtype} {kw} "
        f"radius={'tensor' if raw is not None else 'scalar'}")
    o0 = oracle.quantify(c.cpu(), ids.cpu().numpy(), _oparams(oracle, ciar.Params(**kw)), vocab=V,
                         radius=None if raw is None else raw.cpu())
    tau = float(np.float32(np.median(o0["score"])))
    _, _, exf, st = _run_case(ciar, oracle, c, t, ids, ua, ur, ciar.Params(tau=tau, **kw), vocab=V,
                              tag=f"random many rows {seed}", radius=raw)
    assert exf <= 2 + N // 500 and st["exempt_accept"] <= 2 + N // 1000


def _random_shape(rng):
    dtype = (torch.float32, torch.bfloat16)[int(rng.integers(0, 2))]
    epv = 4 if dtype == torch.float32 else 8
    vmax = 32768 if dtype == torch.float32 else 65536
    V = int(min(vmax, max(2, round(2.0 ** rng.uniform(1.0, 16.0)))))
    stride = -(-V // epv) * epv + epv * int(rng.integers(0, 3))
    if stride > vmax:
        stride = -(-V // epv) * epv
    return dtype, V, stride


@pytest.mark.parametrize("seed", _sweep_seeds("CIAR_RANDOM_BATCHES", 6))
def test_random_batches(ciar, oracle, seed):
    """Whole batches of random size (one row to several thousand: one row per workgroup up to many, windows inside
    workgroups and across them, the last one ragged), window length, vocabulary (every tile), dtype and radius mode,
    every entry point against the oracle.  The threshold sits at the median score of a first pass."""
    rng = np.random.default_rng(39000 + seed)
    dtype = (torch.float32, torch.bfloat16)[int(rng.integers(0, 2))]
    V = int(rng.choice([257, 1024, 4096, 8192, 16384, 32768 if dtype == torch.float32 else 65536]))
    N = int(min(max(1, round(2.0 ** rng.uniform(0.0, 13.0))), max(1, 30_000_000 // V)))
    K = int(rng.choice([1, 2, 3, 4, 8, 16, 37, 255, 300]))
    stride = -(-V // 8) * 8                                        # rows are 16-byte aligned in either dtype
    c, t, ids, ua, ur = _random_case(V, stride, N, K, dtype, seed=39100 + seed, sigma=float(10.0 ** rng.uniform(-1.5, 0.3)))
    raw = _raw_radius(N, stride, V, dtype, seed=39200 + seed) if rng.integers(0, 3) == 0 else None
    kw = dict(confidence=float(rng.choice([0.8, 0.9, 0.95])), window=K)
    if raw is not None:
        kw["radius_scale"] = 1.0
    o0 = oracle.quantify(c.cpu(), ids.cpu().numpy(), _oparams(oracle, ciar.Params(tau=0.3, **kw)),
                         radius=None if raw is None else raw.cpu())
    tau = float(np.float32(np.median(np.asarray(o0["score"], dtype=np.float64))))
    _run_case(ciar, oracle, c, t, ids, ua, ur, ciar.Params(tau=tau, **kw), vocab=V, tag=f"random batch {seed}", radius=raw)


@pytest.mark.parametrize("seed", [201046])
def test_random_batches_found_cases(ciar, oracle, seed):
    """A batch that a long run of the sweep above found (bf16, V = 4096, tensor radius).  Row 1465 is rejected and its
    u_res R lies 5e-8 R above the lower edge of the oracle's token, behind a stretch of tokens without residual mass:
    the fused call and the verify-only call, both inside the margin band, drew different tokens (1662 and 1671; the
    oracle 1672), and the test then demanded that the entry points agree on every row.  They are now compared with
    each other where the oracle's margin is not below the exemption's, and each with the oracle under the margin rule."""
    test_random_batches(ciar, oracle, seed)


@pytest.mark.parametrize("seed", [10812])
def test_random_parameters_multihead_found_cases(ciar, oracle, seed):
    """A case that a long run of the random sweep below found.  10812: two heads under a radius tensor of scale 17, one
    with widths next to 1 and one with widths next to nothing, so that every averaged width is about 1/2 and their
    spread 2e-4 of that: the fp32 token arithmetic of the Ensemble sweep left the score 2e-5 off (such rows are now
    swept again in fp64)."""
    _random_multihead_case(ciar, oracle, seed)


@pytest.mark.parametrize("seed", _sweep_seeds("CIAR_RANDOM_CASES", 16))
def test_random_parameters_multihead(ciar, oracle, seed):
    """Ensemble and Voting with the number of heads, the shapes and the quantifier's parameters drawn at random."""
    _random_multihead_case(ciar, oracle, seed)


def _random_multihead_case(ciar, oracle, seed):
    rng = np.random.default_rng(19000 + seed)
    dtype, V, stride = _random_shape(rng)
    H = int(rng.integers(1, 9))
    N = int(rng.integers(1, 14))
    gen = torch.Generator(device="cuda").manual_seed(19100 + seed)
    base = _archetype_rows(N, V, stride, torch.float32, rng, gen)
    noise = float(10.0 ** rng.uniform(-2.0, 0.3))
    heads = torch.stack([base + noise * torch.randn((N, stride), generator=gen, device="cuda") for _ in range(H)])
    heads = torch.where(torch.isfinite(base).unsqueeze(0).expand_as(heads), heads, base.unsqueeze(0).expand_as(heads))
    if stride > V:
        heads[:, :, V:] = 1e30
    heads = heads.to(dtype).contiguous()
    ids = torch.randint(0, V, (N,), generator=gen, device="cuda").to(torch.int32)
    raw = None
    if rng.integers(0, 2):
        raw = torch.stack([_raw_radius(N, stride, V, dtype, seed=19200 + 10 * seed + h,
                                       mu_lo=float(rng.uniform(-10.0, 0.0)), mu_hi=float(rng.uniform(0.0, 10.0)),
                                       sd=float(10.0 ** rng.uniform(-1.0, 0.7))) for h in range(H)]).contiguous()
    kw = dict(radius_scale=float(10.0 ** rng.uniform(-3.0, 1.3)), radius_max=float(rng.uniform(0.3, 16.0)),
              normalize=bool(rng.integers(0, 4)),
              lower_cap=float(rng.choice([0.99, 0.9, 0.5, 1.0])), upper_cap=float(rng.choice([1.01, 1.1, 2.0, 1.0])))
    say(f"[random multihead {seed}] H={H} V={V} stride={stride} N={N} {dtype} {kw} "
        f"radius={'tensor' if raw is not None else 'scalar'}")
    hh, rh = heads.cpu(), None if raw is None else raw.cpu()
    P0 = ciar.Params(**kw)
    o0 = oracle.quantify_multihead(hh, ids.cpu().numpy(), _oparams(oracle, P0), oracle.ENSEMBLE, vocab=V,
                                   radius_heads=rh)
    sc = np.sort(np.asarray(o0["score"], dtype=np.float64))
    lo, hi = sc[(N - 1) // 2], sc[min(N - 1, (N - 1) // 2 + 1)]
    tau = float(np.float32(0.5 * (lo + hi) if hi - lo > 1e-3 * hi else 0.5 * lo))
    P = ciar.Params(tau=tau, **kw)
    OP = _oparams(oracle, P)
    ge = ciar.quantify_multihead(heads, ids, P, ciar.ENSEMBLE, vocab=V, radius_heads=raw)
    gv = ciar.quantify_multihead(heads, ids, P, ciar.VOTING, vocab=V, radius_heads=raw)
    torch.cuda.synchronize()
    oe = oracle.quantify_multihead(hh, ids.cpu().numpy(), OP, oracle.ENSEMBLE, vocab=V, radius_heads=rh)
    ov = oracle.quantify_multihead(hh, ids.cpu().numpy(), OP, oracle.VOTING, vocab=V, radius_heads=rh)
    parity.check_floats(ge, oe)
    parity.check_flags(ge["flags"], oe, float(np.float32(tau)))
    for h in range(H):
        gh = {k: gv[k][h] for k in parity.FLOAT_KEYS}
        oh = {k: ov[k][h] for k in parity.FLOAT_KEYS}
        oh["flags"] = ov["head_flags"][h]
        parity.check_floats(gh, oh)
        parity.check_flags(gv["head_flags"][h], oh, float(np.float32(tau)))
    votes = gv["head_flags"].sum(0, dtype=torch.int32)
    assert torch.equal(gv["flags"], (2 * votes > H).to(torch.uint8))


@pytest.mark.parametrize("seed", [938, 3757, 106102, 303924])
def test_random_parameters_interdro_found_cases(ciar, oracle, seed):
    """Cases that long runs of the random sweep below found (all: a cloud row close to the centre row).  938: the KL
    term, then formed as the difference of two cross-entropy-sized sums, missed its absolute bound by a quarter (it is
    now summed over the per-token differences).  3757: an L1 distance of 4e-4 was off by 1.06e-7 because the ratio of
    the two normalisers was rounded to one float (now two).  106102 (scalar radius, so the three distributions are
    the same one): the L1 distances to softmax(c + r) and softmax(c - r), 6e-3, were off by +1.7e-7 and -1.6e-7 because
    the constant r - r* was added to the exponents before the exponential, which rounds all exponents of a binade the
    same way (the exponentials are now products e^(c - c*) e^(+-(r - r*))).  303924 (radius tensor, scale 3.9, two tokens
    of probability ~1/2): the same two distances, 2.5e-3 and 6.6e-3, were off by +1.9e-7 and -2.2e-7 because the
    Softplus formed ln(1 + t) from the rounded sum 1 + t, 6e-8 absolute times the scale in the radius (what the sum
    loses is now given back)."""
    _random_interdro_case(ciar, oracle, seed)


@pytest.mark.parametrize("seed", _sweep_seeds("CIAR_RANDOM_CASES", 16))
def test_random_parameters_interdro(ciar, oracle, seed):
    """The Inter-DRO loss with shapes, radius mode, scale, clamp, weights and temperature drawn at random."""
    _random_interdro_case(ciar, oracle, seed)


def _random_interdro_case(ciar, oracle, seed):
    rng = np.random.default_rng(29000 + seed)
    dtype, V, stride = _random_shape(rng)
    N = int(rng.integers(1, 40))
    gen = torch.Generator(device="cuda").manual_seed(29100 + seed)
    c = torch.randn((N, stride), generator=gen, device="cuda") * float(10.0 ** rng.uniform(-1.5, 0.8))
    t = c + float(10.0 ** rng.uniform(-2.0, 0.5)) * torch.randn((N, stride), generator=gen, device="cuda")
    if rng.integers(0, 2) and V > 4:
        t[int(rng.integers(0, N)), int(rng.integers(0, V))] = float("-inf")   # a token the cloud rules out
    if stride > V:
        c[:, V:] = 1e30
        t[:, V:] = 1e30
    c, t = c.to(dtype), t.to(dtype)
    raw = None
    if rng.integers(0, 2):
        raw = _raw_radius(N, stride, V, dtype, seed=29200 + seed, mu_lo=float(rng.uniform(-6.0, 0.0)),
                          mu_hi=float(rng.uniform(0.0, 3.0)), sd=float(10.0 ** rng.uniform(-1.0, 0.3)))
    kw = dict(radius_scale=float(10.0 ** rng.uniform(-2.0, 0.7)), radius_max=float(rng.uniform(0.3, 8.0)))
    lam = tuple(float(10.0 ** rng.uniform(-1.0, 0.7)) for _ in range(3)) + (float(10.0 ** rng.uniform(-1.0, 0.5)),)
    say(f"[random interdro {seed}] V={V} stride={stride} N={N} {dtype} {kw} lam={lam} "
        f"radius={'tensor' if raw is not None else 'scalar'}")
    P = ciar.Params(**kw)
    g = ciar.interdro_loss(c, raw, t, P, *lam, vocab=V)
    torch.cuda.synchronize()
    o = oracle.interdro_loss(c.cpu(), None if raw is None else raw.cpu(), t.cpu(), _oparams(oracle, P), *lam, vocab=V)
    _check_dro(g, o, N)


def test_timed_stage_records_the_kernel_and_changes_nothing(ciar):
    """ciar_stream_rows_timed: same results as the untimed stage, and the two events enclose the kernel."""
    c, t, ids, ua, ur = _random_case(16384, 16384, 512, 8, torch.float32, seed=91)
    P = ciar.Params(window=8)
    ws = torch.empty(ciar.workspace_bytes(512, P.to_c(c)), dtype=torch.uint8, device="cuda")
    say("[timed stage] V=16384 N=512")
    ref = ciar.stream_rows(c, t, ids, ua, ur, P, ws)
    ref = ciar.finish_rows(c, t, ids, ua, ur, P, ws, out=ref)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(); e1.record()
    torch.cuda.synchronize()
    for _ in range(3):
        got = ciar.stream_rows(c, t, ids, ua, ur, P, ws, events=(e0, e1))
        got = ciar.finish_rows(c, t, ids, ua, ur, P, ws, out=got)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        assert 0.002 < ms < 5.0, ms                                    # a kernel over 64 MB: microseconds, not zero
    for k in ref:
        assert torch.equal(ref[k], got[k]), k


def test_bad_arguments_raise(ciar):
    c = torch.zeros((4, 1024), device="cuda")
    with pytest.raises(ciar.CiarError, match="CIAR_EUNSUPPORTED"):
        ciar.quantify(torch.zeros((2, 40000), device="cuda"), None, ciar.Params())
    with pytest.raises(ciar.CiarError, match="CIAR_EALIGN"):
        ciar.quantify(torch.zeros((4, 1028), device="cuda")[:, 1:1025], None, ciar.Params())
    with pytest.raises(ciar.CiarError, match="CIAR_EINVAL"):
        ciar.quantify(c, None, ciar.Params(confidence=1.5))
    with pytest.raises(ciar.CiarError, match="radius_max"):
        ciar.quantify(c, None, ciar.Params(radius_max=16.5))
    with pytest.raises(TypeError):
        ciar.quantify(c.half(), None, ciar.Params())
