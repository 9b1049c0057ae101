"""Pins of the fp64 CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU or the HIP library.  Each pin compares the oracle with
something other than itself: a library routine (scipy softmax / expit / erfinv, numpy std),
a closed form, a bound or identity proved in the paper's appendix, or brute-force enumeration
on a tiny vocabulary.  Citations name the paper's sections, equations and claims.
"""
import math
import os

import numpy as np
import pytest
import scipy.special as sps
import scipy.stats as spst

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


def _golden():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    return vals


def _rows(rng, n, V, scale=2.0):
    return (rng.standard_normal((n, V)) * scale).astype(np.float32)


# ---- radius from the interval confidence -------------------------------------------------

def test_kappa_is_the_two_sided_normal_quantile(oracle):
    g = _golden()
    # textbook z-table values (two-sided 80 / 90 / 95 % intervals)
    assert abs(oracle.kappa(0.80) - g["kappa_0.80"]) < 5e-5
    assert abs(oracle.kappa(0.90) - g["kappa_0.90"]) < 5e-5
    assert abs(oracle.kappa(0.95) - g["kappa_0.95"]) < 5e-5
    for gam in (0.1, 0.5, 0.8, 0.9, 0.95, 0.999):
        assert abs(oracle.kappa(gam) - math.sqrt(2.0) * sps.erfinv(gam)) < 1e-12
        assert abs(oracle.kappa(gam) - spst.norm.ppf(0.5 + gam / 2)) < 1e-10


# ---- softmax and InterFuse --------------------------------------------------------------

def test_zero_radius_reduces_to_library_softmax(oracle):
    """r = 0, no caps: p^l = p^u = softmax(c); Omega = Sigma = U = 0.  (InterFuse equations with r_i = 0)"""
    rng = np.random.default_rng(1)
    c = _rows(rng, 5, 97, 3.0)
    P = oracle.Params(kappa=0.0, normalize=False)
    lo, mid, hi = oracle.dense_intervals(c, P)
    ref = sps.softmax(c.astype(np.float64), axis=1)
    np.testing.assert_allclose(mid, ref, rtol=1e-13, atol=0)
    np.testing.assert_allclose(lo, ref, rtol=1e-13, atol=0)
    np.testing.assert_allclose(hi, ref, rtol=1e-13, atol=0)
    np.testing.assert_allclose(mid.sum(1), 1.0, rtol=1e-13)
    q = oracle.quantify(c, None, P)
    assert np.all(np.abs(q["omega"]) < 1e-14) and np.all(q["score"] < 1e-15)


def test_zero_radius_with_caps_scales_by_099_and_101(oracle):
    """r = 0 with the normalisation on: S_l = S_u = 1, so p^l = 0.99 p, p^u = 1.01 p,
    Omega = 0.02 and Sigma = 0.02 std(p).  (normalisation equations of the validity appendix)"""
    rng = np.random.default_rng(2)
    c = _rows(rng, 4, 64, 2.0)
    P = oracle.Params(kappa=0.0, normalize=True)
    lo, mid, hi = oracle.dense_intervals(c, P)
    ref = sps.softmax(c.astype(np.float64), axis=1)
    np.testing.assert_allclose(lo, 0.99 * ref, rtol=1e-12)
    np.testing.assert_allclose(hi, 1.01 * ref, rtol=1e-12)
    q = oracle.quantify(c, None, P)
    np.testing.assert_allclose(q["omega"], 0.02, rtol=1e-10)
    np.testing.assert_allclose(q["sigma"], 0.02 * ref.std(axis=1), rtol=1e-9)


def test_two_token_vocabulary_is_the_logistic_sigmoid(oracle):
    """V = 2: p_1 = sigma(c1 - c2), p^u_1 = sigma(c1 - c2 + r), p^l_1 = sigma(c1 - c2 - r)."""
    rng = np.random.default_rng(3)
    c = _rows(rng, 50, 2, 3.0)
    r = 0.7
    lo, mid, hi = oracle.dense_intervals(c, oracle.Params(kappa=r, normalize=False))
    d = c[:, 0].astype(np.float64) - c[:, 1].astype(np.float64)
    np.testing.assert_allclose(mid[:, 0], sps.expit(d), rtol=1e-13)
    np.testing.assert_allclose(hi[:, 0], sps.expit(d + r), rtol=1e-13)
    np.testing.assert_allclose(lo[:, 0], sps.expit(d - r), rtol=1e-13)
    np.testing.assert_allclose(hi[:, 1], sps.expit(-d + r), rtol=1e-13)
    np.testing.assert_allclose(lo[:, 1], sps.expit(-d - r), rtol=1e-13)


def test_interfuse_equals_softmax_of_the_row_with_one_logit_shifted(oracle):
    """The denominator of p^u_i is the partition sum of the row whose i-th logit is raised by r
    (and lowered by r for p^l_i): brute force with a library softmax, one perturbed row per token."""
    rng = np.random.default_rng(4)
    V, r = 11, 1.3
    c = _rows(rng, 3, V, 2.5)
    lo, mid, hi = oracle.dense_intervals(c, oracle.Params(kappa=r, normalize=False))
    for n in range(c.shape[0]):
        for i in range(V):
            up = c[n].astype(np.float64).copy(); up[i] += r
            dn = c[n].astype(np.float64).copy(); dn[i] -= r
            assert abs(hi[n, i] - sps.softmax(up)[i]) < 1e-14
            assert abs(lo[n, i] - sps.softmax(dn)[i]) < 1e-14


def test_radius_clamp_and_confidence_mapping(oracle):
    rng = np.random.default_rng(5)
    c = _rows(rng, 2, 33)
    a = oracle.dense_intervals(c, oracle.Params(kappa=50.0, radius_max=1.5, normalize=False))
    b = oracle.dense_intervals(c, oracle.Params(kappa=1.5, radius_max=10.0, normalize=False))
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    g = oracle.dense_intervals(c, oracle.Params(confidence=0.9, normalize=False))
    k = oracle.dense_intervals(c, oracle.Params(kappa=math.sqrt(2) * sps.erfinv(0.9), normalize=False))
    for x, y in zip(g, k):
        np.testing.assert_allclose(x, y, rtol=1e-12)


def test_validity_and_ordering_invariants(oracle):
    """p^l <= p_mid <= p^u, S_l <= 1 <= S_u raw; S_l <= 0.99 and S_u >= 1.01 after the caps."""
    rng = np.random.default_rng(6)
    for V, scale in ((7, 1.0), (256, 0.2), (256, 4.0), (1000, 8.0)):
        c = _rows(rng, 6, V, scale)
        c[0, :] = 0.0                      # uniform
        c[1, :] = 0.0; c[1, 3] = 40.0      # one-hot
        for kap in (0.0, 0.3, 1.6449, 10.0):
            lo, mid, hi = oracle.dense_intervals(c, oracle.Params(kappa=kap, normalize=False))
            assert np.all(lo >= 0) and np.all(hi <= 1.0 + 1e-15)
            assert np.all(lo <= mid * (1 + 1e-14)) and np.all(mid <= hi * (1 + 1e-14))
            assert np.all(lo.sum(1) <= 1 + 1e-12) and np.all(hi.sum(1) >= 1 - 1e-12)
            lo, mid, hi = oracle.dense_intervals(c, oracle.Params(kappa=kap, normalize=True))
            assert np.all(lo.sum(1) <= 0.99 * (1 + 1e-12))
            assert np.all(hi.sum(1) >= 1.01 * (1 - 1e-12))
            np.testing.assert_allclose(mid.sum(1), 1.0, rtol=1e-12)


def test_uniform_row_closed_form(oracle):
    """c = const, radius r: p^u = a/(V-1+a), p^l = b/(V-1+b), a = e^r, b = e^-r; Sigma = U = 0."""
    g = _golden()
    V = 16384
    c = np.full((1, V), 0.37, dtype=np.float32)
    P = oracle.Params(confidence=0.9, normalize=True)
    q = oracle.quantify(c, np.array([5]), P)
    r = math.sqrt(2) * sps.erfinv(0.9)
    a, b = math.exp(r), math.exp(-r)
    pu, pl = a / (V - 1 + a), b / (V - 1 + b)
    assert V * pl < 0.99 and V * pu > 1.01          # caps inactive for this row
    np.testing.assert_allclose(q["p_hi"], pu, rtol=1e-12)
    np.testing.assert_allclose(q["p_lo"], pl, rtol=1e-12)
    np.testing.assert_allclose(q["p_mid"], 1.0 / V, rtol=1e-12)
    np.testing.assert_allclose(q["omega"], V * (pu - pl), rtol=1e-12)
    assert abs(q["omega"][0] - g["omega_uniform_V16384_conf0.9"]) < 1e-6
    assert q["sigma"][0] < 1e-12 and q["score"][0] < 1e-12
    assert q["flags"][0] == 0


def test_one_hot_row_closed_form(oracle):
    """One logit far above the rest.  Raw: Omega -> 0 (local-certainty proposition).
    With the caps: delta = 0.02 on that token only, so Omega = 0.02 and
    U = 0.02^2 sqrt(V-1)/V, the equality case of the Sigma <= sqrt(n-1)/n Omega claim."""
    g = _golden()
    V = 16384
    c = np.zeros((1, V), dtype=np.float32)
    c[0, 77] = 80.0
    raw = oracle.quantify(c, np.array([77]), oracle.Params(confidence=0.9, normalize=False))
    assert raw["omega"][0] < 1e-25 and raw["score"][0] < 1e-40
    np.testing.assert_allclose(raw["p_lo"], 1.0, rtol=1e-12)
    np.testing.assert_allclose(raw["p_hi"], 1.0, rtol=1e-12)
    q = oracle.quantify(c, np.array([77]), oracle.Params(confidence=0.9, normalize=True))
    np.testing.assert_allclose(q["omega"], 0.02, rtol=1e-9)
    np.testing.assert_allclose(q["score"], 0.02 ** 2 * math.sqrt(V - 1) / V, rtol=1e-9)
    assert abs(q["score"][0] - g["score_onehot_V16384"]) < 1e-10
    np.testing.assert_allclose(q["p_lo"], 0.99, rtol=1e-12)
    np.testing.assert_allclose(q["p_hi"], 1.01, rtol=1e-12)   # the caps may lift p^u above 1


def test_dominant_token_bounds_against_50_digit_arithmetic(oracle):
    """A token that holds all but 1e-13 of the mass, thousands of others each below an ulp of 1, and a radius
    with e^-r ~ 1e-7: the dominant token's lower bound is 1 / (1 + rest / e^-r) with rest = the sum over the
    OTHER tokens, as the defining equations of the validity appendix have it.  Evaluated here with Python's
    decimal module at 50 digits straight from those equations; a partition sum that has already absorbed the
    dominant term cannot give rest back by subtraction (off by tens of percent in double)."""
    from decimal import Decimal, getcontext
    getcontext().prec = 50
    rng = np.random.default_rng(44)
    V = 6000
    c = (rng.standard_normal((1, V)) * 1.5).astype(np.float32)
    c[0, 1234] = 42.25
    r = 15.5
    P = oracle.Params(kappa=r, radius_max=16.0, normalize=False)
    lo, mid, hi = oracle.dense_intervals(c, P)
    cs = [Decimal(float(v)) for v in c[0]]
    m = max(cs)
    es = [(v - m).exp() for v in cs]
    a, b = Decimal(r).exp(), (-Decimal(r)).exp()
    for i in (1234, 0, 17):
        rest = sum(e for k, e in enumerate(es) if k != i)
        pl = es[i] * b / (rest + es[i] * b)
        pu = es[i] * a / (rest + es[i] * a)
        # compare the distances from 1 (dominant token) or the values themselves (the others)
        if i == 1234:
            assert abs(Decimal(1) - Decimal(float(lo[0, i])) - (1 - pl)) < Decimal(1e-9) * (1 - pl) + Decimal(2e-16)
            assert float(1 - pl) > 1e-8                              # the test has something to resolve
        else:
            assert abs(Decimal(float(lo[0, i])) - pl) < Decimal(1e-12) * pl
        assert abs(Decimal(float(hi[0, i])) - pu) < Decimal(1e-12) * pu + Decimal(2e-16)
    q = oracle.quantify(c, np.array([1234]), P)
    S = sum(es)
    width = sum(es[i] * a / (S - es[i] + es[i] * a) - es[i] * b / (S - es[i] + es[i] * b) for i in range(V))
    assert abs(Decimal(float(q["omega"][0])) - width) < Decimal(1e-9) * width


# ---- the score -----------------------------------------------------------------------------

def test_omega_sigma_score_against_numpy_on_the_dense_curves(oracle):
    """Omega = ||delta||_1, Sigma = population std of delta (numpy.std, ddof = 0), U = Omega Sigma.
    (Eq. uncertainty_score)"""
    rng = np.random.default_rng(7)
    c = _rows(rng, 8, 311, 2.0)
    for norm in (False, True):
        P = oracle.Params(confidence=0.9, normalize=norm)
        lo, mid, hi = oracle.dense_intervals(c, P)
        d = hi - lo
        q = oracle.quantify(c, None, P)
        np.testing.assert_allclose(q["omega"], d.sum(1), rtol=1e-12)
        np.testing.assert_allclose(q["sigma"], d.std(axis=1, ddof=0), rtol=1e-10)
        np.testing.assert_allclose(q["score"], d.sum(1) * d.std(axis=1), rtol=1e-10)
        # a sample (ddof = 1) standard deviation must be told apart
        assert np.all(np.abs(q["sigma"] - d.std(axis=1, ddof=1)) > 1e-6 * q["sigma"])
        # reported token defaults to the lowest-index argmax
        am = c.argmax(1)
        np.testing.assert_allclose(q["p_mid"], mid[np.arange(8), am], rtol=1e-13)
        np.testing.assert_allclose(q["p_lo"], lo[np.arange(8), am], rtol=1e-13)
        np.testing.assert_allclose(q["p_hi"], hi[np.arange(8), am], rtol=1e-13)


def test_appendix_bounds_and_rewrites(oracle):
    """Sigma <= sqrt(n-1)/n Omega; U <= sum(delta^2)/2; U = n mu^2 CV; U(alpha delta) = alpha^2 U."""
    rng = np.random.default_rng(8)
    for V, scale in ((16, 1.0), (500, 3.0), (4096, 0.5)):
        c = _rows(rng, 10, V, scale)
        P = oracle.Params(confidence=0.95, normalize=True)
        q = oracle.quantify(c, None, P)
        lo, _, hi = oracle.dense_intervals(c, P)
        d = hi - lo
        assert np.all(q["score"] >= 0)
        assert np.all(q["sigma"] <= math.sqrt(V - 1) / V * q["omega"] * (1 + 1e-12))
        assert np.all(q["score"] <= 0.5 * (d ** 2).sum(1) * (1 + 1e-12))
        mu = q["omega"] / V
        np.testing.assert_allclose(q["score"], V * mu ** 2 * (q["sigma"] / mu), rtol=1e-12)
    # scaling claim: with r = 0 and the caps on, delta = (hi_cap - lo_cap) p, so widening the
    # caps from (0.99, 1.01) to (0.98, 1.02) doubles delta and must quadruple U.
    c = _rows(rng, 5, 128, 2.0)
    u1 = oracle.quantify(c, None, oracle.Params(kappa=0.0, lower_cap=0.99, upper_cap=1.01))["score"]
    u2 = oracle.quantify(c, None, oracle.Params(kappa=0.0, lower_cap=0.98, upper_cap=1.02))["score"]
    np.testing.assert_allclose(u2, 4.0 * u1, rtol=1e-9)


def test_feasible_set_diameter(oracle):
    """||p - q||_1 <= Omega for distributions inside the interval box (diameter proposition)."""
    rng = np.random.default_rng(9)
    V = 12
    c = _rows(rng, 1, V, 1.5)
    lo, mid, hi = oracle.dense_intervals(c, oracle.Params(kappa=0.8, normalize=False))
    lo, mid, hi = lo[0], mid[0], hi[0]
    omega = oracle.quantify(c, None, oracle.Params(kappa=0.8, normalize=False))["omega"][0]
    pts = []
    for _ in range(200):
        p = mid.copy()
        for _ in range(30):     # move mass between random pairs while staying inside the box
            i, j = rng.choice(V, 2, replace=False)
            room = min(hi[i] - p[i], p[j] - lo[j])
            step = rng.random() * room
            p[i] += step; p[j] -= step
        assert abs(p.sum() - 1) < 1e-12 and np.all(p >= lo - 1e-15) and np.all(p <= hi + 1e-15)
        pts.append(p)
    pts = np.array(pts)
    diam = np.abs(pts[:, None, :] - pts[None, :, :]).sum(-1).max()
    assert 0 < diam <= omega


def test_width_identity_for_a_constant_radius(oracle):
    """delta_i = x(1-x)(a-b) / [(1+(a-1)x)(1-(1-b)x)], x = p_mid,i, a = e^r, b = e^-r."""
    rng = np.random.default_rng(10)
    c = _rows(rng, 4, 200, 3.0)
    r = 1.1
    lo, mid, hi = oracle.dense_intervals(c, oracle.Params(kappa=r, normalize=False))
    a, b = math.exp(r), math.exp(-r)
    x = mid
    ident = x * (1 - x) * (a - b) / ((1 + (a - 1) * x) * (1 - (1 - b) * x))
    np.testing.assert_allclose(hi - lo, ident, rtol=1e-11, atol=1e-300)


def test_intervals_are_nested_and_monotone_in_the_confidence(oracle):
    """Raw InterFuse: gamma1 < gamma2 gives [p^l, p^u](gamma1) inside [p^l, p^u](gamma2); Omega grows."""
    rng = np.random.default_rng(11)
    c = _rows(rng, 6, 300, 2.0)
    prev = None
    for gam in (0.5, 0.8, 0.9, 0.95, 0.99):
        P = oracle.Params(confidence=gam, normalize=False)
        lo, _, hi = oracle.dense_intervals(c, P)
        om = oracle.quantify(c, None, P)["omega"]
        if prev is not None:
            assert np.all(lo <= prev[0]) and np.all(hi >= prev[1]) and np.all(om > prev[2])
        prev = (lo, hi, om)


def test_total_ambiguity_is_maximal_at_the_uniform_row(oracle):
    """With one radius for all tokens the width is a concave function of p_mid, so Omega is
    Schur-concave and the uniform row maximises it (U itself is zero there by design)."""
    rng = np.random.default_rng(12)
    V = 64
    P = oracle.Params(confidence=0.9, normalize=False)
    uni = oracle.quantify(np.zeros((1, V), np.float32), None, P)["omega"][0]
    c = np.concatenate([_rows(rng, 100, V, s) for s in (0.05, 0.5, 2.0)])
    om = oracle.quantify(c, None, P)["omega"]
    assert np.all(om < uni)
    assert om[:100].max() > 0.99 * uni     # nearly flat rows come close


def test_threshold_polarity_and_equality(oracle):
    """Algorithm 1: accept locally iff U <= tau; the flag marks the other branch."""
    rng = np.random.default_rng(13)
    c = _rows(rng, 6, 100, 2.0)
    U = oracle.quantify(c, None, oracle.Params(tau=0.0))["score"]
    for n in range(6):
        row = c[n:n + 1]
        assert oracle.quantify(row, None, oracle.Params(tau=float(U[n])))["flags"][0] == 0
        assert oracle.quantify(row, None, oracle.Params(tau=float(np.nextafter(U[n], 0))))["flags"][0] == 1
        assert oracle.quantify(row, None, oracle.Params(tau=float(np.nextafter(U[n], 1))))["flags"][0] == 0


# ---- input handling ------------------------------------------------------------------------

def test_bf16_rows_are_widened_exactly_and_stride_padding_is_ignored(oracle):
    import torch
    rng = np.random.default_rng(14)
    V, stride = 50, 56
    c32 = _rows(rng, 3, stride, 2.0)
    cb = torch.from_numpy(c32).to(torch.bfloat16)
    widened = cb.to(torch.float32).numpy()
    P = oracle.Params(confidence=0.9)
    a = oracle.quantify(cb, None, P, vocab=V)
    b = oracle.quantify(np.ascontiguousarray(widened[:, :V]), None, P)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])
    poisoned = widened.copy()
    poisoned[:, V:] = 1e30
    d = oracle.quantify(poisoned, None, P, vocab=V)
    for k in a:
        np.testing.assert_array_equal(a[k], d[k])


def test_masked_tokens_have_zero_probability_and_zero_width(oracle):
    """A -inf logit is a masked token: e = 0, p^l = p_mid = p^u = 0; the other tokens are unchanged."""
    rng = np.random.default_rng(15)
    c = _rows(rng, 2, 40, 2.0)
    keep = np.ones(40, bool); keep[[3, 17, 39]] = False
    cm = c.copy(); cm[:, ~keep] = -np.inf
    P = oracle.Params(confidence=0.9, normalize=False)
    lo, mid, hi = oracle.dense_intervals(cm, P)
    lo2, mid2, hi2 = oracle.dense_intervals(np.ascontiguousarray(c[:, keep]), P)
    assert np.all(lo[:, ~keep] == 0) and np.all(mid[:, ~keep] == 0) and np.all(hi[:, ~keep] == 0)
    np.testing.assert_allclose(lo[:, keep], lo2, rtol=1e-14)
    np.testing.assert_allclose(hi[:, keep], hi2, rtol=1e-14)
    q = oracle.quantify(cm, None, P)
    d = hi - lo
    np.testing.assert_allclose(q["sigma"], d.std(axis=1), rtol=1e-12)   # masked tokens still count in V


# ---- verification --------------------------------------------------------------------------

def _verify_grid(oracle, c_row, t_row, x, ua, ur, K=1):
    n = len(ua)
    c = np.repeat(c_row[None, :], n, 0).astype(np.float32)
    t = np.repeat(t_row[None, :], n, 0).astype(np.float32)
    return oracle.verify(c, t, np.full(n, x), np.asarray(ua, np.float32), np.asarray(ur, np.float32),
                         oracle.Params(window=K))


@pytest.mark.parametrize("V", [2, 3, 8])
def test_speculative_sampling_law_by_enumeration(oracle, V):
    """Brute force on a tiny vocabulary: integrating the accept test over u_accept and the residual
    draw over u_resample, the emitted token is distributed exactly as the target q:
      sum_x p_x [ min(1, q_x/p_x) 1[x=j] + (1 - min(1, q_x/p_x)) res_j / R ] = q_j,
    and the set of u_resample mapped to token j is the interval [C_{j-1}/R, C_j/R)."""
    rng = np.random.default_rng(100 + V)
    G = 1 << 12
    grid = (np.arange(G) + 0.5) / G
    for trial in range(3):
        c = (rng.standard_normal(V) * 1.5).astype(np.float32)
        t = (c + rng.standard_normal(V)).astype(np.float32)
        p = sps.softmax(c.astype(np.float64)); q = sps.softmax(t.astype(np.float64))
        res = np.maximum(q - p, 0); R = res.sum()
        out = np.zeros(V)
        for x in range(V):
            # measure of accepted u_accept
            acc = _verify_grid(oracle, c, t, x, grid, np.zeros(G))["accept"].mean()
            beta = min(1.0, q[x] / p[x])
            assert abs(acc - beta) <= 1.0 / G
            out[x] += p[x] * beta
            if beta < 1.0:
                # always rejected at u_accept -> 1; distribution of the residual draw
                v = _verify_grid(oracle, c, t, x, np.full(G, 1 - 2.0 ** -24), grid)
                assert not v["accept"].any()
                freq = np.bincount(v["row_id"], minlength=V) / G
                assert np.all(np.abs(freq - res / R) <= 2.0 / G)
                out += p[x] * (1 - beta) * freq
                # interval end points: just below / above each C_j / R
                cdf = np.cumsum(res) / R
                for j in range(V):
                    if res[j] / R < 1e-3:
                        continue
                    lo_u = (cdf[j - 1] if j else 0.0) + 1e-5
                    hi_u = cdf[j] - 1e-5
                    vv = _verify_grid(oracle, c, t, x, [1 - 2.0 ** -24] * 2, [lo_u, hi_u])
                    assert list(vv["row_id"]) == [j, j]
        np.testing.assert_allclose(out, q, atol=3.0 / G)


def test_accept_test_takes_target_over_draft(oracle):
    """A token the target likes less than the draft is rejected with probability 1 - q_x/p_x, one it
    likes more is always accepted (swapping the two distributions would invert this)."""
    c = np.array([2.0, 0.0, 0.0, 0.0], np.float32)
    t = np.array([0.0, 2.0, 0.0, 0.0], np.float32)
    p = sps.softmax(c.astype(np.float64)); q = sps.softmax(t.astype(np.float64))
    ua = np.array([0.0, 0.1, 0.5, 0.9, 0.999], np.float32)
    v0 = _verify_grid(oracle, c, t, 0, ua, np.zeros(5))
    assert list(v0["accept"]) == [int(u < q[0] / p[0]) for u in ua]
    np.testing.assert_allclose(v0["log_ratio"], math.log(q[0] / p[0]), rtol=1e-12)
    v1 = _verify_grid(oracle, c, t, 1, ua, np.zeros(5))
    assert v1["accept"].all() and np.all(v1["row_id"] == -1)
    # the only token with positive residual mass is token 1
    assert np.all(v0["row_id"][v0["accept"] == 0] == 1)


def test_identical_rows_always_accept(oracle):
    rng = np.random.default_rng(16)
    N, V, K = 37, 129, 8
    c = _rows(rng, N, V, 3.0)
    ua = rng.random(N).astype(np.float32)
    ua[:3] = [0.0, 1 - 2.0 ** -24, 0.5]
    v = oracle.verify(c, c.copy(), rng.integers(0, V, N), ua, rng.random(N).astype(np.float32),
                      oracle.Params(window=K))
    assert v["accept"].all() and np.all(v["row_id"] == -1)
    W = (N + K - 1) // K
    assert list(v["accept_len"]) == [K] * (W - 1) + [N - K * (W - 1)]
    assert np.all(v["resampled_id"] == -1)


def test_window_outputs_on_a_hand_built_pattern(oracle):
    """accept_len = leading accepted rows of each window of K; resampled id = draw of the first
    rejected row; a fully accepted window reports -1; the last window may be ragged."""
    V, K = 4, 4
    c_rej = np.array([9.0, 0, 0, 0], np.float32)      # drafted token 0, target hates it
    t_rej = np.array([-9.0, 5.0, 0, 0], np.float32)   # residual mass almost all on token 1
    c_acc = np.array([0.0, 1, 2, 3], np.float32)
    pattern = [1, 1, 0, 1,   0, 0, 1, 1,   1, 1, 1, 1,   1, 0]    # 1 = accepted; N = 14, W = 4
    N = len(pattern)
    c = np.stack([c_acc if a else c_rej for a in pattern])
    t = np.stack([c_acc if a else t_rej for a in pattern])
    ids = np.zeros(N, np.int64)
    ua = np.full(N, 0.5, np.float32)
    ur = np.full(N, 0.5, np.float32)
    ur[4] = 1 - 2.0 ** -24     # the tail of the residual: the last token with positive mass
    v = oracle.verify(c, t, ids, ua, ur, oracle.Params(window=K))
    assert list(v["accept"]) == pattern
    assert list(v["accept_len"]) == [2, 0, 4, 1]
    q = sps.softmax(t_rej.astype(np.float64)); p = sps.softmax(c_rej.astype(np.float64))
    res = np.maximum(q - p, 0)
    tail = int(np.nonzero(np.cumsum(res) > (1 - 2.0 ** -24) * res.sum())[0][0])
    assert list(v["resampled_id"]) == [1, tail, -1, 1]
    assert [int(i) for i in v["row_id"]] == [-1, -1, 1, -1, tail, 1, -1, -1, -1, -1, -1, -1, -1, 1]


def test_residual_cdf_and_margin_diagnostics(oracle):
    rng = np.random.default_rng(17)
    V = 60
    c = _rows(rng, 4, V, 2.0)
    t = (c + rng.standard_normal(c.shape)).astype(np.float32)
    P = oracle.Params(window=2)
    p = sps.softmax(c.astype(np.float64), axis=1); q = sps.softmax(t.astype(np.float64), axis=1)
    for row in range(4):
        cdf, R = oracle.residual_cdf(c, t, row, P)
        ref = np.cumsum(np.maximum(q[row] - p[row], 0))
        np.testing.assert_allclose(cdf, ref, rtol=1e-11, atol=1e-16)
        assert abs(R - ref[-1]) < 1e-14
        # total residual mass equals the total-variation distance
        assert abs(R - 0.5 * np.abs(p[row] - q[row]).sum()) < 1e-13
    ids = p.argmax(1)      # over-drafted tokens are likely rejected at u -> 1
    v = oracle.verify(c, t, ids, np.full(4, 1 - 2.0 ** -24, np.float32), np.full(4, 0.3, np.float32), P)
    for row in range(4):
        if not v["accept"][row]:
            cdf, R = oracle.residual_cdf(c, t, row, P)
            j = v["row_id"][row]
            T = np.float64(np.float32(0.3)) * R
            assert cdf[j] > T and (j == 0 or cdf[j - 1] <= T)
            m = min(abs(cdf[j] - T), abs((cdf[j - 1] if j else 0.0) - T)) / R
            assert abs(v["res_margin"][row] - m) < 1e-12


def test_acceptance_rate_for_gaussian_target_noise(oracle):
    """Statistical sanity (not exact): target = draft + N(0, sigma^2) on a large flat vocabulary gives
    E[min(1, q/p)] = 1 - TV ~ 2 Phi(-sigma/2)."""
    rng = np.random.default_rng(18)
    N, V, sigma = 400, 4096, 0.5
    c = _rows(rng, N, V, 1.0)
    t = (c + sigma * rng.standard_normal(c.shape)).astype(np.float32)
    p = sps.softmax(c.astype(np.float64), axis=1)
    ids = np.array([rng.choice(V, p=p[n]) for n in range(N)])
    v = oracle.verify(c, t, ids, rng.random(N).astype(np.float32), rng.random(N).astype(np.float32),
                      oracle.Params(window=8))
    expect = 2 * spst.norm.cdf(-sigma / 2)
    assert abs(v["accept"].mean() - expect) < 4 * math.sqrt(expect * (1 - expect) / N) + 0.01


def test_threads_do_not_change_results(oracle):
    rng = np.random.default_rng(19)
    c = _rows(rng, 33, 257, 2.0)
    t = (c + 0.5 * rng.standard_normal(c.shape)).astype(np.float32)
    ids = rng.integers(0, 257, 33)
    ua, ur = rng.random(33).astype(np.float32), rng.random(33).astype(np.float32)
    P = oracle.Params(window=4)
    a = oracle.quantify(c, ids, P, threads=1); b = oracle.quantify(c, ids, P, threads=5)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])
    a = oracle.verify(c, t, ids, ua, ur, P, threads=1); b = oracle.verify(c, t, ids, ua, ur, P, threads=5)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


def test_empty_batch(oracle):
    c = np.zeros((0, 16), np.float32)
    q = oracle.quantify(c, np.zeros(0, np.int32), oracle.Params())
    assert all(v.shape == (0,) for v in q.values())
    v = oracle.verify(c, c, np.zeros(0, np.int32), np.zeros(0, np.float32), np.zeros(0, np.float32),
                      oracle.Params(window=4))
    assert v["accept_len"].shape == (0,)


# ---- tensor radius: r_i = min(kappa * Softplus(raw_i), radius_max)  (Sec. 3.2.3, Interval Head) ----------

def _raw_radius(rng, n, V, mu=0.0, sd=1.5):
    return (mu + sd * rng.standard_normal((n, V))).astype(np.float32)


def test_tensor_radius_two_token_vocabulary_is_the_logistic_sigmoid(oracle):
    """V = 2 with one radius per token: p^u_i = sigma(c_i - c_j + r_i), p^l_i = sigma(c_i - c_j - r_i), with
    r_i = kappa * ln(1 + e^raw_i) from numpy's log1p / exp (pins the Softplus and which token's radius is used)."""
    rng = np.random.default_rng(41)
    c = _rows(rng, 60, 2, 3.0)
    raw = _raw_radius(rng, 60, 2, sd=3.0)
    kap = 0.8
    r = kap * np.log1p(np.exp(raw.astype(np.float64)))
    lo, mid, hi = oracle.dense_intervals(c, oracle.Params(kappa=kap, radius_max=1e9, normalize=False), radius=raw)
    d = c[:, 0].astype(np.float64) - c[:, 1].astype(np.float64)
    np.testing.assert_allclose(mid[:, 0], sps.expit(d), rtol=1e-13)
    np.testing.assert_allclose(hi[:, 0], sps.expit(d + r[:, 0]), rtol=1e-12)
    np.testing.assert_allclose(lo[:, 0], sps.expit(d - r[:, 0]), rtol=1e-12)
    np.testing.assert_allclose(hi[:, 1], sps.expit(-d + r[:, 1]), rtol=1e-12)
    np.testing.assert_allclose(lo[:, 1], sps.expit(-d - r[:, 1]), rtol=1e-12)
    # the two tokens' radii differ, so using the other token's radius must be told apart
    assert np.max(np.abs(hi[:, 0] - sps.expit(d + r[:, 1]))) > 1e-3


def test_unit_scale_tensor_radius_is_rational_in_the_probability(oracle):
    """kappa = 1: e^Softplus(raw) = 1 + e^raw exactly, so with E_i = e^raw_i and x_i = softmax(c)_i the bounds are
    rational functions free of any logarithm: p^u_i = (1 + E_i) x_i / (1 + E_i x_i) and
    p^l_i = x_i / (1 + E_i (1 - x_i)) (Sec. 3.2.3: r = Softplus(raw); App. "Proof of Interval Validity" with
    a = e^r, b = 1/a).  Pins the Softplus against its closed form and the pairing of a and b."""
    rng = np.random.default_rng(43)
    c = _rows(rng, 40, 37, 2.0)
    raw = _raw_radius(rng, 40, 37, mu=-1.0, sd=3.0)
    lo, mid, hi = oracle.dense_intervals(c, oracle.Params(kappa=1.0, radius_max=1e9, normalize=False), radius=raw)
    x = sps.softmax(c.astype(np.float64), axis=1)
    E = np.exp(raw.astype(np.float64))
    np.testing.assert_allclose(mid, x, rtol=1e-13)
    np.testing.assert_allclose(hi, (1.0 + E) * x / (1.0 + E * x), rtol=1e-12)
    np.testing.assert_allclose(lo, x / (1.0 + E * (1.0 - x)), rtol=1e-12)
    # a scale other than 1 is told apart
    lo2, _, hi2 = oracle.dense_intervals(c, oracle.Params(kappa=1.1, radius_max=1e9, normalize=False), radius=raw)
    assert np.max(np.abs(hi2 - hi)) > 1e-3 and np.max(np.abs(lo2 - lo)) > 1e-4


def test_tensor_radius_equals_softmax_of_the_row_with_one_logit_shifted_by_its_own_radius(oracle):
    """Brute force over tokens with a library softmax; radii and rows differ from row to row (a wrong row
    stride or a transposed radius tensor fails)."""
    rng = np.random.default_rng(42)
    V, kap = 9, 1.0
    stride = 12
    c = np.full((4, stride), 1e30, dtype=np.float32)
    raw = np.full((4, stride), -1e30, dtype=np.float32)
    c[:, :V] = _rows(rng, 4, V, 2.5)
    raw[:, :V] = _raw_radius(rng, 4, V)
    lo, mid, hi = oracle.dense_intervals(c, oracle.Params(kappa=kap, normalize=False), vocab=V, radius=raw)
    for n in range(4):
        cn = c[n, :V].astype(np.float64)
        for i in range(V):
            r = kap * sps.log1p(math.exp(float(raw[n, i])))
            up = cn.copy(); up[i] += r
            dn = cn.copy(); dn[i] -= r
            assert abs(hi[n, i] - sps.softmax(up)[i]) < 1e-14
            assert abs(lo[n, i] - sps.softmax(dn)[i]) < 1e-14


def test_constant_raw_radius_reduces_to_the_scalar_mode(oracle):
    """raw = const: every token has r = kappa * Softplus(const), which is the scalar mode with that radius
    (already pinned above).  Softplus(0) = ln 2."""
    rng = np.random.default_rng(43)
    c = _rows(rng, 6, 257, 2.0)
    ids = rng.integers(0, 257, 6).astype(np.int32)
    for const, kap in ((0.0, 1.7), (1.25, 1.0), (-2.0, 3.0)):
        raw = np.full_like(c, const)
        r = kap * (math.log(2.0) if const == 0.0 else math.log1p(math.exp(const)))
        for norm in (False, True):
            t = oracle.quantify(c, ids, oracle.Params(kappa=kap, normalize=norm, tau=0.01), radius=raw)
            s = oracle.quantify(c, ids, oracle.Params(kappa=r, normalize=norm, tau=0.01))
            for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score"):
                np.testing.assert_allclose(t[k], s[k], rtol=1e-12, atol=1e-18)
            np.testing.assert_array_equal(t["flags"], s["flags"])


def test_tensor_radius_limits_and_clamp(oracle):
    """raw -> -inf: r -> 0 and the interval collapses onto the softmax; raw large: Softplus(raw) = raw without
    overflow, and the clamp turns every radius into radius_max (= scalar mode at radius_max)."""
    rng = np.random.default_rng(44)
    c = _rows(rng, 3, 40, 2.0)
    lo, mid, hi = oracle.dense_intervals(c, oracle.Params(kappa=1.0, normalize=False),
                                         radius=np.full_like(c, -800.0))
    np.testing.assert_allclose(lo, mid, rtol=1e-13)
    np.testing.assert_allclose(hi, mid, rtol=1e-13)
    np.testing.assert_allclose(mid, sps.softmax(c.astype(np.float64), axis=1), rtol=1e-13)
    big = oracle.dense_intervals(c, oracle.Params(kappa=1.0, radius_max=2.5, normalize=False),
                                 radius=np.full_like(c, 900.0))
    ref = oracle.dense_intervals(c, oracle.Params(kappa=2.5, normalize=False))
    for x, y in zip(big, ref):
        assert np.all(np.isfinite(x))
        np.testing.assert_array_equal(x, y)
    # unclamped large raw: Softplus(30) = 30 + ln(1 + e^-30)
    one = oracle.dense_intervals(c[:1, :2], oracle.Params(kappa=1.0, radius_max=1e9, normalize=False),
                                 radius=np.full((1, 2), 30.0, dtype=np.float32))
    d = float(c[0, 0]) - float(c[0, 1])
    assert abs(one[2][0, 0] - sps.expit(d + 30.0 + math.log1p(math.exp(-30.0)))) < 1e-15


def test_tensor_radius_scores_against_numpy_and_invariants(oracle):
    """Omega, Sigma, U from numpy on the dense curves; validity p^l <= p <= p^u, S_l <= 1 <= S_u (raw) and the
    0.99 / 1.01 caps (normalised); widths grow with kappa (raw InterFuse)."""
    rng = np.random.default_rng(45)
    c = _rows(rng, 8, 300, 2.0)
    raw = _raw_radius(rng, 8, 300)
    for norm in (False, True):
        P = oracle.Params(kappa=1.0, normalize=norm)
        lo, mid, hi = oracle.dense_intervals(c, P, radius=raw)
        d = hi - lo
        q = oracle.quantify(c, None, P, radius=raw)
        np.testing.assert_allclose(q["omega"], d.sum(1), rtol=1e-12)
        np.testing.assert_allclose(q["sigma"], d.std(axis=1, ddof=0), rtol=1e-10)
        np.testing.assert_allclose(q["score"], d.sum(1) * d.std(axis=1), rtol=1e-10)
        am = c.argmax(1)
        np.testing.assert_allclose(q["p_lo"], lo[np.arange(8), am], rtol=1e-13)
        np.testing.assert_allclose(q["p_hi"], hi[np.arange(8), am], rtol=1e-13)
        if norm:
            assert np.all(lo.sum(1) <= 0.99 + 1e-12) and np.all(hi.sum(1) >= 1.01 - 1e-12)
        else:
            assert np.all(lo <= mid * (1 + 1e-15)) and np.all(mid <= hi * (1 + 1e-15))
            assert np.all(lo.sum(1) <= 1.0) and np.all(hi.sum(1) >= 1.0)
    a = oracle.dense_intervals(c, oracle.Params(kappa=0.5, normalize=False), radius=raw)
    b = oracle.dense_intervals(c, oracle.Params(kappa=1.0, normalize=False), radius=raw)
    assert np.all(b[0] <= a[0]) and np.all(a[2] <= b[2])


def test_tensor_radius_bf16_is_widened_exactly(oracle):
    import torch
    rng = np.random.default_rng(46)
    c = torch.from_numpy(_rows(rng, 4, 64, 2.0)).to(torch.bfloat16)
    raw = torch.from_numpy(_raw_radius(rng, 4, 64)).to(torch.bfloat16)
    a = oracle.quantify(c, None, oracle.Params(kappa=1.0), radius=raw)
    b = oracle.quantify(c.float(), None, oracle.Params(kappa=1.0), radius=raw.float())
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


# ---- several heads: Voting and Ensemble (Sec. 4, ablation on the Inter-Head) ------------------------------

def _heads(rng, H, n, V, scale=2.0):
    base = _rows(rng, n, V, scale)
    return np.stack([base + 0.5 * _rows(rng, n, V, 1.0) for _ in range(H)]).astype(np.float32)


def test_ensemble_is_numpy_mean_of_the_heads_dense_curves(oracle):
    """Ensemble: token-wise mean of the per-head curves (each from the already pinned single-head path, computed
    here with numpy), then Omega = sum, Sigma = numpy std (ddof 0), U, flag.  Heads differ and one head has a
    radius tensor of its own."""
    rng = np.random.default_rng(51)
    H, n, V = 3, 6, 211
    c = _heads(rng, H, n, V)
    raw = np.stack([_raw_radius(rng, n, V) for _ in range(H)])
    ids = rng.integers(0, V, n).astype(np.int32)
    for radius, P in ((None, oracle.Params(confidence=0.9, tau=0.02)), (raw, oracle.Params(kappa=1.0, tau=0.02))):
        curves = [oracle.dense_intervals(c[h], P, radius=None if radius is None else radius[h]) for h in range(H)]
        lo = np.mean([x[0] for x in curves], axis=0)
        mid = np.mean([x[1] for x in curves], axis=0)
        hi = np.mean([x[2] for x in curves], axis=0)
        d = hi - lo
        q = oracle.quantify_multihead(c, ids, P, oracle.ENSEMBLE, radius_heads=radius)
        np.testing.assert_allclose(q["omega"], d.sum(1), rtol=1e-12)
        np.testing.assert_allclose(q["sigma"], d.std(axis=1), rtol=1e-10)
        np.testing.assert_allclose(q["score"], d.sum(1) * d.std(axis=1), rtol=1e-10)
        np.testing.assert_array_equal(q["flags"], (q["score"] > P.tau).astype(np.uint8))
        r = np.arange(n)
        np.testing.assert_allclose(q["p_lo"], lo[r, ids], rtol=1e-13)
        np.testing.assert_allclose(q["p_mid"], mid[r, ids], rtol=1e-13)
        np.testing.assert_allclose(q["p_hi"], hi[r, ids], rtol=1e-13)
        # averaging keeps the caps: sum of lower bounds <= 0.99, of upper bounds >= 1.01; centres sum to one
        assert np.all(lo.sum(1) <= 0.99 + 1e-12) and np.all(hi.sum(1) >= 1.01 - 1e-12)
        np.testing.assert_allclose(mid.sum(1), 1.0, rtol=1e-12)
        # no ids: the arg-max of the averaged centre distribution
        qa = oracle.quantify_multihead(c, None, P, oracle.ENSEMBLE, radius_heads=radius)
        np.testing.assert_allclose(qa["p_mid"], mid.max(1), rtol=1e-13)
    # the ensemble of different heads is not the score of any single head, nor the mean of the heads' scores
    P = oracle.Params(confidence=0.9)
    q = oracle.quantify_multihead(c, ids, P, oracle.ENSEMBLE)
    singles = np.stack([oracle.quantify(c[h], ids, P)["score"] for h in range(H)])
    assert np.all(np.abs(q["score"] - singles.mean(0)) > 1e-9)


def test_ensemble_of_one_or_identical_heads_is_the_single_head(oracle):
    rng = np.random.default_rng(52)
    c = _rows(rng, 5, 97, 2.0)
    ids = rng.integers(0, 97, 5).astype(np.int32)
    P = oracle.Params(confidence=0.9, tau=0.01)
    s = oracle.quantify(c, ids, P)
    for H in (1, 4):
        q = oracle.quantify_multihead(np.stack([c] * H), ids, P, oracle.ENSEMBLE)
        for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score"):
            np.testing.assert_allclose(q[k], s[k], rtol=1e-12, atol=1e-18)
        np.testing.assert_array_equal(q["flags"], s["flags"])


def test_voting_is_the_strict_majority_of_the_heads_flags(oracle):
    """Voting: every head's outputs equal the single-head quantifier on that head; the vote is 2 * votes > H
    (a tie of an even number of heads does not flag); the order of the heads does not matter."""
    rng = np.random.default_rng(53)
    n, V = 64, 129
    for H in (1, 2, 3, 5):
        c = _heads(rng, H, n, V, scale=1.5)
        ids = rng.integers(0, V, n).astype(np.int32)
        med = float(np.median(oracle.quantify(c[0], ids, oracle.Params(confidence=0.9))["score"]))
        P = oracle.Params(confidence=0.9, tau=med)
        q = oracle.quantify_multihead(c, ids, P, oracle.VOTING)
        votes = np.zeros(n, dtype=int)
        for h in range(H):
            s = oracle.quantify(c[h], ids, P)
            for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score"):
                np.testing.assert_array_equal(q[k][h], s[k])
            np.testing.assert_array_equal(q["head_flags"][h], s["flags"])
            votes += s["flags"]
        np.testing.assert_array_equal(q["flags"], (2 * votes > H).astype(np.uint8))
        if H > 1:
            assert 0 < q["flags"].sum() < n                      # both outcomes occur
            p = oracle.quantify_multihead(c[::-1].copy(), ids, P, oracle.VOTING)
            np.testing.assert_array_equal(p["flags"], q["flags"])
        if H == 2:
            assert np.any(votes == 1) and not np.any(q["flags"][votes == 1])


def test_multihead_head_stride_and_bf16(oracle):
    import torch
    rng = np.random.default_rng(54)
    c = torch.from_numpy(_heads(rng, 2, 4, 64)).to(torch.bfloat16)
    ids = np.array([1, 5, 9, 63], dtype=np.int32)
    P = oracle.Params(confidence=0.9)
    a = oracle.quantify_multihead(c, ids, P, oracle.ENSEMBLE)
    b = oracle.quantify_multihead(c.float(), ids, P, oracle.ENSEMBLE)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


# ---- Inter-DRO loss, forward (Sec. 3.2.3: anchor, DRO and alignment equations) -----------------------------

def _dro_inputs(rng, n, V, scale=2.0, noise=0.6):
    c = _rows(rng, n, V, scale)
    t = (c + noise * rng.standard_normal((n, V))).astype(np.float32)
    raw = _raw_radius(rng, n, V)
    return c, raw, t


def test_interdro_terms_against_scipy(oracle):
    """Per-row terms from library routines: p = scipy softmax of c, c + r, c - r; L1 by numpy; CE = H(p_cloud) +
    KL(p_cloud || p) with scipy.stats.entropy; KL by scipy.special.rel_entr.  r = kappa * log1p(exp(raw)) by numpy."""
    rng = np.random.default_rng(61)
    n, V, kap = 7, 193, 1.0
    c, raw, t = _dro_inputs(rng, n, V)
    q = oracle.interdro_loss(c, raw, t, oracle.Params(kappa=kap), 0.7, 1.3, 0.4, 2.0)
    c64, t64 = c.astype(np.float64), t.astype(np.float64)
    r = kap * np.log1p(np.exp(raw.astype(np.float64)))
    pc = sps.softmax(t64, axis=1)
    ps = {"mid": sps.softmax(c64, axis=1), "up": sps.softmax(c64 + r, axis=1), "lo": sps.softmax(c64 - r, axis=1)}
    for k, p in ps.items():
        np.testing.assert_allclose(q[f"l1_{k}"], np.abs(p - pc).sum(1), rtol=1e-12)
        ce = np.array([spst.entropy(pc[i]) + spst.entropy(pc[i], p[i]) for i in range(n)])
        np.testing.assert_allclose(q[f"ce_{k}"], ce, rtol=1e-12)
    np.testing.assert_allclose(q["kl"], sps.rel_entr(pc, ps["mid"]).sum(1), rtol=1e-11, atol=1e-15)
    # the three distributions differ: shifting by +r is not shifting by -r
    assert np.all(np.abs(q["ce_up"] - q["ce_lo"]) > 1e-6)
    # Gibbs and Pinsker
    H = np.array([spst.entropy(pc[i]) for i in range(n)])
    assert np.all(q["ce_mid"] >= H - 1e-12) and np.all(q["kl"] >= -1e-15)
    assert np.all(q["l1_mid"] ** 2 <= 2 * q["kl"] + 1e-12)


def test_interdro_batch_weights_and_total(oracle):
    """w = scipy softmax of alpha * CE(p_lo) over the batch; DRO = sum w CE; anchor / alignment terms are batch
    means with the lambdas; total is their sum.  alpha = 0 gives uniform weights, a large alpha the worst row."""
    rng = np.random.default_rng(62)
    n, V = 33, 101
    c, raw, t = _dro_inputs(rng, n, V)
    lv, lp, lb, alpha = 0.5, 2.0, 0.25, 3.0
    q = oracle.interdro_loss(c, raw, t, oracle.Params(kappa=1.0), lv, lp, lb, alpha)
    w = sps.softmax(alpha * q["ce_lo"])
    np.testing.assert_allclose(q["weights"], w, rtol=1e-12)
    np.testing.assert_allclose(q["dro"], float(np.dot(w, q["ce_lo"])), rtol=1e-12)
    centre = np.mean(lv * q["l1_mid"] + lp * q["ce_mid"] + lb * q["kl"])
    upper = np.mean(lv * q["l1_up"] + lp * q["ce_up"])
    lower = np.mean(lv * q["l1_lo"] + lp * q["ce_lo"])
    np.testing.assert_allclose([q["center"], q["upper"], q["lower"]], [centre, upper, lower], rtol=1e-12)
    np.testing.assert_allclose(q["total"], centre + upper + lower + q["dro"], rtol=1e-12)
    q0 = oracle.interdro_loss(c, raw, t, oracle.Params(kappa=1.0), lv, lp, lb, 0.0)
    np.testing.assert_allclose(q0["weights"], 1.0 / n, rtol=1e-12)
    np.testing.assert_allclose(q0["dro"], q["ce_lo"].mean(), rtol=1e-12)
    qi = oracle.interdro_loss(c, raw, t, oracle.Params(kappa=1.0), lv, lp, lb, 1e4)
    np.testing.assert_allclose(qi["dro"], q["ce_lo"].max(), rtol=1e-9)
    assert q0["dro"] < q["dro"] < qi["dro"]                      # harder rows weigh more as alpha grows


def test_interdro_special_cases(oracle):
    """cloud == centre and zero radius: every distance vanishes and CE is the entropy.  A scalar radius shifts
    every logit alike, so p_up = p_lo = p_mid.  V = 2: CE(p_mid) = softplus form of the two-class cross-entropy."""
    rng = np.random.default_rng(63)
    c = _rows(rng, 5, 64, 2.0)
    q = oracle.interdro_loss(c, np.full_like(c, -900.0), c, oracle.Params(kappa=1.0), 1.0, 1.0, 1.0, 1.0)
    H = np.array([spst.entropy(sps.softmax(c[i].astype(np.float64))) for i in range(5)])
    for k in ("l1_mid", "l1_up", "l1_lo", "kl"):
        np.testing.assert_allclose(q[k], 0.0, atol=1e-14)
    for k in ("ce_mid", "ce_up", "ce_lo"):
        np.testing.assert_allclose(q[k], H, rtol=1e-12)
    t = (c + rng.standard_normal(c.shape)).astype(np.float32)
    s = oracle.interdro_loss(c, None, t, oracle.Params(kappa=1.7), 1.0, 1.0, 1.0, 1.0)
    np.testing.assert_allclose(s["ce_up"], s["ce_mid"], rtol=1e-12)
    np.testing.assert_allclose(s["l1_lo"], s["l1_mid"], rtol=1e-12, atol=1e-16)
    c2 = _rows(rng, 9, 2, 2.0)
    t2 = _rows(rng, 9, 2, 2.0)
    b = oracle.interdro_loss(c2, None, t2, oracle.Params(kappa=0.0), 1.0, 1.0, 1.0, 0.0)
    d = c2[:, 0].astype(np.float64) - c2[:, 1]
    dt = t2[:, 0].astype(np.float64) - t2[:, 1]
    pc0 = sps.expit(dt)
    ce = pc0 * np.log1p(np.exp(-d)) + (1 - pc0) * np.log1p(np.exp(d))
    np.testing.assert_allclose(b["ce_mid"], ce, rtol=1e-12)
    np.testing.assert_allclose(b["l1_mid"], 2 * np.abs(sps.expit(d) - pc0), rtol=1e-12, atol=1e-16)


def test_interdro_masked_cloud_tokens_stride_and_bf16(oracle):
    import torch
    rng = np.random.default_rng(64)
    V, stride = 50, 56
    c = np.full((4, stride), 1e30, dtype=np.float32)
    t = np.full((4, stride), 1e30, dtype=np.float32)
    raw = np.full((4, stride), np.nan, dtype=np.float32)
    c[:, :V], raw[:, :V], t[:, :V] = _dro_inputs(rng, 4, V)
    t[:, 3] = -np.inf                                             # a token the cloud model rules out
    q = oracle.interdro_loss(c, raw, t, oracle.Params(kappa=1.0), 1.0, 1.0, 1.0, 1.0, vocab=V)
    assert all(np.all(np.isfinite(q[k])) for k in oracle.DRO_TERMS) and np.isfinite(q["total"])
    pc = sps.softmax(t[:, :V].astype(np.float64), axis=1)
    assert np.all(pc[:, 3] == 0.0)
    p = sps.softmax(c[:, :V].astype(np.float64), axis=1)
    keep = np.arange(V) != 3
    np.testing.assert_allclose(q["kl"], (pc[:, keep] * (np.log(pc[:, keep]) - np.log(p[:, keep]))).sum(1), rtol=1e-11)
    cb, rb, tb = (torch.from_numpy(x[:, :V].copy()).to(torch.bfloat16) for x in (c, np.nan_to_num(raw), t))
    a = oracle.interdro_loss(cb, rb, tb, oracle.Params(kappa=1.0), 1.0, 1.0, 1.0, 1.0)
    b = oracle.interdro_loss(cb.float(), rb.float(), tb.float(), oracle.Params(kappa=1.0), 1.0, 1.0, 1.0, 1.0)
    for k in oracle.DRO_TERMS:
        np.testing.assert_array_equal(a[k], b[k])
