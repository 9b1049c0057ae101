"""GPU parity of the Interval Head entry points (ciar_interhead_logits, ciar_interhead_quantify) against the fp64
oracle on identical bf16 operands.

Tolerances.  The contraction accumulates D bf16 x bf16 products (each exact in fp32) in fp32 on the matrix cores,
in an order the hardware fixes; against the fp64 sum that leaves at most D * 2^-24 * sum_k |h_k w_k| and, for
rounding errors of either sign, about 2^-24 * sum_k |h_k w_k|.  The logits are held to
|gpu - oracle| <= 1e-6 * sum_k |h_k w_k| + 2^-24 |oracle| (final rounding to fp32).
A logit error eps moves ln p_i by at most 2 eps and the radius by at most eps, so the quantifier's outputs are held
to RTOL = 1e-5 + 4 eps, with eps = 2^-24 * max sum_k |h_k w_k| of the case (the size of the accumulation error for
rounding errors of either sign; measured errors stay below a fifth of this RTOL), and a flag is exempt when the
oracle's score lies within 1e-6 + RTOL * U of tau.
"""
import numpy as np
import pytest
import torch

import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ciar():
    import paper_2603_25463_amd as m
    m.lib()
    assert torch.cuda.is_available()
    return m


def say(*a):
    print(*a, flush=True)


def _case(N, D, V, seed, with_bias=True, scale=2.0):
    """Hidden states ~ N(0, 1); weights ~ N(0, scale^2 / D) so that centre logits are N(0, scale^2); the radius
    half is shifted down (raw ~ N(-1, .)) as a trained head's small radii would be; one peaked token per row."""
    g = torch.Generator().manual_seed(0xC1A2_0400 + seed)
    h = torch.randn((N, D), generator=g).bfloat16()
    w = (torch.randn((2 * V, D), generator=g) * (scale / D ** 0.5)).bfloat16()
    b = None
    if with_bias:
        b = torch.randn(2 * V, generator=g) * 0.5
        b[V:] -= 1.0
        b[torch.randint(0, V, (1,), generator=g)] += 6.0
    ids = torch.randint(0, V, (N,), generator=g, dtype=torch.int32)
    return h, w, b, ids


def _logit_bound(h, w, ref):
    absum = h.double().abs() @ w.double().abs().T
    return 1e-6 * absum.numpy() + 2.0 ** -24 * np.abs(ref)


SHAPES = [  # N, D, V, row_stride
    (1, 64, 128, 128), (130, 64, 128, 128), (127, 192, 256, 260), (257, 128, 384, 384), (300, 1280, 1024, 1024),
    (128, 4096, 128, 128),
    (200, 64, 256, 256), (129, 128, 512, 516), (385, 192, 256, 256),     # the large tile with one, two and three k tiles
]


@pytest.mark.parametrize("N,D,V,stride", SHAPES)
def test_interhead_logits(ciar, oracle, N, D, V, stride):
    h, w, b, _ = _case(N, D, V, seed=N + D + V)
    say(f"[interhead logits] N={N} D={D} V={V} stride={stride}")
    out = (torch.full((N, stride), 7.0, device="cuda"), torch.full((N, stride), 7.0, device="cuda"))
    c, r = ciar.interhead_logits(h.cuda(), w.cuda(), b.cuda(), ciar.Params(), row_stride=stride, out=out)
    torch.cuda.synchronize()
    oc, orr = oracle.interhead_logits(h, w, b.numpy())
    both = np.concatenate([oc, orr], axis=1)
    bound = _logit_bound(h, w, both)
    for got, ref, bd, name in ((c, oc, bound[:, :V], "centre"), (r, orr, bound[:, V:], "radius")):
        g = got.cpu().numpy().astype(np.float64)
        err = np.abs(g[:, :V] - ref)
        assert np.all(err <= bd), (name, float((err / bd).max()), np.unravel_index(np.argmax(err / bd), err.shape))
        assert np.all(g[:, V:] == 7.0), f"{name}: padding between rows was written"


@pytest.mark.parametrize("seed", [int(__import__("os").environ.get("CIAR_RANDOM_FIRST", "0")) + k for k in range(int(__import__("os").environ.get("CIAR_RANDOM_CASES", "8")))])
def test_interhead_logits_random_shapes(ciar, oracle, seed):
    """Batch size, hidden width (1 to 20 k tiles), vocabulary (both tiles: multiples of 128 and of 256) and output stride
    drawn at random; small integer operands, so that every partial sum is exact in fp32 and the kernel must match the
    fp64 product bit for bit whatever the shape."""
    rng = np.random.default_rng(49000 + seed)
    N = int(rng.integers(1, 700))
    D = 64 * int(rng.integers(1, 21))
    V = 128 * int(rng.integers(1, 9))
    stride = V + 4 * int(rng.integers(0, 3))
    g = torch.Generator().manual_seed(49100 + seed)
    h = torch.randint(-3, 4, (N, D), generator=g).to(torch.bfloat16)
    w = torch.randint(-2, 3, (2 * V, D), generator=g).to(torch.bfloat16)
    b = torch.randint(-5, 6, (2 * V,), generator=g).to(torch.float32) if rng.integers(0, 2) else None
    say(f"[interhead random {seed}] N={N} D={D} V={V} stride={stride} bias={b is not None}")
    out = (torch.full((N, stride), 7.0, device="cuda"), torch.full((N, stride), 7.0, device="cuda"))
    c, r = ciar.interhead_logits(h.cuda(), w.cuda(), None if b is None else b.cuda(), ciar.Params(), row_stride=stride, out=out)
    torch.cuda.synchronize()
    oc, orr = oracle.interhead_logits(h, w, None if b is None else b.numpy())
    for got, ref, name in ((c, oc, "centre"), (r, orr, "radius")):
        gg = got.cpu().numpy().astype(np.float64)
        assert np.array_equal(gg[:, :V], ref), (name, np.unravel_index(np.argmax(np.abs(gg[:, :V] - ref)), ref.shape))
        assert np.all(gg[:, V:] == 7.0), f"{name}: padding between rows was written"


def test_interhead_logits_without_bias_and_exact_integers(ciar, oracle):
    """Small integer operands: every product and partial sum is exact in fp32, so the kernel must match bit for bit
    (any wrong lane, row or column mapping of the matrix instruction shows as a wrong integer)."""
    g = torch.Generator().manual_seed(77)
    N, D, V = 200, 128, 256
    h = torch.randint(-4, 5, (N, D), generator=g).bfloat16()
    w = torch.randint(-4, 5, (2 * V, D), generator=g).bfloat16()
    say(f"[interhead integers] N={N} D={D} V={V}")
    c, r = ciar.interhead_logits(h.cuda(), w.cuda(), None, ciar.Params())
    torch.cuda.synchronize()
    oc, orr = oracle.interhead_logits(h, w)
    assert np.array_equal(c.cpu().numpy().astype(np.float64), oc)
    assert np.array_equal(r.cpu().numpy().astype(np.float64), orr)


@pytest.mark.parametrize("N,D,V,stride", [(130, 64, 128, 128), (257, 256, 1024, 1024), (515, 1280, 4096, 4096),
                                          (64, 512, 16384, 16384)])
def test_interhead_quantify(ciar, oracle, N, D, V, stride):
    h, w, b, ids = _case(N, D, V, seed=7 * N + V)
    say(f"[interhead quantify] N={N} D={D} V={V} stride={stride}")
    oc, orr = oracle.interhead_logits(h, w, b.numpy())
    eps = 2.0 ** -24 * float((h.double().abs() @ w.double().abs().T).max())
    rtol = 1e-5 + 4 * eps
    # threshold at the oracle's median score: both flag values occur
    OP = oracle.Params(kappa=1.0, tau=0.3)
    ref = oracle.interhead_quantify(h, w, b.numpy(), ids.numpy(), OP)
    tau = float(np.float32(np.median(ref["score"])))
    ref["flags"] = (ref["score"] > tau).astype(np.uint8)
    P = ciar.Params(radius_scale=1.0, tau=tau)
    got = ciar.interhead_quantify(h.cuda(), w.cuda(), b.cuda(), ids.cuda(), P, row_stride=stride)
    torch.cuda.synchronize()
    worst = parity.check_floats(got, ref, rtol=rtol)
    say(f"    eps={eps:.2e} rtol={rtol:.2e} worst/bound={worst}")
    gf = got["flags"].cpu().numpy()
    diff = np.nonzero(gf != ref["flags"])[0]
    for i in diff:
        assert abs(ref["score"][i] - tau) < 1e-6 + rtol * ref["score"][i], (i, ref["score"][i], tau)
    assert len(diff) <= max(2, N // 50)
    assert 0 < int(ref["flags"].sum()) < N
    # the same call twice gives the same bits; without ids the arg-max token is reported
    again = ciar.interhead_quantify(h.cuda(), w.cuda(), b.cuda(), ids.cuda(), P, row_stride=stride)
    for k in got:
        assert torch.equal(got[k], again[k]), k


def test_interhead_quantify_at_the_benchmark_shape(ciar, oracle):
    """2048 positions, V = 16384, D = 1280 (the shape bench.py --interhead times, 256 x 256 tiles over the whole
    chip): the GPU runs every row, the oracle every eighth one."""
    N, D, V = 2048, 1280, 16384
    h, w, b, ids = _case(N, D, V, seed=2048)
    say(f"[interhead quantify, benchmark shape] N={N} D={D} V={V}")
    P = ciar.Params(radius_scale=1.0, tau=0.3)
    got = ciar.interhead_quantify(h.cuda(), w.cuda(), b.cuda(), ids.cuda(), P)
    torch.cuda.synchronize()
    rows = np.arange(0, N, 8)
    hs = h[rows].contiguous()
    eps = 2.0 ** -24 * float((hs.double().abs() @ w.double().abs().T).max())
    rtol = 1e-5 + 4 * eps
    ref = oracle.interhead_quantify(hs, w, b.numpy(), ids.numpy()[rows], oracle.Params(kappa=1.0, tau=0.3))
    sub = {k: v[torch.as_tensor(rows, device=v.device)] for k, v in got.items()}
    worst = parity.check_floats(sub, ref, rtol=rtol)
    say(f"    eps={eps:.2e} rtol={rtol:.2e} worst/bound={worst}")
    tau = float(np.float32(0.3))
    diff = np.nonzero(sub["flags"].cpu().numpy() != ref["flags"])[0]
    for i in diff:
        assert abs(ref["score"][i] - tau) < 1e-6 + rtol * ref["score"][i], (i, ref["score"][i])


def test_interhead_rejects_unsupported_shapes(ciar):
    h = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ciar.CiarError, match="CIAR_EUNSUPPORTED"):
        ciar.interhead_logits(h, torch.zeros((2 * 100, 64), dtype=torch.bfloat16, device="cuda"), None, ciar.Params(),
                              row_stride=100)
    with pytest.raises(ciar.CiarError, match="CIAR_EUNSUPPORTED"):
        ciar.interhead_logits(torch.zeros((4, 96), dtype=torch.bfloat16, device="cuda"),
                              torch.zeros((256, 96), dtype=torch.bfloat16, device="cuda"), None, ciar.Params())
    with pytest.raises(ciar.CiarError, match="CIAR_EWORKSPACE"):
        ciar.interhead_quantify(h, torch.zeros((256, 64), dtype=torch.bfloat16, device="cuda"), None, None,
                                ciar.Params(), workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    out = ciar.interhead_quantify(h[:0], torch.zeros((256, 64), dtype=torch.bfloat16, device="cuda"), None, None,
                                  ciar.Params())
    assert out["score"].numel() == 0
