"""CPU pins of the oracle's Interval Head (Sec. 3.2.1, "Interval Head Architecture": c_t = Linear_center(h_t),
r_t = Softplus(Linear_radius(h_t)), output dimension 2|V|): special cases with closed forms, a second
library's linear map, and reductions to functions that are pinned elsewhere."""
import numpy as np
import torch


def _bf16(a):
    return torch.as_tensor(np.asarray(a, dtype=np.float32)).bfloat16()


def _f64(t):
    return t.float().numpy().astype(np.float64)


def test_one_hot_hidden_state_selects_a_weight_column(oracle):
    """h = e_k: centre[n, j] = W[j, k] and raw[n, j] = W[V + j, k], exactly (a transposed operand or swapped
    halves of the head fail here)."""
    rng = np.random.default_rng(3)
    V, D = 5, 7
    w = _bf16(rng.normal(size=(2 * V, D)))
    for k in (0, 3, 6):
        h = torch.zeros((2, D)).bfloat16()
        h[:, k] = 1.0
        c, r = oracle.interhead_logits(h, w)
        assert np.array_equal(c, np.broadcast_to(_f64(w)[:V, k], (2, V)))
        assert np.array_equal(r, np.broadcast_to(_f64(w)[V:, k], (2, V)))


def test_zero_weights_leave_the_bias(oracle):
    rng = np.random.default_rng(4)
    V, D = 6, 8
    b = rng.normal(size=2 * V).astype(np.float32)
    c, r = oracle.interhead_logits(_bf16(rng.normal(size=(3, D))), torch.zeros((2 * V, D)).bfloat16(), b)
    assert np.array_equal(c, np.broadcast_to(b[:V].astype(np.float64), (3, V)))
    assert np.array_equal(r, np.broadcast_to(b[V:].astype(np.float64), (3, V)))


def test_matches_torch_linear_in_double(oracle):
    """A second library's routine for the same map: torch.nn.functional.linear on float64 tensors."""
    rng = np.random.default_rng(5)
    N, D, V = 9, 96, 40
    h, w = _bf16(rng.normal(size=(N, D))), _bf16(rng.normal(size=(2 * V, D)) / 8)
    b = rng.normal(size=2 * V).astype(np.float32)
    c, r = oracle.interhead_logits(h, w, b)
    ref = torch.nn.functional.linear(h.double(), w.double(), torch.as_tensor(b).double()).numpy()
    assert np.allclose(c, ref[:, :V], rtol=0, atol=1e-12)
    assert np.allclose(r, ref[:, V:], rtol=0, atol=1e-12)


def test_small_integers_are_exact_and_additive(oracle):
    """Integer-valued operands: every product and sum is exact, so the map is additive in h to the last bit
    and equals integer arithmetic."""
    rng = np.random.default_rng(6)
    N, D, V = 4, 16, 3
    h1, h2 = rng.integers(-8, 9, size=(N, D)), rng.integers(-8, 9, size=(N, D))
    w = rng.integers(-8, 9, size=(2 * V, D))
    c1, r1 = oracle.interhead_logits(_bf16(h1), _bf16(w))
    c2, r2 = oracle.interhead_logits(_bf16(h2), _bf16(w))
    c12, r12 = oracle.interhead_logits(_bf16(h1 + h2), _bf16(w))
    assert np.array_equal(c12, c1 + c2) and np.array_equal(r12, r1 + r2)
    exact = (h1[:, None, :] * w[None, :, :]).sum(-1)               # integer arithmetic
    assert np.array_equal(c1, exact[:, :V].astype(np.float64)) and np.array_equal(r1, exact[:, V:].astype(np.float64))


def test_constant_radius_head_is_the_scalar_mode(oracle):
    """Radius half with zero weights and a constant bias t: r = Softplus(t) for every token, so the head's
    quantifier equals the scalar-radius quantifier at kappa = ln(1 + e^t) on the centre logits."""
    rng = np.random.default_rng(7)
    N, D, V = 6, 32, 48
    t = 0.75
    w = _bf16(rng.normal(size=(2 * V, D)) / 4)
    w[V:] = 0
    b = np.concatenate([rng.normal(size=V), np.full(V, t)]).astype(np.float32)
    h = _bf16(rng.normal(size=(N, D)))
    ids = rng.integers(0, V, size=N).astype(np.int32)
    P = oracle.Params(kappa=1.0, tau=0.01)
    got = oracle.interhead_quantify(h, w, b, ids, P)
    centre, _ = oracle.interhead_logits(h, w, b)
    ref = oracle.quantify(centre, ids, oracle.Params(kappa=float(np.log1p(np.exp(np.float64(np.float32(t))))), tau=0.01))
    for k in ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score"):
        assert np.allclose(got[k], ref[k], rtol=1e-12, atol=1e-15), k
    assert np.array_equal(got["flags"], ref["flags"])


def test_double_logits_agree_with_their_float_roundings(oracle):
    """The fp64 logit input of the quantifier: logits that are exactly representable in float32 give
    bit-identical results through the float32 input."""
    rng = np.random.default_rng(8)
    c32 = rng.normal(size=(5, 64)).astype(np.float32)
    r32 = rng.normal(size=(5, 64)).astype(np.float32)
    ids = rng.integers(0, 64, size=5).astype(np.int32)
    P = oracle.Params(kappa=1.0, tau=0.01)
    a = oracle.quantify(c32, ids, P, radius=r32)
    b = oracle.quantify(c32.astype(np.float64), ids, P, radius=r32.astype(np.float64))
    for k in a:
        assert np.array_equal(a[k], b[k]), k
