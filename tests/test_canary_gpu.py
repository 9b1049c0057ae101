"""Guard words around every output and around the workspace of every entry point of the C ABI: a kernel that
writes one element before or after an array it was given (a ragged tail handled with a full vector store, a
window count rounded the wrong way, a workspace region carved too small) changes a guard.  Shapes are ragged in N,
K and V on purpose.  The values themselves are the parity tests' business."""
import ctypes

import pytest
import torch

pytestmark = pytest.mark.gpu

GUARD = 64                     # elements on either side of an array
CIAR_STATIC_MAX_ROWS = 32768   # include/ciar.h
F_KEYS = ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score")


class Guarded:
    """Tensors carved out of larger ones whose margins hold a pattern."""

    def __init__(self, dev):
        self.dev, self.items = dev, []

    def new(self, n, dtype, name):
        pattern = {torch.float32: -12345.5, torch.uint8: 0xA5, torch.int32: -0x5A5A5A5}[dtype]
        whole = torch.full((n + 2 * GUARD,), pattern, dtype=dtype, device=self.dev)
        self.items.append((name, whole, n, pattern))
        return whole[GUARD:GUARD + n]

    def check(self, what):
        torch.cuda.synchronize()
        for name, whole, n, pattern in self.items:
            lo, hi = whole[:GUARD], whole[GUARD + n:]
            assert bool((lo == pattern).all()), f"{what}: something wrote in front of {name}"
            assert bool((hi == pattern).all()), f"{what}: something wrote behind {name}"


def _rows(N, V, dtype, dev, seed, scale=2.0):
    per16 = 4 if dtype == torch.float32 else 8
    stride = (V + per16 - 1) // per16 * per16
    g = torch.Generator(device="cpu").manual_seed(seed)
    t = (torch.randn((max(N, 1), stride), generator=g) * scale).to(dtype).to(dev)
    return t[:N]


def _inputs(N, V, dtype, dev, seed):
    g = torch.Generator(device="cpu").manual_seed(seed + 1)
    c, t = _rows(N, V, dtype, dev, seed), _rows(N, V, dtype, dev, seed + 7, 2.5)
    if N:
        t[::3] = c[::3]                                       # a third of the rows agree: accepted rows and rejected rows
    ids = torch.randint(0, V, (N,), generator=g, dtype=torch.int32).to(dev)
    ua = torch.rand((N,), generator=g).to(dev)
    ur = torch.rand((N,), generator=g).to(dev)
    return c, t, ids, ua, ur


SHAPES = [  # N, V, K, dtype
    (1, 1, 1, torch.float32), (7, 37, 3, torch.float32), (129, 1000, 8, torch.float32), (300, 16384, 7, torch.float32),
    (1031, 4099, 255, torch.float32), (515, 16384, 300, torch.float32), (130, 32768, 8, torch.float32),
    (5, 29, 2, torch.bfloat16), (257, 16384, 8, torch.bfloat16), (100, 65536, 9, torch.bfloat16),
    (2053, 130, 5, torch.float32), (4100, 64, 16, torch.bfloat16),
]


@pytest.mark.parametrize("N,V,K,dtype", SHAPES)
@pytest.mark.parametrize("tensor_radius", [False, True])
def test_per_row_entry_points_stay_inside_their_arrays(N, V, K, dtype, tensor_radius):
    import paper_2603_25463_amd as ciar
    from paper_2603_25463_amd.binding import _check, _ptr, _stream
    L = ciar.lib()
    dev = torch.device("cuda:0")
    c, t, ids, ua, ur = _inputs(N, V, dtype, dev, 1000 + N)
    rad = _rows(N, V, dtype, dev, 99, 1.0) if tensor_radius else None
    P = ciar.Params(confidence=0.9, tau=0.01, window=K)
    cp = P.to_c(c, V)
    W = (N + K - 1) // K
    sp = _stream(None)
    print(f"canary: N={N} V={V} K={K} {dtype} tensor_radius={tensor_radius}", flush=True)

    def outputs(g):
        o = {k: g.new(N, torch.float32, k) for k in F_KEYS}
        o["flags"] = g.new(N, torch.uint8, "flags")
        o["accept"] = g.new(N, torch.uint8, "accept")
        o["row_id"] = g.new(N, torch.int32, "row_id")
        o["accept_len"] = g.new(W, torch.int32, "accept_len")
        o["resampled_id"] = g.new(W, torch.int32, "resampled_id")
        return o

    def workspace(g):
        nbytes = ciar.workspace_bytes(N, cp)
        return g.new(nbytes, torch.uint8, "workspace"), nbytes

    names = F_KEYS + ("flags", "accept", "row_id", "accept_len", "resampled_id")
    # the fused call with every output
    g = Guarded(dev); o = outputs(g); ws, nb = workspace(g)
    _check(L.ciar_quantify_verify(_ptr(c), _ptr(rad), _ptr(t), _ptr(ids), _ptr(ua), _ptr(ur), N, ctypes.byref(cp),
                                  *[_ptr(o[k]) for k in names], _ptr(ws), nb, sp))
    g.check("ciar_quantify_verify")
    # ... with the window outputs only (accept bits and draws go through the workspace)
    g = Guarded(dev); o = outputs(g); ws, nb = workspace(g)
    _check(L.ciar_quantify_verify(_ptr(c), _ptr(rad), _ptr(t), _ptr(ids), _ptr(ua), _ptr(ur), N, ctypes.byref(cp),
                                  None, None, None, None, None, _ptr(o["score"]), None, None, None, _ptr(o["accept_len"]),
                                  _ptr(o["resampled_id"]), _ptr(ws), nb, sp))
    g.check("ciar_quantify_verify (window outputs)")
    # the allocation-free variant
    if N <= CIAR_STATIC_MAX_ROWS:
        g = Guarded(dev); o = outputs(g)
        _check(L.ciar_quantify_verify_static(_ptr(c), _ptr(rad), _ptr(t), _ptr(ids), _ptr(ua), _ptr(ur), N, ctypes.byref(cp),
                                             *[_ptr(o[k]) for k in names], sp))
        g.check("ciar_quantify_verify_static")
    # quantify, with and without drafted ids
    for use_ids in (True, False):
        g = Guarded(dev); o = outputs(g); ws, nb = workspace(g)
        _check(L.ciar_quantify(_ptr(c), _ptr(rad), _ptr(ids) if use_ids else None, N, ctypes.byref(cp),
                               *[_ptr(o[k]) for k in F_KEYS], _ptr(o["flags"]), _ptr(ws), nb, sp))
        g.check(f"ciar_quantify (ids={use_ids})")
    # verify
    g = Guarded(dev); o = outputs(g); ws, nb = workspace(g)
    _check(L.ciar_verify(_ptr(c), _ptr(t), _ptr(ids), _ptr(ua), _ptr(ur), N, ctypes.byref(cp), _ptr(o["accept"]),
                         _ptr(o["row_id"]), _ptr(o["accept_len"]), _ptr(o["resampled_id"]), _ptr(ws), nb, sp))
    g.check("ciar_verify")
    acc, rid = o["accept"], o["row_id"]
    g = Guarded(dev); al = g.new(W, torch.int32, "accept_len"); rs = g.new(W, torch.int32, "resampled_id")
    _check(L.ciar_window_epilogue(_ptr(acc), _ptr(rid), N, ctypes.byref(cp), _ptr(al), _ptr(rs), sp))
    g.check("ciar_window_epilogue")
    # the loss and the plain read
    g = Guarded(dev)
    terms, wts, losses = g.new(7 * N, torch.float32, "row_terms"), g.new(N, torch.float32, "weights"), g.new(5, torch.float32, "losses")
    _check(L.ciar_interdro_loss(_ptr(c), _ptr(rad), _ptr(t), N, ctypes.byref(cp), 0.5, 0.1, 0.01, 0.9, _ptr(terms), _ptr(wts),
                                _ptr(losses), sp))
    g.check("ciar_interdro_loss")
    g = Guarded(dev); rsum = g.new(N, torch.float32, "row_sum")
    _check(L.ciar_read_rows(_ptr(c), _ptr(t), N, ctypes.byref(cp), _ptr(rsum), sp))
    g.check("ciar_read_rows")
    if N * int(cp.row_stride) <= 1 << 22:
        g = Guarded(dev)
        d = [g.new(N * int(cp.row_stride), torch.float32, k) for k in ("dense p_lo", "dense p_mid", "dense p_hi")]
        _check(L.ciar_dense_intervals(_ptr(c), _ptr(rad), N, ctypes.byref(cp), _ptr(d[0]), _ptr(d[1]), _ptr(d[2]), sp))
        g.check("ciar_dense_intervals")


@pytest.mark.parametrize("N,V,H", [(1, 5, 1), (37, 130, 3), (257, 16384, 5), (1030, 1000, 8), (9, 32768, 2)])
@pytest.mark.parametrize("strategy", [0, 1])
@pytest.mark.parametrize("tensor_radius", [False, True])
def test_multihead_stays_inside_its_arrays(N, V, H, strategy, tensor_radius):
    import paper_2603_25463_amd as ciar
    from paper_2603_25463_amd.binding import _check, _ptr, _stream
    L = ciar.lib()
    dev = torch.device("cuda:0")
    heads = torch.stack([_rows(N, V, torch.float32, dev, 50 + h) for h in range(H)])
    rad = torch.stack([_rows(N, V, torch.float32, dev, 80 + h, 1.0) for h in range(H)]) if tensor_radius else None
    ids = torch.randint(0, V, (N,), generator=torch.Generator().manual_seed(3), dtype=torch.int32).to(dev)
    P = ciar.Params(confidence=0.9, tau=0.01, window=4)
    cp = P.to_c(heads[0], V)
    per = H * N if strategy == 0 else N
    print(f"canary multihead: N={N} V={V} H={H} strategy={strategy} tensor_radius={tensor_radius}", flush=True)
    for use_ids in (True, False):
        g = Guarded(dev)
        o = {k: g.new(per, torch.float32, k) for k in F_KEYS}
        flags, hf = g.new(N, torch.uint8, "flags"), g.new(H * N, torch.uint8, "head_flags")
        nb = int(L.ciar_multihead_workspace_bytes(N, H, ctypes.byref(cp)))
        ws = g.new(nb, torch.uint8, "workspace")
        _check(L.ciar_quantify_multihead(_ptr(heads), _ptr(rad), H, int(heads.stride(0)), _ptr(ids) if use_ids else None, N,
                                         ctypes.byref(cp), strategy, *[_ptr(o[k]) for k in F_KEYS], _ptr(flags),
                                         _ptr(hf) if strategy == 0 else None, _ptr(ws), nb, _stream(None)))
        g.check(f"ciar_quantify_multihead (ids={use_ids})")


@pytest.mark.parametrize("N,V,D", [(1, 128, 64), (127, 256, 128), (129, 1024, 192), (300, 16384, 256)])
def test_interval_head_stays_inside_its_arrays(N, V, D):
    import paper_2603_25463_amd as ciar
    from paper_2603_25463_amd.binding import _check, _ptr, _stream
    L = ciar.lib()
    dev = torch.device("cuda:0")
    g0 = torch.Generator(device="cpu").manual_seed(5)
    hidden = (torch.randn((N, D), generator=g0)).to(torch.bfloat16).to(dev)
    weight = (torch.randn((2 * V, D), generator=g0) / D ** 0.5).to(torch.bfloat16).to(dev)
    bias = torch.randn((2 * V,), generator=g0).to(dev)
    ids = torch.randint(0, V, (N,), generator=g0, dtype=torch.int32).to(dev)
    P = ciar.Params(confidence=0.9, tau=0.01, window=4, radius_scale=1.0)
    cp = P.to_c(torch.empty((N, V), dtype=torch.float32), V)
    print(f"canary interval head: N={N} V={V} D={D}", flush=True)
    g = Guarded(dev)
    centre, radius = g.new(N * V, torch.float32, "centre"), g.new(N * V, torch.float32, "radius")
    _check(L.ciar_interhead_logits(_ptr(hidden), _ptr(weight), _ptr(bias), D, N, ctypes.byref(cp), _ptr(centre), _ptr(radius),
                                   _stream(None)))
    g.check("ciar_interhead_logits")
    g = Guarded(dev)
    o = {k: g.new(N, torch.float32, k) for k in F_KEYS}
    flags = g.new(N, torch.uint8, "flags")
    nb = int(L.ciar_interhead_workspace_bytes(N, ctypes.byref(cp)))
    ws = g.new(nb, torch.uint8, "workspace")
    _check(L.ciar_interhead_quantify(_ptr(hidden), _ptr(weight), _ptr(bias), D, _ptr(ids), N, ctypes.byref(cp),
                                     *[_ptr(o[k]) for k in F_KEYS], _ptr(flags), _ptr(ws), nb, _stream(None)))
    g.check("ciar_interhead_quantify")
