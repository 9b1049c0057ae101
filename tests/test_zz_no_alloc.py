"""The allocation-free entry point (ciar_quantify_verify_static) against ciar_quantify_verify, through the C ABI:
two calls in a row on the library's built-in scratch buffer, the second with a smaller input, so that what the
first call left in the buffer would show.  Same kernels on both sides: every output must be bit-identical."""
import ctypes

import pytest
import torch

pytestmark = pytest.mark.gpu

KEYS_F = ("p_lo", "p_mid", "p_hi", "omega", "sigma", "score")


def _outputs(N, K, dev, fill):
    W = (N + K - 1) // K
    o = {k: torch.full((N,), float(fill), dtype=torch.float32, device=dev) for k in KEYS_F}
    o["flags"] = torch.full((N,), 7, dtype=torch.uint8, device=dev)
    o["accept"] = torch.full((N,), 7, dtype=torch.uint8, device=dev)
    o["row_id"] = torch.full((N,), -7, dtype=torch.int32, device=dev)
    o["accept_len"] = torch.full((W,), -7, dtype=torch.int32, device=dev)
    o["resampled_id"] = torch.full((W,), -7, dtype=torch.int32, device=dev)
    return o


def _both(ciar, wl, workload, rows, tau):
    from paper_2603_25463_amd.binding import _check, _ptr, _stream
    dev = torch.device("cuda:0")
    w = wl.make(workload, device=dev, rows=rows)
    N, K = w.rows, w.spec.window
    P = ciar.Params(confidence=0.9, tau=tau, window=K)
    cp = P.to_c(w.draft)
    L = ciar.lib()
    ref = _outputs(N, K, dev, -1.0)
    ws = torch.empty(ciar.workspace_bytes(N, cp), dtype=torch.uint8, device=dev)
    ins = (_ptr(w.draft), None, _ptr(w.target), _ptr(w.ids), _ptr(w.u_accept), _ptr(w.u_resample), N, ctypes.byref(cp))
    names = KEYS_F + ("flags", "accept", "row_id", "accept_len", "resampled_id")
    sp = _stream(None)
    _check(L.ciar_quantify_verify(*ins, *[_ptr(ref[k]) for k in names], _ptr(ws), ws.numel(), sp))
    got = _outputs(N, K, dev, -2.0)
    print(f"static call: workload {workload} rows={N} V={w.spec.vocab} K={K}", flush=True)
    _check(L.ciar_quantify_verify_static(*ins, *[_ptr(got[k]) for k in names], sp))
    torch.cuda.synchronize()
    for k in names:
        assert torch.equal(ref[k], got[k]), f"{k} differs between the static and the workspace entry point"
    assert int((ref["accept"] == 0).sum()) > 0, "the case should contain rejected rows"
    return ref


def test_static_entry_point_matches_on_two_calls_in_a_row():
    import paper_2603_25463_amd as ciar
    from paper_2603_25463_amd import workloads as wl
    ciar.lib()
    # first a batch that fills a good part of the buffer, then a smaller one of another shape (bf16, another
    # vocabulary tile): whatever the first call left behind must not leak into the second
    _both(ciar, wl, 4, 4096, 0.01)
    _both(ciar, wl, 3, 300, 0.01)
    _both(ciar, wl, 1, 37, 0.01)


def test_static_entry_point_rejects_more_rows_than_it_holds():
    import paper_2603_25463_amd as ciar
    from paper_2603_25463_amd.binding import CiarParams, last_error
    L = ciar.lib()
    p = CiarParams()
    L.ciar_params_default(ctypes.byref(p))
    p.vocab, p.row_stride = 1024, 1024
    fake = 0x7f0000000000
    rc = L.ciar_quantify_verify_static(fake, None, fake, fake, fake, fake, ciar.binding.STATIC_MAX_ROWS + 1,
                                       ctypes.byref(p), *([fake] * 11), None)
    assert rc == -3 and "CIAR_STATIC_MAX_ROWS" in last_error()


def test_static_entry_point_empty_batch():
    import paper_2603_25463_amd as ciar
    from paper_2603_25463_amd.binding import CiarParams
    L = ciar.lib()
    p = CiarParams()
    L.ciar_params_default(ctypes.byref(p))
    p.vocab, p.row_stride = 1024, 1024
    fake = 0x7f0000000000
    assert L.ciar_quantify_verify_static(fake, None, fake, fake, fake, fake, 0, ctypes.byref(p), *([fake] * 11), None) == 0
