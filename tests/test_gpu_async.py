"""The library's entry points only enqueue work: none of them waits for the stream.

Each call is made behind a kernel that keeps the stream busy for a long time (a loop of
matrix-core instructions from the library's own measuring aids); when the call returns, an event
recorded behind that kernel must still be pending.  The results are checked after the wait, so the
calls did run, in stream order, behind it.
"""
import time

import numpy as np
import pytest
import torch

from paper_2209_03704_amd import binding as kst
from paper_2209_03704_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def busy_iterations():
    """Iterations of the measuring kernel that keep the chip busy for about 0.2 s."""
    sink = torch.zeros(kst.kst_yardstick_mfma_sink_elems(), dtype=torch.float32, device=DEV)
    it = 20_000
    kst.kst_yardstick_mfma(kst.KST_BF16, it, sink)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    kst.kst_yardstick_mfma(kst.KST_BF16, it, sink)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return sink, min(max(it, int(it * 0.2 / dt)), 50_000_000)


def test_calls_return_while_the_stream_is_still_busy():
    import oracle
    layer = wl.Layer("async", 4, 64, 128, 12, 4, "f32", "relu_normal", w_std=0.1)
    small = wl.Layer("async_direct", 2, 1, 1, 40, 5, "f32", "normal")
    x, w = wl.make_tensors(layer, 11)
    xs, wsm = wl.make_tensors(small, 12)
    xd, wd, xsd, wsd = x.to(DEV), w.to(DEV), xs.to(DEV), wsm.to(DEV)
    P = 2
    Mp = kst.kst_out_size_padded(layer.N, layer.n, P)
    g = torch.randn((layer.B, layer.Cout, Mp, Mp), generator=torch.Generator().manual_seed(5)).to(DEV)
    w_seg = torch.empty(kst.kst_segregated_elems(layer.Cin, layer.Cout, layer.n, kst.KST_F32), device=DEV)
    out_seg = torch.empty(layer.out_shape, device=DEV)
    out_static = torch.empty(layer.out_shape, device=DEV)
    out_whole = torch.empty(layer.out_shape, device=DEV)
    out_pad = torch.empty((layer.B, layer.Cout, Mp, Mp), device=DEV)
    out_small = torch.empty(small.out_shape, device=DEV)
    din = torch.empty(layer.in_shape, device=DEV)
    dw = torch.empty(layer.w_shape, device=DEV)
    need = kst.kst_workspace_bytes(layer.B, layer.Cin, layer.Cout, layer.N, layer.n, kst.KST_F32, kst.KST_PATH_AUTO)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    ws_bi = torch.empty(max(kst.kst_backward_input_workspace_bytes(
        layer.B, layer.Cin, layer.Cout, layer.N, layer.n, P, kst.KST_F32), 16), dtype=torch.uint8, device=DEV)
    ws_bw = torch.empty(max(kst.kst_backward_weight_workspace_bytes(
        layer.B, layer.Cin, layer.Cout, layer.N, layer.n, P, kst.KST_F32), 16), dtype=torch.uint8, device=DEV)

    calls = [
        ("kst_segregate_weights", lambda: kst.kst_segregate_weights(wd, w_seg)),
        ("kst_forward_seg", lambda: kst.kst_forward_seg(xd, w_seg, layer.Cout, layer.n, out=out_seg, ws=ws)),
        ("kst_forward_seg_static", lambda: kst.kst_forward_seg_static(xd, w_seg, layer.Cout, layer.n, out_static)),
        ("kst_forward", lambda: kst.kst_forward(xd, wd, out=out_whole)),
        ("kst_forward_padded", lambda: kst.kst_forward_padded(xd, wd, P, out=out_pad)),
        ("kst_forward (direct)", lambda: kst.kst_forward(xsd, wsd, out=out_small)),
        ("kst_backward_input", lambda: kst.kst_backward_input(g, wd, layer.N, P, din=din, ws=ws_bi)),
        ("kst_backward_weight", lambda: kst.kst_backward_weight(xd, g, layer.n, P, dw=dw, ws=ws_bw)),
    ]
    # First use on the device may set things up (the library's memory pool, the address of its
    # fixed workspace): that is allowed to wait, a later call is not.
    for _, fn in calls:
        fn()
    torch.cuda.synchronize()
    for t in (out_seg, out_static, out_whole, out_pad, out_small, din, dw):
        t.fill_(float("nan"))
    sink, iters = busy_iterations()
    for name, fn in calls:
        torch.cuda.synchronize()
        kst.kst_yardstick_mfma(kst.KST_BF16, iters, sink)
        behind = torch.cuda.Event()
        behind.record()
        t0 = time.perf_counter()
        fn()
        host_s = time.perf_counter() - t0
        pending = not behind.query()
        torch.cuda.synchronize()
        assert pending, "%s returned only after the stream had drained (%.1f ms on the host)" % (name, host_s * 1e3)
        assert host_s < 0.1, "%s took %.1f ms on the host behind a 200 ms kernel" % (name, host_s * 1e3)

    want = oracle.forward(wl.to_f64(x), wl.to_f64(w))
    scale = np.abs(want).max()
    for got in (out_seg, out_static, out_whole):
        assert np.abs(got.cpu().numpy() - want).max() <= 2e-5 * scale
    want_p = oracle.forward(wl.to_f64(x), wl.to_f64(w), P)
    assert np.abs(out_pad.cpu().numpy() - want_p).max() <= 2e-5 * np.abs(want_p).max()
    want_s = oracle.forward(wl.to_f64(xs), wl.to_f64(wsm))
    assert np.abs(out_small.cpu().numpy() - want_s).max() <= 2e-5 * np.abs(want_s).max()
    g64 = g.cpu().to(torch.float64).numpy()
    want_din = oracle.backward_input(g64, wl.to_f64(w), layer.N, P)
    want_dw = oracle.backward_weight(wl.to_f64(x), g64, layer.n, P)
    assert np.abs(din.cpu().numpy() - want_din).max() <= 2e-5 * np.abs(want_din).max()
    assert np.abs(dw.cpu().numpy() - want_dw).max() <= 2e-5 * np.abs(want_dw).max()
