"""The entry point that allocates nothing (kst_forward_seg_static) against kst_forward_seg.

Same kernels on the same inputs, so the two results must agree bit for bit; each is also held to
the oracle.  Two calls in a row share the library's fixed workspace, the second on a smaller layer
(whatever the first left behind must not show); a layer that needs more workspace than the
array holds must be refused before anything is launched.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_03704_amd import binding as kst
from paper_2209_03704_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_both(layer, seed, path):
    x, w = wl.make_tensors(layer, seed)
    xd, wd = x.to(DEV), w.to(DEV)
    w_seg = kst.kst_segregate_weights(wd)
    code = {"f32": kst.KST_F32, "bf16": kst.KST_BF16}[layer.dtype]
    need = kst.kst_workspace_bytes(layer.B, layer.Cin, layer.Cout, layer.N, layer.n, code, path)
    want_gpu = kst.kst_forward_seg(xd, w_seg, layer.Cout, layer.n, path=path)
    out = torch.full(layer.out_shape, float("nan"), dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    kst.kst_forward_seg_static(xd, w_seg, layer.Cout, layer.n, out, path=path)
    torch.cuda.synchronize()
    return x, w, out, want_gpu, need


def test_static_workspace_entry_point_two_calls_in_a_row():
    # 1: one tile x 128 channel chunks in even shares over 128 workgroups (forced): the whole 64 MiB array
    # 2: a smaller layer whose reduction is split over workgroups (partial sums + summing pass)
    # 3: 16-bit operands, split reduction; 4: a direct-path layer that needs no workspace at all
    cases = [(wl.Layer("static_1", 2, 512, 128, 8, 4, "f32", "relu_normal", w_std=0.1), kst.KST_PATH_IGEMM_EVEN),
             (wl.Layer("static_2", 3, 100, 132, 12, 5, "f32", "relu_normal", w_std=0.1), kst.KST_PATH_AUTO),
             (wl.Layer("static_3", 9, 130, 16, 6, 4, "bf16", "relu_normal", w_std=0.1), kst.KST_PATH_IGEMM),
             (wl.Layer("static_4", 2, 3, 2, 33, 3, "f32", "normal", w_std=0.2), kst.KST_PATH_AUTO)]
    needs = []
    for k, (layer, path) in enumerate(cases):
        x, w, out, want_gpu, need = run_both(layer, 600 + k, path)
        needs.append(need)
        assert need <= kst.KST_STATIC_SCRATCH_BYTES
        assert torch.equal(out, want_gpu), layer.name
        want = oracle.forward(wl.to_f64(x), wl.to_f64(w))
        err = np.abs(out.cpu().numpy().astype(np.float64) - want).max() / np.abs(want).max()
        assert err <= 2e-5, "%s: rel err %.3e" % (layer.name, err)
    assert needs[0] == kst.KST_STATIC_SCRATCH_BYTES and 0 < needs[1] < needs[0] and needs[2] > 0 and needs[3] == 0


def test_static_workspace_entry_point_refuses_what_does_not_fit():
    layer = wl.Layer("static_big", 4, 1024, 512, 4, 4, "f32", "relu_normal")
    path = kst.KST_PATH_IGEMM_EVEN                   # even shares of this layer want 128 MiB of slots
    assert kst.kst_workspace_bytes(4, 1024, 512, 4, 4, kst.KST_F32, path) > kst.KST_STATIC_SCRATCH_BYTES
    x, w = wl.make_tensors(layer, 1)
    xd, wd = x.to(DEV), w.to(DEV)
    out = torch.full(layer.out_shape, float("nan"), dtype=torch.float32, device=DEV)
    with pytest.raises(kst.KstError) as e:
        kst.kst_forward_seg_static(xd, kst.kst_segregate_weights(wd), layer.Cout, layer.n, out, path=path)
    assert e.value.status == 4                       # KST_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.isnan(out).all()                    # nothing was launched
