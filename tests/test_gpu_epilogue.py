"""Bias + activation applied at the kernels' stores (kst_forward_seg_epilogue) against the oracle.

One shape per kernel of every path -- each has a store site of its own -- with each activation,
with and without a bias, at padding factors 0, 2 and 3.  Small integers make ReLU layers exact:
those must match the oracle bit for bit, with NaN guard words around `out`.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_03704_amd import binding as kst
from paper_2209_03704_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-5          # fp32 sums, fp32 bias and activation (tanhf: a few ulp) against fp64

D, G, E = kst.KST_PATH_DIRECT, kst.KST_PATH_IGEMM, kst.KST_PATH_IGEMM_EVEN
# (B, Cin, Cout, N, n, P, dtype, path, which kernel stores the final values)
CASES = [
    (2, 1, 2, 64, 5, 0, "f32", D, "flat-output kernel, one input channel"),
    (1, 1, 3, 50, 3, 0, "f32", D, "row-strip direct kernel (N not a multiple of 4)"),
    (2, 1, 2, 45, 4, 0, "bf16", D, "row-strip direct kernel, 16-bit operands"),
    (1, 2, 3, 7, 9, 0, "f32", D, "generic direct kernel (9 x 9)"),
    (2, 20, 3, 32, 4, 2, "f32", D, "multi-channel direct kernel, frame read in place"),
    (1, 128, 3, 32, 4, 2, "f32", D, "multi-channel direct kernel, four lane groups"),
    (2, 9, 5, 19, 3, 3, "bf16", D, "multi-channel direct kernel, odd padding factor (cropped copy)"),
    (16, 32, 128, 16, 4, 2, "f32", G, "fp32 matrix-core kernel, whole tiles"),
    (2, 64, 128, 8, 4, 2, "f32", G, "fp32 matrix-core kernel, split reduction + summing pass"),
    (1, 512, 128, 4, 4, 2, "f32", G, "fp32 matrix-core kernel, 64+ splits: summing pass with shares"),
    (2, 512, 128, 8, 4, 0, "f32", E, "fp32 even shares: whole tiles and the slot-summing pass"),
    (2, 18, 40, 9, 3, 1, "f32", G, "fp32 matrix-core kernel without pipelining (ragged channels), odd P"),
    (9, 130, 16, 6, 4, 0, "bf16", G, "first 16-bit matrix-core kernel, split reduction"),
    (3, 37, 40, 17, 5, 0, "f16", G, "first 16-bit matrix-core kernel, whole tiles"),
    (3, 40, 130, 34, 4, 0, "bf16", G, "16-bit row-strip kernel"),
    (2, 48, 64, 30, 2, 2, "bf16", G, "16-bit LDS-ring kernel (framed to 32 x 32)"),
    (4, 32, 256, 64, 3, 0, "bf16", G, "16-bit wide-tile kernel"),
    (29, 112, 128, 32, 2, 0, "f16", G, "16-bit wide-tile kernel, 32 x 32 maps"),
]
ACTS = {"none": (kst.KST_ACT_NONE, oracle.ACT_NONE), "relu": (kst.KST_ACT_RELU, oracle.ACT_RELU),
        "tanh": (kst.KST_ACT_TANH, oracle.ACT_TANH)}


def make(case, dist, seed):
    B, Cin, Cout, N, n, P, dtype, path, _ = case
    layer = wl.Layer("epi", B, Cin, Cout, N, n, dtype, dist, w_std=0.1, P=P)
    x, w = wl.make_tensors(layer, seed)
    g = torch.Generator().manual_seed(seed + 1)
    if dist == "integer":
        bias = torch.randint(-40, 41, (Cout,), generator=g).to(torch.float32)
    else:
        bias = torch.randn((Cout,), generator=g, dtype=torch.float32) * 0.5
    return layer, x, w, bias


@pytest.mark.parametrize("act", ["none", "relu", "tanh"])
@pytest.mark.parametrize("case", CASES, ids=[c[-1] for c in CASES])
def test_bias_and_activation_at_the_stores(case, act):
    B, Cin, Cout, N, n, P, dtype, path, _ = case
    layer, x, w, bias = make(case, "normal", 7000 + 13 * N + n)
    w_seg = kst.kst_segregate_weights(w.to(DEV))
    got = kst.kst_forward_seg_epilogue(x.to(DEV), w_seg, Cout, n, bias.to(DEV), ACTS[act][0], P, path=path)
    nobias = kst.kst_forward_seg_epilogue(x.to(DEV), w_seg, Cout, n, None, ACTS[act][0], P, path=path)
    torch.cuda.synchronize()
    want = oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), bias.numpy().astype(np.float64), ACTS[act][1], P)
    # tolerance relative to the scale of what goes into the activation (tanh squashes the result itself)
    scale = max(1.0, np.abs(oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), bias.numpy().astype(np.float64),
                                                    oracle.ACT_NONE, P)).max())
    assert got.shape == want.shape
    err = np.abs(got.cpu().numpy() - want).max()
    assert err <= TOL * scale, "%s / %s: abs err %.3e (scale %.3g)" % (case[-1], act, err, scale)
    want0 = oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), None, ACTS[act][1], P)
    err0 = np.abs(nobias.cpu().numpy() - want0).max()
    assert err0 <= TOL * scale, "%s / %s without bias: abs err %.3e" % (case[-1], act, err0)


@pytest.mark.parametrize("case", CASES, ids=[c[-1] for c in CASES])
def test_relu_layer_is_exact_on_integers_and_stays_inside_out(case):
    B, Cin, Cout, N, n, P, dtype, path, _ = case
    layer, x, w, bias = make(case, "integer", 7100 + N + n)
    M = kst.kst_out_size_padded(N, n, P)
    shape = (B, Cout, M, M)
    numel = int(np.prod(shape))
    guard = 4096
    buf = torch.full((numel + 2 * guard,), float("nan"), device=DEV)
    out = buf[guard:guard + numel].view(shape)
    kst.kst_forward_seg_epilogue(x.to(DEV), kst.kst_segregate_weights(w.to(DEV)), Cout, n, bias.to(DEV),
                                 kst.KST_ACT_RELU, P, out=out, path=path)
    torch.cuda.synchronize()
    host = buf.cpu()
    assert torch.isnan(host[:guard]).all() and torch.isnan(host[guard + numel:]).all()
    want = oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), bias.numpy().astype(np.float64), oracle.ACT_RELU, P)
    got = host[guard:guard + numel].view(shape).numpy().astype(np.float64)
    assert (want == 0).any() and (want > 0).any()          # the clip is exercised
    assert np.array_equal(got, want), case[-1]


def test_without_bias_and_activation_it_is_the_bare_layer_bit_for_bit():
    for case in (CASES[0], CASES[4], CASES[8], CASES[16]):
        B, Cin, Cout, N, n, P, dtype, path, _ = case
        layer, x, w, _ = make(case, "normal", 7200 + N)
        xd, w_seg = x.to(DEV), kst.kst_segregate_weights(w.to(DEV))
        a = kst.kst_forward_seg_epilogue(xd, w_seg, Cout, n, None, kst.KST_ACT_NONE, P, path=path)
        b = kst.kst_forward_seg_padded(xd, w_seg, Cout, n, P, path=path)
        torch.cuda.synchronize()
        assert torch.equal(a, b), case[-1]


def test_full_size_generator_layers_with_their_activations():
    """Table 3's 16 -> 32 DCGAN layer at a batch of 64 with bias + ReLU, and its 128 -> 3 output
    layer with bias + tanh: every batch item x one channel of every block of 32, whole planes."""
    for (B, Cin, Cout, N, act) in ((64, 256, 128, 16, "relu"), (64, 128, 3, 32, "tanh")):
        layer = wl.Layer("epi_full", B, Cin, Cout, N, 4, "f32", "relu_normal", P=2)
        x, w = wl.make_tensors(layer, 7300 + N)
        bias = torch.randn((Cout,), generator=torch.Generator().manual_seed(N), dtype=torch.float32) * 0.2
        out = kst.kst_forward_seg_epilogue(x.to(DEV), kst.kst_segregate_weights(w.to(DEV)), Cout, 4, bias.to(DEV),
                                           ACTS[act][0], 2)
        torch.cuda.synchronize()
        b_idx, co_idx = [], []
        for b in range(B):
            for g0 in range(0, Cout, 32):
                width = min(32, Cout - g0)
                b_idx.append(b)
                co_idx.append(g0 + (5 * b + 3 * (g0 // 32)) % width)
        bare = oracle.forward_planes(wl.to_f64(x), wl.to_f64(w), b_idx, co_idx, 2)
        pre = bare + bias.numpy().astype(np.float64)[np.array(co_idx)][:, None, None]
        want = np.maximum(pre, 0.0) if act == "relu" else np.tanh(pre)
        got = out[torch.tensor(b_idx), torch.tensor(co_idx)].cpu().numpy()
        assert np.abs(got - want).max() <= TOL * max(1.0, np.abs(pre).max())


def test_arguments_are_checked_before_anything_is_launched():
    case = CASES[4]
    B, Cin, Cout, N, n, P, dtype, path, _ = case
    layer, x, w, bias = make(case, "normal", 1)
    xd, w_seg = x.to(DEV), kst.kst_segregate_weights(w.to(DEV))
    out = torch.full((B, Cout, 2 * N + 2 * P - n, 2 * N + 2 * P - n), float("nan"), device=DEV)
    with pytest.raises(kst.KstError) as e:
        kst.kst_forward_seg_epilogue(xd, w_seg, Cout, n, bias.to(DEV), 3, P, out=out, path=path)
    assert e.value.status == 8                           # KST_ERR_ACT
    # the row-parity-passes kernel stores bare sums only
    big = wl.Layer("pp", 7, 256, 128, 64, 3, "bf16", "relu_normal")
    xb, wb = wl.make_tensors(big, 2)
    with pytest.raises(kst.KstError) as e:
        kst.kst_forward_seg_epilogue(xb.to(DEV), kst.kst_segregate_weights(wb.to(DEV)), 128, 3,
                                     torch.zeros(128, device=DEV), kst.KST_ACT_RELU, 0, path=kst.KST_PATH_IGEMM_PASSES)
    assert e.value.status == 6                           # KST_ERR_PATH
    torch.cuda.synchronize()
    assert torch.isnan(out).all()
