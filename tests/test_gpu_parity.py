"""Parity of the HIP path (through the C ABI) against the CPU fp64 oracle.

Tolerance: max|gpu - oracle| <= 2e-5 * max|oracle|, the bound the baseline fixes for
fp32, applied to 16-bit operands too (see TOL below).  Both sides read the same
seeded inputs (16-bit cases: the same rounded bits).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_03704_amd import binding as kst
from paper_2209_03704_amd import workloads as wl

pytestmark = pytest.mark.gpu

# The baseline's contractual bound for bf16 operands is 1e-2 * max|oracle|.  The tests hold them to
# the fp32 bound instead: both sides read the same rounded operands, a product of two 16-bit
# values is exact in fp32, and the sums are fp32 -- so only the accumulation order differs, as
# for fp32 operands.  At 1e-2 a dropped tap among hundreds of terms could pass.
CONTRACT_TOL = {"f32": 2e-5, "bf16": 1e-2, "f16": 1e-2}
TOL = {"f32": 2e-5, "bf16": 2e-5, "f16": 2e-5}
DEV = "cuda:0"


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    scale = np.abs(want).max()
    if scale == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got.astype(np.float64) - want).max() / scale)


def run_paths(layer, paths, seed=None, skip_unsupported_igemm=False):
    """Yield (name, gpu_output_numpy) for every requested way through the library."""
    x, w = wl.make_tensors(layer, seed)
    xd, wd = x.to(DEV), w.to(DEV)
    res = {}
    for name in paths:
        if name == "forward":
            o = kst.kst_forward(xd, wd)
        elif name == "zero_insert":
            o = kst.kst_forward_zero_insert(xd, wd)
        else:
            path = {"direct": kst.KST_PATH_DIRECT, "igemm": kst.KST_PATH_IGEMM, "auto": kst.KST_PATH_AUTO}[name]
            ws = kst.kst_segregate_weights(wd)
            try:
                o = kst.kst_forward_seg(xd, ws, layer.Cout, layer.n, path=path)
            except kst.KstError as e:
                # The matrix-core kernels decline shapes whose tile does not fit in LDS.
                if name == "igemm" and e.status == 6 and skip_unsupported_igemm:
                    continue
                raise
        torch.cuda.synchronize()
        res[name] = o.cpu().numpy()
    return x, w, res


def check_layer(layer, paths=("direct", "igemm", "forward", "zero_insert"), seed=None,
                skip_unsupported_igemm=False):
    x, w, res = run_paths(layer, paths, seed, skip_unsupported_igemm)
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w))
    for name, got in res.items():
        assert got.shape == want.shape, name
        assert np.isfinite(got).all(), name
        e = rel_err(got, want)
        assert e <= TOL[layer.dtype], "%s on %s: rel err %.3e" % (name, layer, e)


def check_exact_with_guards(layer, path, seed, P=0):
    """Small integers are exact in every operand type and in the fp32 sums, so whatever the
    order of accumulation the result must equal the oracle bit for bit; words before and after
    `out` must keep their NaN pattern and every element of `out` must be written."""
    x, w = wl.make_tensors(layer, seed)
    xd, wd = x.to(DEV), w.to(DEV)
    M = kst.kst_out_size_padded(layer.N, layer.n, P)
    shape = (layer.B, layer.Cout, M, M)
    numel = int(np.prod(shape))
    guard = 4096
    buf = torch.full((numel + 2 * guard,), float("nan"), device=DEV)
    out = buf[guard:guard + numel].view(shape)
    kst.kst_forward_seg_padded(xd, kst.kst_segregate_weights(wd), layer.Cout, layer.n, P, out=out, path=path)
    torch.cuda.synchronize()
    host = buf.cpu()
    assert torch.isnan(host[:guard]).all() and torch.isnan(host[guard + numel:]).all()
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w), P)
    assert np.array_equal(host[guard:guard + numel].view(shape).numpy().astype(np.float64), want)


# ----------------------------------------------------------------------------
# Weight pre-segregation: bit-exact permutation into the documented layout
# ----------------------------------------------------------------------------
def expected_segregation(w: torch.Tensor) -> torch.Tensor:
    """Layout of include/kst.h, built with tensor slicing on the host."""
    Cout, Cin, n, _ = w.shape
    parts = []
    for r in (0, 1):
        for s in (0, 1):
            sub = w[:, :, r::2, s::2]                              # Section 3.2: alternate rows/cols
            T = sub.shape[2] * sub.shape[3]
            if T == 0:
                continue
            sub = sub.reshape(Cout, Cin, T)
            if w.dtype == torch.float32:
                parts.append(sub.permute(1, 2, 0).reshape(-1))    # [Cin][T][Cout]
            else:
                pad = (-Cin) % 8
                sub = torch.nn.functional.pad(sub, (0, 0, 0, pad))  # zero channels up to a multiple of 8
                g = sub.reshape(Cout, (Cin + pad) // 8, 8, T)
                parts.append(g.permute(1, 3, 0, 2).reshape(-1))   # [Cin/8][T][Cout][8]
    return torch.cat(parts)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("Cin,Cout,n", [(1, 1, 3), (3, 2, 5), (5, 7, 4), (16, 33, 1), (9, 4, 2), (13, 3, 7),
                                          (40, 70, 6), (100, 96, 5), (64, 128, 4), (33, 40, 3), (130, 32, 2)])
def test_segregate_weights_is_the_documented_permutation(dtype, Cin, Cout, n):
    g = torch.Generator().manual_seed(Cin * 100 + Cout * 10 + n)
    w = torch.randn((Cout, Cin, n, n), generator=g)
    if dtype != "f32":
        w = w.to(torch.bfloat16 if dtype == "bf16" else torch.float16)
    got = kst.kst_segregate_weights(w.to(DEV)).cpu()
    want = expected_segregation(w)
    code = {"f32": kst.KST_F32, "bf16": kst.KST_BF16, "f16": kst.KST_F16}[dtype]
    assert got.numel() == want.numel() == kst.kst_segregated_elems(Cin, Cout, n, code)
    assert torch.equal(got.view(torch.int32 if dtype == "f32" else torch.int16),
                       want.contiguous().view(torch.int32 if dtype == "f32" else torch.int16))


# ----------------------------------------------------------------------------
# Tiny grid: every kernel size, minimal and ragged maps, every path, both dtypes
# ----------------------------------------------------------------------------
def tiny_shapes():
    for n in range(1, 8):
        nmin = n // 2 + 1
        for N in sorted({nmin, nmin + 1, nmin + 3, 9, 20}):
            yield N, n


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,n", list(tiny_shapes()))
def test_tiny_grid(N, n, dtype):
    for (B, Cin, Cout) in [(1, 1, 1), (2, 3, 5), (3, 5, 2)]:
        layer = wl.Layer("tiny", B, Cin, Cout, N, n, dtype, "normal", w_std=0.5)
        check_layer(layer, seed=1000 * N + 10 * n + B, skip_unsupported_igemm=(n >= 6))


def test_integer_inputs_are_exact_in_fp32():
    """Small integers: every product and partial sum is exact in fp32, so any path must
    reproduce the oracle bit for bit whatever its accumulation order."""
    for (B, Cin, Cout, N, n) in [(2, 3, 2, 11, 3), (1, 9, 17, 7, 4), (2, 4, 3, 40, 5), (1, 24, 40, 9, 5)]:
        layer = wl.Layer("int", B, Cin, Cout, N, n, "f32", "integer")
        x, w, res = run_paths(layer, ("direct", "igemm", "forward", "zero_insert"), seed=B + N)
        want = oracle.forward(wl.to_f64(x), wl.to_f64(w))
        for name, got in res.items():
            assert np.array_equal(got.astype(np.float64), want), name


def test_n9_uses_the_generic_direct_kernel():
    layer = wl.Layer("n9", 2, 2, 3, 12, 9, "f32", "normal", w_std=0.5)
    check_layer(layer, paths=("direct", "auto", "forward", "zero_insert"), seed=9)
    with pytest.raises(kst.KstError):
        run_paths(layer, ("igemm",), seed=9)


# ----------------------------------------------------------------------------
# Several tiles and ragged tails
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Cin,Cout,N,n", [
    (2, 3, 2, 150, 5),      # direct: 3 x 19 tiles of quads, ragged in both directions
    (1, 1, 3, 131, 3),      # odd M, last tile one quad wide
    (3, 2, 1, 70, 4),       # even kernel, E = 68
    (1, 1, 1, 300, 2),
])
def test_direct_multi_tile(B, Cin, Cout, N, n, dtype):
    layer = wl.Layer("mt", B, Cin, Cout, N, n, dtype, "normal", w_std=0.3)
    check_layer(layer, paths=("direct", "forward"), seed=N + n)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Cin,Cout,N,n", [
    (2, 3, 1, 70, 3),       # Table 1's channel counts: one output channel, chunks of 4 channels
    (2, 3, 1, 70, 4),
    (1, 3, 1, 45, 5),
    (2, 20, 3, 32, 4),      # the last generator layer's shape (-> RGB): three chunks, the last ragged
    (1, 9, 2, 37, 5),       # two channels per lane, odd M, a tile one quad wide
    (1, 4, 4, 33, 6),       # exactly one chunk of 4 (fp32) / half a chunk of 8 (bf16)
    (2, 5, 5, 19, 3),       # Cout = 5: one channel per lane
    (1, 17, 6, 21, 7),      # Cout = 6: lanes take 3 channels each; largest kernel
    (1, 8, 8, 18, 2),       # Cout = 8: groups of 4
    (3, 2, 7, 12, 1),       # n = 1: three empty sub-kernels
    (1, 33, 12, 70, 4),     # several tiles in both directions, groups of 4 of 12 channels
])
def test_direct_several_input_channels(B, Cin, Cout, N, n, dtype):
    """Direct path with Cin >= 2: the kernel that keeps a quad of up to four output channels per lane."""
    layer = wl.Layer("multi", B, Cin, Cout, N, n, dtype, "normal", w_std=0.3)
    check_layer(layer, paths=("direct",), seed=31 * N + 7 * n + Cin)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Cin,Cout,N,n,P", [
    (1, 128, 3, 32, 4, 2),    # Table 3's 128 -> 3 output layer on one sample: four lane groups, four rounds
    (2, 64, 3, 32, 4, 2),     # the 64 -> 3 one: two rounds
    (1, 72, 3, 20, 4, 0),     # nine chunks over four groups: three groups idle in the last round
    (1, 40, 2, 37, 5, 0),     # two groups, five chunks; odd M, two channels per lane
    (2, 100, 4, 18, 3, 1),    # ragged last chunk (100 = 12 * 8 + 4), four channels per lane, odd padding factor
    (1, 64, 4, 16, 4, 2),     # 4 x 4 with four channels per lane: two groups (registers)
    (1, 96, 1, 40, 5, 2),     # one channel per lane, 5 x 5
    (3, 33, 6, 21, 2, 0),     # Cout = 6: lanes take 3 channels; a chunk with one channel in it
    (1, 256, 3, 9, 1, 0),     # n = 1: three empty sub-kernels, 32 chunks
])
def test_direct_many_input_channels_in_lane_groups(B, Cin, Cout, N, n, P, dtype):
    """Few tiles and many input channels: the workgroup's lane groups share the reduction of a tile
    and their sums are added in a fixed order (bit-reproducible)."""
    layer = wl.Layer("multi_groups", B, Cin, Cout, N, n, dtype, "normal", w_std=0.3)
    x, w = wl.make_tensors(layer, 500 + Cin + 3 * n)
    xd, w_seg = x.to(DEV), kst.kst_segregate_weights(w.to(DEV))
    got = kst.kst_forward_seg_padded(xd, w_seg, Cout, n, P, path=kst.KST_PATH_DIRECT)
    again = kst.kst_forward_seg_padded(xd, w_seg, Cout, n, P, path=kst.KST_PATH_DIRECT)
    torch.cuda.synchronize()
    assert torch.equal(got, again)
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w), P)
    e = rel_err(got.cpu().numpy(), want)
    assert e <= TOL[dtype], "rel err %.3e" % e
    int_layer = wl.Layer("multi_groups_int", B, Cin, Cout, N, n, dtype, "integer")
    check_exact_with_guards(int_layer, kst.KST_PATH_DIRECT, 600 + Cin, P=P)


def test_direct_several_input_channels_is_exact_on_integers_and_stays_inside_out():
    for (B, Cin, Cout, N, n, P) in [(2, 20, 3, 32, 4, 0), (1, 9, 2, 37, 5, 0), (2, 3, 1, 30, 3, 2), (1, 6, 4, 11, 4, 3),
                                    (1, 5, 3, 2, 5, 2)]:
        layer = wl.Layer("multi_int", B, Cin, Cout, N, n, "f32", "integer")
        x, w = wl.make_tensors(layer, 100 + N)
        xd, wd = x.to(DEV), w.to(DEV)
        M = kst.kst_out_size_padded(N, n, P)
        numel = B * Cout * M * M
        guard = 2048
        buf = torch.full((numel + 2 * guard,), float("nan"), device=DEV)
        out = buf[guard:guard + numel].view(B, Cout, M, M)
        kst.kst_forward_seg_padded(xd, kst.kst_segregate_weights(wd), Cout, n, P, out=out, path=kst.KST_PATH_DIRECT)
        torch.cuda.synchronize()
        host = buf.cpu()
        assert torch.isnan(host[:guard]).all() and torch.isnan(host[guard + numel:]).all()
        want = oracle.forward(wl.to_f64(x), wl.to_f64(w), P)
        assert np.array_equal(host[guard:guard + numel].view(out.shape).numpy().astype(np.float64), want), (N, n, P)


@pytest.mark.parametrize("B,Cout,N,n", [
    (2, 3, 100, 5),     # M = 195: planes end off 16-byte boundaries, several output channels
    (3, 2, 64, 4),      # even kernel
    (5, 1, 48, 3),      # M*M just above one block: most blocks touch two planes
    (1, 2, 200, 7),
    (2, 2, 52, 1),      # n = 1: three empty sub-kernels, zeros must still be written
    (3, 1, 60, 2),
    (1, 3, 96, 6),
    (2, 1, 512, 5),     # the headline layer's map size
])
def test_direct_single_channel_flat_kernel(B, Cout, N, n):
    """fp32, one input channel, N a multiple of 4: the persistent flat-output kernel."""
    layer = wl.Layer("flat", B, 1, Cout, N, n, "f32", "normal", w_std=0.3)
    check_layer(layer, paths=("direct", "forward"), seed=N * 3 + n)
    layer = wl.Layer("flat_int", B, 1, Cout, N, n, "f32", "integer")
    x, w, res = run_paths(layer, ("direct",), seed=N + n)
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w))
    assert np.array_equal(res["direct"].astype(np.float64), want)


@pytest.mark.parametrize("B,Cin,Cout,N,n,P", [
    # (three channels take this kernel from 1024 blocks of 8192 outputs on: hence the batch sizes)
    (520, 3, 1, 64, 3, 2),    # Table 1's channel counts at a small map: frame of one, M = 129
    (61, 3, 2, 132, 5, 2),    # M = 263: the path for maps wider than a wave's 256 floats; two output channels
    (42, 3, 1, 224, 4, 2),    # Table 1's map, even kernel
    (1000, 3, 1, 48, 3, 0),   # three channels without a frame; M * M just above one block
    (253, 3, 2, 64, 7, 4),    # frame of two, largest kernel
    (400, 3, 1, 72, 2, 3),    # odd padding factor: frame of two, rows and columns shifted by one (sub-kernel roles swapped)
    (70, 3, 2, 132, 5, 1),    # odd padding factor on wide maps (M = 261)
    (15, 3, 1, 384, 3, 0),    # three channels on maps too wide for the half-size blocks: blocks of 8192, two workgroups per CU
    (8, 3, 1, 512, 5, 2),     # ... and too wide for those as well: half-size blocks at two per CU
    (2, 3, 1, 64, 3, 2),      # too few blocks: the multi-channel kernel
    (2, 1, 2, 64, 5, 2),      # one input channel with a frame (no framed copy of the input any more)
    (1, 1, 1, 512, 5, 2),     # the headline layer's map with a frame
    (2, 1, 3, 100, 3, 8),     # frame of four (the widest the kernel supplies)
    (1, 1, 1, 60, 6, 3),      # one channel, odd padding factor
    (2, 1, 2, 128, 5, 5),     # one channel, odd padding factor, M = 261
    (1, 1, 1, 64, 3, 7),      # frame of four with the shift
    (1, 3, 1, 40, 5, 6),      # frame of three: pieces that lie entirely inside the frame rows
    (2, 3, 1, 32, 3, 10),     # frame of five: beyond the flat kernel, the multi-channel kernel takes it
])
def test_direct_flat_kernel_with_channels_and_frame(B, Cin, Cout, N, n, P):
    """The flat-output kernel on three input channels (the image layers of Tables 1-2) and on padded
    layers, whose zero frame it keeps in LDS: against the oracle, bit for bit on integers, with guard
    words around `out`, and reproducibly."""
    layer = wl.Layer("flat_ci", B, Cin, Cout, N, n, "f32", "normal", w_std=0.3)
    x, w = wl.make_tensors(layer, 800 + N + 7 * n + P)
    xd, w_seg = x.to(DEV), kst.kst_segregate_weights(w.to(DEV))
    got = kst.kst_forward_seg_padded(xd, w_seg, Cout, n, P, path=kst.KST_PATH_DIRECT)
    again = kst.kst_forward_seg_padded(xd, w_seg, Cout, n, P, path=kst.KST_PATH_DIRECT)
    torch.cuda.synchronize()
    assert torch.equal(got, again)
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w), P)
    e = rel_err(got.cpu().numpy(), want)
    assert e <= TOL["f32"], "rel err %.3e" % e
    check_exact_with_guards(wl.Layer("flat_ci_int", B, Cin, Cout, N, n, "f32", "integer"), kst.KST_PATH_DIRECT,
                            900 + N + n, P=P)
    # no framed copy of the input, and for an odd padding factor no wider result to copy the interior of
    # (the two small three-channel cases go to the multi-channel kernel, which supplies the frame too)
    assert kst.kst_workspace_bytes_padded(B, Cin, Cout, N, n, P, kst.KST_F32, kst.KST_PATH_DIRECT) == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Cin,Cout,N,n", [
    (5, 20, 150, 12, 4),    # 2 channel tiles (ragged), tiles straddle batch items
    (3, 37, 40, 17, 5),     # odd Cin, odd M
    (7, 64, 129, 8, 3),     # tiny maps: many batch items per tile, Cout one over a tile
    (2, 18, 32, 40, 3),     # large map: tiles are row strips of one item
    (9, 130, 16, 6, 4),     # reduction split across workgroups (few tiles)
    (2, 48, 64, 9, 7),
])
def test_igemm_multi_tile(B, Cin, Cout, N, n, dtype):
    layer = wl.Layer("mt", B, Cin, Cout, N, n, dtype, "relu_normal", w_std=0.1)
    # bf16 with a 7 x 7 kernel: the weight tile exceeds LDS, the matrix-core path declines it
    check_layer(layer, paths=("igemm", "auto", "forward", "direct"), seed=N * 7 + n,
                skip_unsupported_igemm=(n == 7 and dtype == "bf16"))


@pytest.mark.parametrize("B,Cin,Cout,N,n", [
    (3, 40, 130, 34, 4),    # E = 32: four quad rows per strip, ragged channel tile
    (2, 24, 40, 64, 2),     # E = 63 with an even kernel (M = 126)
    (1, 17, 33, 50, 1),     # n = 1, Cin not a multiple of 8 or 16
    (2, 9, 16, 128, 3),     # E = 127: one quad row per strip
    (2, 48, 32, 22, 3),     # E = 20: six quad rows per strip, last strip short
])
def test_igemm_bf16_row_strip_kernel(B, Cin, Cout, N, n):
    """bf16 maps whose quad rows hold 16..128 quads take the row-strip matrix-core kernel."""
    layer = wl.Layer("strip", B, Cin, Cout, N, n, "bf16", "relu_normal", w_std=0.1)
    check_layer(layer, paths=("igemm", "forward", "direct"), seed=N * 5 + n)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("B,Cin,Cout,N,n", [
    (2, 24, 40, 34, 4),     # E = 32: four quad rows per strip, ragged channel tile, ragged last chunk
    (1, 17, 33, 50, 1),     # n = 1: three empty sub-kernels whose zeros must be written
    (2, 48, 32, 22, 3),     # E = 21: six quad rows per strip, last strip short, odd M
    (1, 9, 16, 128, 3),     # E = 127: one quad row per strip
])
def test_igemm_bf16_row_strip_kernel_is_exact_on_integers_and_stays_inside_out(B, Cin, Cout, N, n, dtype):
    check_exact_with_guards(wl.Layer("strip_int", B, Cin, Cout, N, n, dtype, "integer"), kst.KST_PATH_IGEMM, 21 + N)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("B,Cin,Cout,N,n", [
    (5, 20, 150, 12, 4),    # 2 channel tiles (ragged), tiles straddle batch items
    (3, 37, 40, 17, 5),     # 5 x 5 kernel (the row-strip kernel stops at 4 x 4), odd Cin, odd M
    (7, 64, 129, 8, 3),     # tiny maps: many batch items per tile, Cout one over a tile
    (9, 130, 16, 6, 4),     # reduction split across workgroups (few tiles): partial sums and the summing pass
    (2, 24, 40, 9, 5),
    (3, 16, 16, 5, 2),
])
def test_igemm_bf16_plain_kernel_is_exact_on_integers_and_stays_inside_out(B, Cin, Cout, N, n, dtype):
    """Maps with fewer than 16 quads per row, odd maps and kernels beyond 4 x 4 take the first
    16-bit matrix-core kernel."""
    check_exact_with_guards(wl.Layer("plain_int", B, Cin, Cout, N, n, dtype, "integer"), kst.KST_PATH_IGEMM, 31 + N)


@pytest.mark.parametrize("B,Cin,Cout,N,n", [
    (2, 32, 64, 32, 3),     # E = 31: one column block, four quad rows per tile, last tile short
    (2, 48, 64, 32, 2),     # even kernel, three chunks
    (3, 16, 64, 64, 3),     # E = 63: two column blocks, a single chunk
    (1, 32, 128, 64, 2),    # two channel tiles
    (2, 16, 64, 32, 3),     # a single chunk
    (1, 64, 64, 64, 3),     # four chunks: the three-stage ring wraps
])
def test_igemm_bf16_lds_ring_kernel(B, Cin, Cout, N, n):
    """bf16 maps of 32 or 64 pixels a side with whole channel tiles take the kernel that
    fills an LDS ring with LDS-direct loads and fetches operands with transposing reads."""
    layer = wl.Layer("ring", B, Cin, Cout, N, n, "bf16", "relu_normal", w_std=0.1)
    check_layer(layer, paths=("igemm", "forward", "direct"), seed=N * 3 + n)


def test_igemm_bf16_lds_ring_kernel_is_exact_on_integers_and_stays_inside_out():
    """Small integers are exact in bf16 and in the fp32 accumulators, so the result must equal
    the oracle bit for bit; guard words around `out` must survive."""
    layer = wl.Layer("ring_int", 2, 32, 64, 64, 3, "bf16", "integer")
    x, w = wl.make_tensors(layer, 11)
    xd, wd = x.to(DEV), w.to(DEV)
    ws = kst.kst_segregate_weights(wd)
    numel = int(np.prod(layer.out_shape))
    guard = 4096
    buf = torch.full((numel + 2 * guard,), float("nan"), device=DEV)
    out = buf[guard:guard + numel].view(layer.out_shape)
    kst.kst_forward_seg(xd, ws, layer.Cout, layer.n, out=out, path=kst.KST_PATH_IGEMM)
    torch.cuda.synchronize()
    host = buf.cpu()
    assert torch.isnan(host[:guard]).all() and torch.isnan(host[guard + numel:]).all()
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w))
    assert np.array_equal(host[guard:guard + numel].view(layer.out_shape).numpy().astype(np.float64), want)


@pytest.mark.parametrize("B,Cin,Cout,N,n", [
    (4, 32, 256, 64, 3),     # 256 tiles of four quad rows x 64 channels, two chunks, last strip short
    (8, 96, 128, 64, 2),     # even kernel, six chunks: the five-stage ring wraps
    (32, 48, 128, 32, 3),    # one column block: a wave holds four quad rows
    (29, 112, 128, 32, 2),   # seven chunks, 232 tiles on 256 CUs
    (5, 16, 256, 64, 3),     # 320 tiles: some workgroups walk over two tiles; a single chunk
])
def test_igemm_bf16_wide_kernel(B, Cin, Cout, N, n):
    """Layers with at least about one tile per CU take the persistent wide-tile kernel
    (one wave per SIMD, 256 accumulators, fragments refreshed in place)."""
    layer = wl.Layer("wide", B, Cin, Cout, N, n, "bf16", "relu_normal", w_std=0.1)
    check_layer(layer, paths=("igemm", "forward"), seed=N * 7 + n)


def test_igemm_bf16_wide_kernel_is_exact_on_integers_and_stays_inside_out():
    """Small integers are exact in bf16 and in the fp32 accumulators, so the result must equal
    the oracle bit for bit, tile after tile of a persistent workgroup; guard words around
    `out` must survive."""
    layer = wl.Layer("wide_int", 5, 32, 256, 64, 3, "bf16", "integer")
    x, w = wl.make_tensors(layer, 13)
    xd, wd = x.to(DEV), w.to(DEV)
    ws = kst.kst_segregate_weights(wd)
    numel = int(np.prod(layer.out_shape))
    guard = 4096
    buf = torch.full((numel + 2 * guard,), float("nan"), device=DEV)
    out = buf[guard:guard + numel].view(layer.out_shape)
    kst.kst_forward_seg(xd, ws, layer.Cout, layer.n, out=out, path=kst.KST_PATH_IGEMM)
    torch.cuda.synchronize()
    host = buf.cpu()
    assert torch.isnan(host[:guard]).all() and torch.isnan(host[guard + numel:]).all()
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w))
    assert np.array_equal(host[guard:guard + numel].view(layer.out_shape).numpy().astype(np.float64), want)


@pytest.mark.parametrize("B,Cout,dtype,dist", [
    (7, 128, "bf16", "relu_normal"),     # 224 tiles: one per workgroup (first tile = last tile)
    (9, 128, "bf16", "relu_normal"),     # 288 tiles: some workgroups walk over two
    (5, 192, "f16", "relu_normal"),      # three channel tiles, half-precision multiply
    (7, 128, "bf16", "integer"),         # exact: must equal the oracle bit for bit
    (20, 64, "f16", "integer"),          # 320 tiles, one channel tile
])
def test_igemm_bf16_row_parity_passes_kernel(B, Cout, dtype, dist):
    """The forced path IGEMM_PASSES: the kernel that works a tile's even and odd output rows in two
    passes and drains one pass's rows while the other multiplies (3 x 3 kernels, 64 x 64 maps, 256
    input channels; not taken by AUTO: it measures slower than the wide-tile kernel).  Every
    batch item and every block of 32 channels is held to the oracle plane by plane, the whole tensor
    through channel projections; guard words around `out` must survive."""
    layer = wl.Layer("pp", B, 256, Cout, 64, 3, dtype, dist, w_std=0.1)
    x, w = wl.make_tensors(layer, 40 + B + Cout)
    xd, wd = x.to(DEV), w.to(DEV)
    numel = int(np.prod(layer.out_shape))
    guard = 4096
    buf = torch.full((numel + 2 * guard,), float("nan"), device=DEV)
    out = buf[guard:guard + numel].view(layer.out_shape)
    kst.kst_forward_seg(xd, kst.kst_segregate_weights(wd), Cout, 3, out=out, path=kst.KST_PATH_IGEMM_PASSES)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[guard + numel:]).all()
    assert torch.isfinite(out).all()
    again = torch.empty_like(out)
    kst.kst_forward_seg(xd, kst.kst_segregate_weights(wd), Cout, 3, out=again, path=kst.KST_PATH_IGEMM_PASSES)
    torch.cuda.synchronize()
    assert torch.equal(out, again)                     # fixed order everywhere: bit-reproducible
    b_idx, co_idx = covering_planes(B, Cout)
    check_planes(out, x, w, b_idx, co_idx, TOL[dtype], exact=(dist == "integer"))
    check_channel_projection(out, x, w, TOL[dtype], seed=B)
    # the kernel AUTO takes for the same layer agrees with it (both hold fp32 sums of exact products)
    auto = kst.kst_forward_seg(xd, kst.kst_segregate_weights(wd), Cout, 3, path=kst.KST_PATH_IGEMM)
    torch.cuda.synchronize()
    assert rel_err(out.cpu().numpy(), auto.cpu().numpy().astype(np.float64)) <= TOL[dtype]
    with pytest.raises(kst.KstError):                  # any other shape is refused
        kst.kst_forward_seg(xd[:, :128].contiguous(), kst.kst_segregate_weights(wd[:, :128].contiguous()), Cout, 3,
                            path=kst.KST_PATH_IGEMM_PASSES)


@pytest.mark.parametrize("B,Cin,Cout,N,n", [
    (32, 64, 768, 16, 4),    # 294 tiles x 16 chunks over 256 workgroups: whole tiles and partial pieces per range
    (8, 256, 128, 16, 4),    # 13 tiles x 64 chunks: every tile shared by about 20 workgroups
    (3, 100, 132, 12, 5),    # 6 tiles (ragged both ways) x 25 chunks: one chunk per workgroup
    (20, 32, 384, 12, 3),    # 264 tiles x 8 chunks, odd M: a round of whole tiles, then 8 tiles shared by 256 workgroups
    (84, 8, 256, 16, 4),     # 258 tiles x 2 chunks: a round of whole tiles, then 4 shared units for 256 workgroups
    (83, 8, 256, 16, 4),     # 256 tiles: whole tiles only, nothing shared and no second pass
    (16, 16, 256, 16, 4),    # 50 tiles x 4 chunks: fewer units than workgroups
    (40, 64, 64, 16, 4),     # tiles of 64 output channels: 62 tiles x 16 chunks
    (9, 40, 44, 12, 5),      # ... ragged in the channels (44 of 64), odd M: 8 tiles x 10 chunks
    (70, 16, 64, 32, 3),     # ... 526 tiles x 4 chunks: two rounds of whole tiles, then 14 tiles shared
])
def test_igemm_f32_even_shares(B, Cin, Cout, N, n):
    """fp32 matrix-core path where the (tile, chunk) list is cut into equal ranges: pieces that
    are whole tiles, pieces that go through the partial slots, and their sum in a second pass."""
    layer = wl.Layer("shares", B, Cin, Cout, N, n, "f32", "relu_normal", w_std=0.1)
    x, w = wl.make_tensors(layer, 900 + Cin + N)
    xd, wd = x.to(DEV), w.to(DEV)
    # two partial-tile slots per workgroup, one workgroup per CU or per unit; a slot is one tile's accumulators:
    # 128 positions x 4 classes x 128 output channels (64 for layers with up to 64 of them)
    M = 2 * N - n
    E = (M + 1) // 2
    tco = 64 if Cout <= 64 else 128
    units = ((B * E * E + 127) // 128) * ((Cout + tco - 1) // tco) * (Cin // 4)
    assert kst.kst_workspace_bytes(B, Cin, Cout, N, n, kst.KST_F32, kst.KST_PATH_IGEMM_EVEN) == \
        2 * min(256, units) * 128 * tco * 4 * 4
    out = kst.kst_forward_seg(xd, kst.kst_segregate_weights(wd), Cout, n, path=kst.KST_PATH_IGEMM_EVEN)
    again = kst.kst_forward_seg(xd, kst.kst_segregate_weights(wd), Cout, n, path=kst.KST_PATH_IGEMM_EVEN)
    whole = kst.kst_forward_seg(xd, kst.kst_segregate_weights(wd), Cout, n, path=kst.KST_PATH_IGEMM)
    torch.cuda.synchronize()
    assert rel_err(out.cpu().numpy(), whole.cpu().numpy().astype(np.float64)) <= TOL["f32"]
    assert torch.isfinite(out).all()
    assert torch.equal(out, again)                     # fixed summing order: bit-reproducible
    b_idx, co_idx = covering_planes(B, Cout)
    check_planes(out, x, w, b_idx, co_idx, TOL["f32"])
    check_channel_projection(out, x, w, TOL["f32"], seed=Cin)


def test_igemm_f32_even_shares_are_exact_on_integers_and_stay_inside_out():
    layer = wl.Layer("shares_int", 8, 256, 128, 16, 4, "f32", "integer")
    x, w = wl.make_tensors(layer, 12)
    xd, wd = x.to(DEV), w.to(DEV)
    numel = int(np.prod(layer.out_shape))
    guard = 4096
    buf = torch.full((numel + 2 * guard,), float("nan"), device=DEV)
    out = buf[guard:guard + numel].view(layer.out_shape)
    kst.kst_forward_seg(xd, kst.kst_segregate_weights(wd), layer.Cout, layer.n, out=out, path=kst.KST_PATH_IGEMM_EVEN)
    torch.cuda.synchronize()
    host = buf.cpu()
    assert torch.isnan(host[:guard]).all() and torch.isnan(host[guard + numel:]).all()
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w))
    assert np.array_equal(host[guard:guard + numel].view(layer.out_shape).numpy().astype(np.float64), want)


# ----------------------------------------------------------------------------
# Boundary behaviour: nothing outside `out` is written; results are reproducible
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("path", ["direct", "igemm"])
def test_no_write_outside_out_and_every_element_written(path):
    layer = wl.Layer("canary", 3, 16, 24, 13, 5, "f32", "normal", w_std=0.2)   # odd M = 21
    x, w = wl.make_tensors(layer, 5)
    xd, wd = x.to(DEV), w.to(DEV)
    ws = kst.kst_segregate_weights(wd)
    numel = int(np.prod(layer.out_shape))
    guard = 4096
    buf = torch.full((numel + 2 * guard,), float("nan"), device=DEV)
    out = buf[guard:guard + numel].view(layer.out_shape)
    code = kst.KST_PATH_DIRECT if path == "direct" else kst.KST_PATH_IGEMM
    kst.kst_forward_seg(xd, ws, layer.Cout, layer.n, out=out, path=code)
    torch.cuda.synchronize()
    host = buf.cpu()
    assert torch.isnan(host[:guard]).all() and torch.isnan(host[guard + numel:]).all()
    assert not torch.isnan(host[guard:guard + numel]).any()
    again = torch.empty_like(out)
    kst.kst_forward_seg(xd, ws, layer.Cout, layer.n, out=again, path=code)
    torch.cuda.synchronize()
    assert torch.equal(again, out)                     # no atomics: bit-reproducible


def test_runs_on_a_side_stream():
    layer = wl.Layer("stream", 2, 3, 2, 33, 3, "f32", "normal", w_std=0.2)
    x, w = wl.make_tensors(layer, 3)
    xd, wd = x.to(DEV), w.to(DEV)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        out = kst.kst_forward(xd, wd)
    s.synchronize()
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w))
    assert rel_err(out.cpu().numpy(), want) <= TOL["f32"]


# ----------------------------------------------------------------------------
# The five benchmark layers at full size, in the configuration bench.py times
# ----------------------------------------------------------------------------
def covering_planes(B, Cout, group=32):
    """Every batch item with one output channel of every `group` consecutive channels (the
    matrix-core kernels store blocks of 32 channels of tiles of 64 or 128); the channel inside
    the group moves with the batch item, so that over the batch every channel is visited."""
    b_idx, co_idx = [], []
    for b in range(B):
        for g0 in range(0, Cout, group):
            width = min(group, Cout - g0)
            b_idx.append(b)
            co_idx.append(g0 + (5 * b + 3 * (g0 // group)) % width)
    return b_idx, co_idx


def check_planes(out, x, w, b_idx, co_idx, tol, P=0, exact=False):
    want = oracle.forward_planes(wl.to_f64(x), wl.to_f64(w), b_idx, co_idx, P)
    got = out[torch.tensor(b_idx), torch.tensor(co_idx)].cpu().numpy()
    assert got.shape == want.shape
    if exact:
        assert np.array_equal(got.astype(np.float64), want)
    e = rel_err(got, want)
    assert e <= tol, "planes: rel err %.3e" % e


def check_channel_projection(out, x, w, tol, P=0, seed=0, count=2):
    """Every element of `out` against the oracle at the price of a one-channel layer: the
    operation is linear in the kernel, so sum_co r[co] * out[b][co] is the oracle's result for
    the single kernel sum_co r[co] * w[co].  Random normal r: a wrong, missing or misplaced
    value anywhere in the tensor changes the projection (two draws)."""
    rng = np.random.default_rng(77 + seed)
    x64, w64 = wl.to_f64(x), wl.to_f64(w)
    host = out.cpu().numpy()
    for _ in range(count):
        r = rng.standard_normal(w64.shape[0])
        want = oracle.forward(x64, np.einsum("o,oiuv->iuv", r, w64)[None], P)[:, 0]
        got = np.stack([np.einsum("o,oyx->yx", r, host[b].astype(np.float64)) for b in range(host.shape[0])])
        # the fp32 rounding of the summed channels adds up like the projection itself
        scale = np.abs(want).max()
        e = float(np.abs(got - want).max() / scale)
        assert e <= tol, "channel projection: rel err %.3e" % e


@pytest.mark.parametrize("idx", [0, 1])
def test_benchmark_layers_full_output(idx):
    layer = wl.LAYERS[idx]
    check_layer(layer, paths=("auto", "forward"))


@pytest.mark.parametrize("idx", [2, 3, 4])
def test_benchmark_layers_full_size(idx):
    """The many-channel benchmark layers at full size, in the launch configuration the bench
    times.  The whole output is held to the oracle twice: complete output planes for every batch
    item and every block of 32 output channels (computed from the definition), and every element
    through random projections over the output channels."""
    layer = wl.LAYERS[idx]
    x, w = wl.make_tensors(layer)
    xd, wd = x.to(DEV), w.to(DEV)
    w_seg = kst.kst_segregate_weights(wd)
    out_seg = kst.kst_forward_seg(xd, w_seg, layer.Cout, layer.n)
    out_fwd = kst.kst_forward(xd, wd)
    torch.cuda.synchronize()
    assert torch.equal(out_seg, out_fwd)
    assert torch.isfinite(out_seg).all()
    b_idx, co_idx = covering_planes(layer.B, layer.Cout)
    check_planes(out_seg, x, w, b_idx, co_idx, TOL[layer.dtype])
    check_channel_projection(out_seg, x, w, TOL[layer.dtype], seed=idx)


def test_zero_insert_reference_on_a_benchmark_layer():
    layer = wl.LAYERS[0]
    check_layer(layer, paths=("zero_insert",))


# ----------------------------------------------------------------------------
# Padding factor P (Section 3.3, Figs. 5-7)
# ----------------------------------------------------------------------------
def padded_outputs(layer, P, seed, paths):
    x, w = wl.make_tensors(layer, seed)
    xd, wd = x.to(DEV), w.to(DEV)
    res = {}
    for name in paths:
        if name == "forward":
            o = kst.kst_forward_padded(xd, wd, P)
        else:
            code = {"direct": kst.KST_PATH_DIRECT, "igemm": kst.KST_PATH_IGEMM, "auto": kst.KST_PATH_AUTO}[name]
            o = kst.kst_forward_seg_padded(xd, kst.kst_segregate_weights(wd), layer.Cout, layer.n, P, path=code)
        torch.cuda.synchronize()
        res[name] = o.cpu().numpy()
    return x, w, res


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Cin,Cout,N,n,P,paths", [
    (1, 1, 1, 4, 5, 2, ("direct", "auto", "forward")),            # Figs. 5-6: 4 x 4 input, 5 x 5 kernel, P = 2
    (1, 1, 1, 4, 5, 3, ("direct", "auto", "forward")),            # Fig. 7: the same with P = 3
    (2, 3, 4, 7, 3, 1, ("direct", "forward")),
    (2, 3, 4, 7, 3, 2, ("direct", "forward")),
    (1, 2, 3, 6, 4, 3, ("direct", "forward")),
    (2, 1, 1, 9, 5, 4, ("direct", "forward")),
    (1, 1, 2, 1, 5, 2, ("direct", "forward")),                    # a map the kernel only covers thanks to the frame
    (2, 16, 32, 16, 4, 2, ("igemm", "auto", "direct", "forward")),   # a GAN layer shape: 16 -> 32
    (2, 16, 32, 14, 4, 1, ("igemm", "direct")),
    (1, 24, 40, 12, 3, 4, ("igemm", "direct")),
    (1, 8, 16, 10, 5, 3, ("igemm", "direct", "forward")),
])
def test_padded_forward(B, Cin, Cout, N, n, P, paths, dtype):
    layer = wl.Layer("padded", B, Cin, Cout, N, n, dtype, "normal", w_std=0.2)
    x, w, res = padded_outputs(layer, P, 1000 + 13 * N + 7 * n + P, paths)
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w), P)
    M = kst.kst_out_size_padded(N, n, P)
    assert want.shape == (B, Cout, M, M)
    for name, got in res.items():
        assert got.shape == want.shape, name
        e = rel_err(got, want)
        assert e <= TOL[dtype], "%s: rel err %.3e" % (name, e)


def test_padded_forward_is_exact_on_integers_and_stays_inside_out():
    layer = wl.Layer("padded_int", 2, 3, 5, 9, 5, "f32", "integer")
    x, w = wl.make_tensors(layer, 77)
    xd, wd = x.to(DEV), w.to(DEV)
    for P in (1, 2, 3):
        M = kst.kst_out_size_padded(layer.N, layer.n, P)
        numel = layer.B * layer.Cout * M * M
        guard = 1024
        buf = torch.full((numel + 2 * guard,), float("nan"), device=DEV)
        out = buf[guard:guard + numel].view(layer.B, layer.Cout, M, M)
        kst.kst_forward_seg_padded(xd, kst.kst_segregate_weights(wd), layer.Cout, layer.n, P, out=out)
        torch.cuda.synchronize()
        host = buf.cpu()
        assert torch.isnan(host[:guard]).all() and torch.isnan(host[guard + numel:]).all()
        want = oracle.forward(wl.to_f64(x), wl.to_f64(w), P)
        assert np.array_equal(host[guard:guard + numel].view(out.shape).numpy().astype(np.float64), want)


@pytest.mark.parametrize("B,Cin,Cout,N,n,P,dtype", [
    (64, 512, 256, 16, 4, 2, "f32"),     # Table 3's 16 -> 32 generator layer at a benchmark batch size
    (4, 64, 128, 60, 3, 4, "bf16"),      # framed to 64 x 64: takes the LDS-ring kernel
    (16, 3, 1, 224, 5, 2, "f32"),        # Table 1's shape: 224 x 224 x 3 -> 447 x 447 x 1
    (8, 3, 1, 224, 4, 3, "f32"),         # the same with an odd padding factor
    (16, 3, 1, 224, 3, 2, "f32"),        # Table 1's 3 x 3 kernel: 449 x 449 x 1
    (256, 3, 1, 224, 3, 2, "f32"),       # the same at the batch the bench times: the flat-output kernel, three channels
    (256, 3, 1, 224, 5, 2, "f32"),
    (64, 128, 3, 32, 4, 2, "f32"),       # Table 3's output layer at the bench's batch: four lane groups per tile
    (1, 2048, 1024, 4, 4, 2, "f32"),     # EB-GAN's first layer on one sample: position blocks of 16
])
def test_padded_forward_full_size(B, Cin, Cout, N, n, P, dtype):
    layer = wl.Layer("padded_full", B, Cin, Cout, N, n, dtype, "relu_normal")
    x, w = wl.make_tensors(layer, 4242 + N + P)
    xd, wd = x.to(DEV), w.to(DEV)
    out = kst.kst_forward_padded(xd, wd, P)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    b_idx, co_idx = covering_planes(B, Cout)
    check_planes(out, x, w, b_idx, co_idx, TOL[dtype], P=P)
    if Cout > 1:                                             # (with one output channel the planes are the whole tensor)
        check_channel_projection(out, x, w, TOL[dtype], P=P, seed=N + P)


@pytest.mark.parametrize("B,Cin,Cout,N,n,P,dtype,path", [
    (16, 32, 128, 16, 4, 1, "f32", kst.KST_PATH_IGEMM),        # pipelined fp32 kernel, whole tiles
    (2, 64, 128, 8, 4, 3, "f32", kst.KST_PATH_IGEMM),          # split reduction + summing pass
    (1, 512, 128, 4, 4, 1, "f32", kst.KST_PATH_IGEMM),         # one sample: 64+ splits
    (2, 512, 128, 8, 4, 1, "f32", kst.KST_PATH_IGEMM_EVEN),    # even shares: slots + slot-summing pass
    (2, 18, 40, 9, 3, 3, "f32", kst.KST_PATH_IGEMM),           # first fp32 kernel (ragged channels), odd map
    (3, 24, 150, 12, 5, 1, "f32", kst.KST_PATH_IGEMM),         # 5 x 5, ragged channel tile
    (9, 130, 16, 6, 4, 1, "bf16", kst.KST_PATH_IGEMM),         # first 16-bit kernel, split reduction
    (3, 37, 40, 17, 5, 3, "f16", kst.KST_PATH_IGEMM),          # first 16-bit kernel, whole tiles
    (2, 48, 64, 30, 2, 1, "bf16", kst.KST_PATH_IGEMM),         # LDS-ring kernel: keeps the wider buffer and the copy
])
def test_odd_padding_factor_on_the_matrix_cores(B, Cin, Cout, N, n, P, dtype, path):
    """Odd padding factors (Fig. 7): the kernels whose accumulators go straight to memory write the
    interior of the wider map directly (no wider workspace buffer, no copy); against the oracle,
    bit for bit on integers, with guard words around `out`."""
    layer = wl.Layer("odd_p", B, Cin, Cout, N, n, dtype, "relu_normal", w_std=0.1)
    x, w = wl.make_tensors(layer, 1300 + N + n + P)
    code = {"f32": kst.KST_F32, "bf16": kst.KST_BF16, "f16": kst.KST_F16}[dtype]
    got = kst.kst_forward_seg_padded(x.to(DEV), kst.kst_segregate_weights(w.to(DEV)), Cout, n, P, path=path)
    torch.cuda.synchronize()
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w), P)
    assert got.shape == want.shape
    e = rel_err(got.cpu().numpy(), want)
    assert e <= TOL[dtype], "rel err %.3e" % e
    check_exact_with_guards(wl.Layer("odd_p_int", B, Cin, Cout, N, n, dtype, "integer"), path, 1400 + N, P=P)
    M = kst.kst_out_size_padded(N, n, P)
    wider = B * Cout * (M + 2) * (M + 2) * 4
    need = kst.kst_workspace_bytes_padded(B, Cin, Cout, N, n, P, code, path)
    even = kst.kst_workspace_bytes_padded(B, Cin, Cout, N, n, P + 1, code, path)
    if N == 30:
        assert need >= wider                      # that kernel leaves through an LDS image of whole rows
    else:
        assert need <= even + 4096                # nothing beyond what the even padding factor above it needs


@pytest.mark.parametrize("B,Cin,Cout,N,n,P", [
    (1, 1024, 512, 4, 4, 2),    # Table 3, DCGAN layer 2 on one sample: 16 positions, one block
    (1, 512, 256, 8, 4, 2),     # ... layer 3: 64 positions, four blocks
    (1, 256, 128, 4, 4, 0),     # no padding: E = 2, four positions of a block's sixteen
    (3, 128, 80, 3, 3, 2),      # three samples, 3 x 3 kernel, odd map, ragged channel block (80 = 64 + 16)
    (2, 64, 16, 4, 5, 3),       # odd padding factor (stores shifted by one), 5 x 5 kernel, smallest channel counts
    (1, 132, 72, 6, 2, 1),      # 2 x 2 kernel, odd padding factor, channel counts that are no powers of two
    (4, 96, 64, 3, 1, 0),       # n = 1: three empty classes whose zeros must be written
    (1, 2048, 1024, 4, 4, 2),   # Table 3, EB-GAN layer 2: 134 MB of weights
    (1, 256, 128, 16, 4, 2),    # Table 3, DCGAN layer 4 on one sample: 256 positions
    (1, 256, 128, 32, 4, 2),    # Table 3, EB-GAN layer 5: 1024 positions -- 64 blocks x 2 MB of weights, just past what the position-block kernel takes: tiles
    (5, 64, 48, 13, 3, 1),      # 5 x 14 x 14 = 980 positions, ragged last block, odd padding factor
    (1, 128, 3, 32, 4, 2),      # Table 3, the generators' output layer on one sample: three of a block's 64 channels
    (1, 64, 5, 16, 3, 1),       # five output channels (weights read one value at a time), odd padding factor
    (1, 128, 64, 64, 4, 2),     # Table 3, EB-GAN layer 6: 4096 positions, half a megabyte of weights (tiles of 64 channels)
    (8, 64, 64, 32, 4, 2),      # a small batch of such a layer: 8192 positions (tiles of 64 channels)
    (2, 64, 32, 32, 3, 2),      # 2178 positions in 137 blocks, 74 KB of weights: position blocks, ragged last block, half a channel block
    (2, 256, 80, 6, 3, 3),      # four waves per workgroup (64 chunks): ragged channel block, ragged position block, odd padding factor
    (1, 384, 5, 8, 4, 1),       # ... with five output channels (weights read one value at a time), 96 chunks in three splits
    (1, 1100, 64, 8, 4, 2),     # ... a chunk count (275: nine per workgroup) that four waves cannot share evenly
])
def test_matrix_cores_on_very_few_positions(B, Cin, Cout, N, n, P):
    """Layers with few quad positions in all (or small weights) take position blocks of 16 on the matrix cores,
    their reduction split over the chip: against the oracle, reproducible, bit for bit on
    integers with guard words around `out`."""
    layer = wl.Layer("small", B, Cin, Cout, N, n, "f32", "relu_normal", w_std=0.05)
    x, w = wl.make_tensors(layer, 1500 + Cin + n + P)
    xd, w_seg = x.to(DEV), kst.kst_segregate_weights(w.to(DEV))
    got = kst.kst_forward_seg_padded(xd, w_seg, Cout, n, P, path=kst.KST_PATH_IGEMM)
    again = kst.kst_forward_seg_padded(xd, w_seg, Cout, n, P, path=kst.KST_PATH_IGEMM)
    torch.cuda.synchronize()
    assert torch.equal(got, again)
    if Cin * Cout > 600_000:
        b_idx, co_idx = covering_planes(B, Cout, group=8)
        check_planes(got, x, w, b_idx, co_idx, TOL["f32"], P=P)
        check_channel_projection(got, x, w, TOL["f32"], P=P, seed=Cin)
    else:
        want = oracle.forward(wl.to_f64(x), wl.to_f64(w), P)
        e = rel_err(got.cpu().numpy(), want)
        assert e <= TOL["f32"], "rel err %.3e" % e
        check_exact_with_guards(wl.Layer("small_int", B, Cin, Cout, N, n, "f32", "integer"), kst.KST_PATH_IGEMM,
                                1600 + Cin, P=P)


TABLE3_CASES = [(m, i) for m in wl.TABLE3_GENERATORS for i in range(len(wl.TABLE3_GENERATORS[m]))]


@pytest.mark.parametrize("model,index", TABLE3_CASES, ids=["%s-%d" % c for c in TABLE3_CASES])
def test_table3_generator_layers_one_sample(model, index):
    """Every transpose-convolution layer Table 3 lists (four generator families), on one input
    sample as the paper times them, through the entry point that takes unsegregated weights."""
    layer, _ = wl.table3_layers(model, 1)[index]
    x, w = wl.make_tensors(layer, 9000 + 31 * index + len(model))
    out = kst.kst_forward_padded(x.to(DEV), w.to(DEV), layer.P)
    torch.cuda.synchronize()
    assert tuple(out.shape) == layer.out_shape and layer.M == 2 * layer.N
    assert torch.isfinite(out).all()
    if layer.Cin * layer.Cout * layer.M * layer.M * 16 <= 600_000_000:
        want = oracle.forward(wl.to_f64(x), wl.to_f64(w), layer.P)
        e = rel_err(out.cpu().numpy(), want)
        assert e <= TOL["f32"], "%s: rel err %.3e" % (layer.name, e)
    else:
        # one plane of every block of 8 output channels, and two projections over all of them
        b_idx, co_idx = covering_planes(1, layer.Cout, group=8)
        check_planes(out, x, w, b_idx, co_idx, TOL["f32"], P=layer.P)
        check_channel_projection(out, x, w, TOL["f32"], P=layer.P, seed=index)


# ----------------------------------------------------------------------------
# Gradients (end of Section 3.3)
# ----------------------------------------------------------------------------
GRAD_TOL = {"f32": 2e-5, "bf16": 2e-5, "f16": 2e-5}     # operands are exact in both cases; the sums are fp32


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Cin,Cout,N,n,P", [
    (1, 1, 1, 4, 5, 2),      # Figs. 5-6 shape
    (1, 1, 1, 4, 5, 3),      # Fig. 7 shape
    (2, 3, 4, 7, 3, 0),
    (2, 3, 4, 6, 4, 0),
    (2, 5, 2, 9, 5, 0),
    (1, 2, 3, 8, 1, 0),
    (2, 3, 2, 5, 2, 1),
    (2, 16, 32, 16, 4, 2),   # a generator layer shape
    (3, 8, 24, 12, 3, 4),
    (1, 40, 72, 10, 5, 0),
    (1, 2, 2, 1, 5, 2),
    (1, 2, 3, 7, 9, 3),      # 9 x 9: the plain kernels on a framed copy, result cropped; odd padding factor
    (2, 2, 2, 6, 8, 2),
])
def test_gradients(B, Cin, Cout, N, n, P, dtype):
    layer = wl.Layer("grad", B, Cin, Cout, N, n, dtype, "normal", w_std=0.2, P=P)
    x, w = wl.make_tensors(layer, 3000 + 13 * N + 7 * n + P)
    M = kst.kst_out_size_padded(N, n, P)
    gen = torch.Generator().manual_seed(17 * N + n + P)
    g = torch.randn((B, Cout, M, M), generator=gen, dtype=torch.float32)
    din = kst.kst_backward_input(g.to(DEV), w.to(DEV), N, P)
    dw = kst.kst_backward_weight(x.to(DEV), g.to(DEV), n, P)
    torch.cuda.synchronize()
    want_din = oracle.backward_input(g.numpy().astype(np.float64), wl.to_f64(w), N, P)
    want_dw = oracle.backward_weight(wl.to_f64(x), g.numpy().astype(np.float64), n, P)
    assert din.shape == want_din.shape and dw.shape == want_dw.shape
    assert rel_err(din.cpu().numpy(), want_din) <= GRAD_TOL[dtype]
    assert rel_err(dw.cpu().numpy(), want_dw) <= GRAD_TOL[dtype]


@pytest.mark.parametrize("B,Cin,Cout,N,n,P", [
    (4, 136, 72, 16, 4, 2),    # two channel tiles, the second ragged; eleven position tiles
    (64, 32, 16, 8, 4, 2),     # tiles that span several batch items
    (2, 16, 264, 6, 5, 1),     # odd padding factor, long reduction: split over launches
    (3, 24, 40, 33, 3, 0),     # odd map, position tiles cut rows
    (2, 8, 8, 20, 2, 0),
    (2, 9, 11, 12, 1, 0),
    (1, 128, 128, 64, 4, 2),   # one row pair per tile
    (8, 40, 48, 4, 4, 2),      # 4 x 4 maps (a generator's first layers): the kernel gradient takes a whole framed map per chunk
    (3, 16, 24, 6, 5, 0),      # 5 x 5 kernel on 6 x 6 maps: three rows per chunk
    (2, 48, 16, 8, 3, 0),      # two channel blocks, two wave quartets, four rows of 8 per chunk
    (2, 80, 9, 18, 2, 1),      # ... rows of 18 cut 10 + 8, two rows per chunk, odd padding factor
    (2, 40, 16, 7, 3, 1),      # two channel blocks on an odd map: one quartet, one row per chunk
])
def test_gradients_on_the_matrix_cores(B, Cin, Cout, N, n, P):
    """fp32 layers with at least 8 channels on either side take the MFMA gradient kernels."""
    layer = wl.Layer("grad_mfma", B, Cin, Cout, N, n, "f32", "normal", w_std=0.2, P=P)
    x, w = wl.make_tensors(layer, 4000 + 13 * N + 7 * n + P)
    M = kst.kst_out_size_padded(N, n, P)
    gen = torch.Generator().manual_seed(19 * N + n + P)
    g = torch.randn((B, Cout, M, M), generator=gen, dtype=torch.float32)
    din = kst.kst_backward_input(g.to(DEV), w.to(DEV), N, P)
    dw = kst.kst_backward_weight(x.to(DEV), g.to(DEV), n, P)
    torch.cuda.synchronize()
    want = oracle.backward_input(g.numpy().astype(np.float64), wl.to_f64(w), N, P)
    assert din.shape == want.shape
    assert rel_err(din.cpu().numpy(), want) <= GRAD_TOL["f32"]
    want_dw = oracle.backward_weight(wl.to_f64(x), g.numpy().astype(np.float64), n, P)
    assert dw.shape == want_dw.shape
    assert rel_err(dw.cpu().numpy(), want_dw) <= GRAD_TOL["f32"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Cin,Cout,N,n,P", [
    (4, 3, 1, 40, 5, 2),       # few channels, many positions: the kernel gradient slices the positions
    (2, 3, 2, 63, 3, 0),
    (16, 1, 1, 33, 4, 1),
    (2, 128, 3, 8, 4, 2),      # many input, few output channels (a generator's last layer): lanes are channels
    (1, 70, 5, 6, 3, 0),       # a ragged second group of 64 channels, one output channel per wave
    (2, 64, 2, 5, 5, 1),       # 5 x 5: two output channels per wave; odd padding factor
    (1, 48, 4, 4, 7, 0),       # 7 x 7: one output channel per wave
    (3, 9, 12, 11, 4, 3),      # input gradient in several passes of 4 output channels, ragged channel group
    (1, 20, 6, 9, 6, 0),
    (3, 100, 7, 9, 2, 1),      # matrix cores with (channel, kernel element) rows: odd map, one row per chunk
    (2, 96, 3, 12, 3, 2),      # ... two quartets, two rows of 12 per chunk
    (2, 64, 6, 16, 4, 0),      # ... 96 rows in three waves
    (2, 64, 3, 6, 1, 0),       # ... 1 x 1 kernels: the rows are the output channels
])
def test_gradients_of_few_channel_layers(B, Cin, Cout, N, n, P, dtype):
    layer = wl.Layer("grad_few", B, Cin, Cout, N, n, dtype, "normal", w_std=0.2, P=P)
    x, w = wl.make_tensors(layer, 5000 + 13 * N + 7 * n + P)
    M = kst.kst_out_size_padded(N, n, P)
    gen = torch.Generator().manual_seed(23 * N + n + P)
    g = torch.randn((B, Cout, M, M), generator=gen, dtype=torch.float32)
    din = kst.kst_backward_input(g.to(DEV), w.to(DEV), N, P)
    dw = kst.kst_backward_weight(x.to(DEV), g.to(DEV), n, P)
    torch.cuda.synchronize()
    want_din = oracle.backward_input(g.numpy().astype(np.float64), wl.to_f64(w), N, P)
    want_dw = oracle.backward_weight(wl.to_f64(x), g.numpy().astype(np.float64), n, P)
    assert rel_err(din.cpu().numpy(), want_din) <= GRAD_TOL[dtype]
    assert rel_err(dw.cpu().numpy(), want_dw) <= GRAD_TOL[dtype]


@pytest.mark.parametrize("B,Cin,Cout,N,n,P,dtype", [
    (6, 3, 1, 224, 3, 2, "f32"),     # Table 1's layer: 28 strips of 8 rows per image, 168 persistent workgroups
    (6, 3, 1, 224, 5, 2, "f32"),     # ... 5 x 5 kernel: 75 sums per lane
    (6, 3, 1, 224, 4, 2, "bf16"),    # ... 16-bit input
    (8, 3, 2, 192, 4, 1, "f32"),     # odd padding factor, two output channels
    (5, 4, 1, 256, 3, 0, "f32"),     # no padding (margins of two zero columns), a map as wide as the workgroup
    (3, 1, 1, 320, 7, 2, "f32"),     # 7 x 7 kernel, one channel, a map wider than the workgroup
    (8, 2, 3, 200, 6, 4, "f32"),     # 6 x 6 kernel, padding factor 4, three output channels
    (5, 3, 1, 228, 5, 0, "bf16"),    # last strip of four rows; taps beyond every edge of the map
    (600, 3, 1, 64, 3, 2, "f32"),    # many small images: more strips than workgroups
])
def test_kernel_gradient_of_image_layers(B, Cin, Cout, N, n, P, dtype):
    """Few channels on large maps: rows of `in` and `g` staged through LDS, one partial result per workgroup."""
    layer = wl.Layer("grad_image", B, Cin, Cout, N, n, dtype, "normal", w_std=0.2, P=P)
    x, w = wl.make_tensors(layer, 5100 + 3 * N + 7 * n + P)
    M = kst.kst_out_size_padded(N, n, P)
    gen = torch.Generator().manual_seed(29 * N + n + P)
    g = torch.randn((B, Cout, M, M), generator=gen, dtype=torch.float32)
    dw = kst.kst_backward_weight(x.to(DEV), g.to(DEV), n, P)
    again = kst.kst_backward_weight(x.to(DEV), g.to(DEV), n, P)
    din = kst.kst_backward_input(g.to(DEV), w.to(DEV), N, P)    # (one output channel, maps up to 512 wide: the same strips)
    torch.cuda.synchronize()
    want_dw = oracle.backward_weight(wl.to_f64(x), g.numpy().astype(np.float64), n, P)
    assert rel_err(dw.cpu().numpy(), want_dw) <= GRAD_TOL[dtype]
    assert torch.equal(dw, again)                      # fixed summing order: bit-reproducible
    want_din = oracle.backward_input(g.numpy().astype(np.float64), wl.to_f64(w), N, P)
    assert din.shape == want_din.shape
    assert rel_err(din.cpu().numpy(), want_din) <= GRAD_TOL[dtype]


@pytest.mark.parametrize("B,Cin,Cout,N,n,P", [
    (3, 24, 16, 10, 5, 2),     # one block of input channels per workgroup
    (2, 72, 40, 6, 3, 1),      # two blocks, the second tile's second block empty; three rows per chunk
    (2, 40, 9, 9, 4, 0),       # two blocks, the second ragged; ragged output channels
])
def test_gradients_on_the_matrix_cores_are_exact_on_integers_and_stay_inside_their_outputs(B, Cin, Cout, N, n, P):
    layer = wl.Layer("grad_mfma_int", B, Cin, Cout, N, n, "f32", "integer", P=P)
    x, w = wl.make_tensors(layer, 98)
    M = kst.kst_out_size_padded(N, n, P)
    gen = torch.Generator().manual_seed(6)
    g = torch.randint(-3, 4, (B, Cout, M, M), generator=gen).to(torch.float32)
    numel = B * Cin * N * N
    guard = 1024
    buf = torch.full((numel + 2 * guard,), float("nan"), device=DEV)
    din = buf[guard:guard + numel].view(B, Cin, N, N)
    kst.kst_backward_input(g.to(DEV), w.to(DEV), N, P, din=din)
    wn = Cout * Cin * n * n
    wbuf = torch.full((wn + 2 * guard,), float("nan"), device=DEV)
    dw = wbuf[guard:guard + wn].view(Cout, Cin, n, n)
    kst.kst_backward_weight(x.to(DEV), g.to(DEV), n, P, dw=dw)
    torch.cuda.synchronize()
    host = buf.cpu()
    assert torch.isnan(host[:guard]).all() and torch.isnan(host[guard + numel:]).all()
    want = oracle.backward_input(g.numpy().astype(np.float64), wl.to_f64(w), N, P)
    assert np.array_equal(host[guard:guard + numel].view(B, Cin, N, N).numpy().astype(np.float64), want)
    whost = wbuf.cpu()
    assert torch.isnan(whost[:guard]).all() and torch.isnan(whost[guard + wn:]).all()
    want_dw = oracle.backward_weight(wl.to_f64(x), g.numpy().astype(np.float64), n, P)
    assert np.array_equal(whost[guard:guard + wn].view(Cout, Cin, n, n).numpy().astype(np.float64), want_dw)


@pytest.mark.parametrize("B,Cin,Cout,N,n,P", [
    (2, 3, 4, 9, 5, 2),        # lanes are positions (kernel gradient), one pass of output channels (input gradient)
    (2, 80, 3, 7, 4, 2),       # lanes are input channels
    (1, 10, 9, 6, 3, 1),
])
def test_gradients_are_exact_on_integers(B, Cin, Cout, N, n, P):
    layer = wl.Layer("grad_int", B, Cin, Cout, N, n, "f32", "integer", P=P)
    x, w = wl.make_tensors(layer, 99)
    M = kst.kst_out_size_padded(layer.N, layer.n, layer.P)
    gen = torch.Generator().manual_seed(5)
    g = torch.randint(-3, 4, (B, Cout, M, M), generator=gen).to(torch.float32)
    guard = 512
    din_buf = torch.full((B * Cin * N * N + 2 * guard,), float("nan"), device=DEV)
    dw_buf = torch.full((Cout * Cin * n * n + 2 * guard,), float("nan"), device=DEV)
    din = din_buf[guard:-guard].view(B, Cin, N, N)
    dw = dw_buf[guard:-guard].view(Cout, Cin, n, n)
    kst.kst_backward_input(g.to(DEV), w.to(DEV), layer.N, layer.P, din=din)
    kst.kst_backward_weight(x.to(DEV), g.to(DEV), layer.n, layer.P, dw=dw)
    torch.cuda.synchronize()
    for buf in (din_buf.cpu(), dw_buf.cpu()):
        assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[-guard:]).all()
    assert np.array_equal(din.cpu().numpy().astype(np.float64),
                          oracle.backward_input(g.numpy().astype(np.float64), wl.to_f64(w), layer.N, layer.P))
    assert np.array_equal(dw.cpu().numpy().astype(np.float64),
                          oracle.backward_weight(wl.to_f64(x), g.numpy().astype(np.float64), layer.n, layer.P))


def _seeded_gradient_shapes(count, seed):
    """Small layers that between them reach every chunk size, row count, channel-block count and
    row mode of the matrix-core gradient kernels (seeded: the same list on every run)."""
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        n = int(rng.integers(1, 6))
        N = int(rng.choice([2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 14, 16, 18, 21, 24, 32, 33]))
        P = int(rng.integers(0, 4))
        if 2 * N + 2 * P - n < 1:
            continue
        Cin = int(rng.choice([8, 24, 33, 40, 64, 72, 100]))
        Cout = int(rng.choice([2, 3, 5, 8, 9, 24, 40]))
        if Cout < 8 and Cin < 64:
            Cin = 64                                             # few output channels: the folded rows need 64 inputs
        B = int(rng.integers(1, 4))
        if B * Cin * Cout * N * N * n * n > 6e8:                 # keeps the oracle to a second or two per case
            continue
        shapes.append((B, Cin, Cout, N, n, P))
    return shapes


@pytest.mark.parametrize("B,Cin,Cout,N,n,P", _seeded_gradient_shapes(40, 20260511))
def test_gradients_on_the_matrix_cores_seeded_shapes(B, Cin, Cout, N, n, P):
    layer = wl.Layer("grad_seeded", B, Cin, Cout, N, n, "f32", "normal", w_std=0.2, P=P)
    x, w = wl.make_tensors(layer, 7000 + 31 * N + 7 * n + P + Cin)
    M = kst.kst_out_size_padded(N, n, P)
    gen = torch.Generator().manual_seed(29 * N + n + P + Cout)
    g = torch.randn((B, Cout, M, M), generator=gen, dtype=torch.float32)
    din = kst.kst_backward_input(g.to(DEV), w.to(DEV), N, P)
    dw = kst.kst_backward_weight(x.to(DEV), g.to(DEV), n, P)
    torch.cuda.synchronize()
    want_din = oracle.backward_input(g.numpy().astype(np.float64), wl.to_f64(w), N, P)
    want_dw = oracle.backward_weight(wl.to_f64(x), g.numpy().astype(np.float64), n, P)
    assert rel_err(din.cpu().numpy(), want_din) <= GRAD_TOL["f32"]
    assert rel_err(dw.cpu().numpy(), want_dw) <= GRAD_TOL["f32"]


def _seeded_few_channel_shapes(count, seed):
    """Layers the register-blocked gradient kernels take: every kernel size up to 7, one to several
    channels per workgroup, ragged channel groups, with and without a padding factor."""
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        n = int(rng.integers(1, 8))
        N = int(rng.choice([1, 2, 3, 5, 8, 11, 17, 30, 45]))
        P = int(rng.integers(0, 4))
        if 2 * N + 2 * P - n < 1:
            continue
        Cin = int(rng.choice([1, 2, 3, 4, 5, 7, 9, 20, 50, 70]))
        Cout = int(rng.choice([1, 2, 3, 4, 6, 7])) if Cin >= 8 else int(rng.choice([1, 2, 3, 4, 6, 12, 33]))
        B = int(rng.integers(1, 5))
        dtype = "bf16" if rng.integers(0, 3) == 0 else "f32"
        if B * Cin * Cout * N * N * n * n > 3e8:
            continue
        shapes.append((B, Cin, Cout, N, n, P, dtype))
    return shapes


@pytest.mark.parametrize("B,Cin,Cout,N,n,P,dtype", _seeded_few_channel_shapes(36, 20260512))
def test_gradients_of_few_channel_layers_seeded_shapes(B, Cin, Cout, N, n, P, dtype):
    layer = wl.Layer("grad_few_seeded", B, Cin, Cout, N, n, dtype, "normal", w_std=0.2, P=P)
    x, w = wl.make_tensors(layer, 8000 + 31 * N + 7 * n + P + Cin)
    M = kst.kst_out_size_padded(N, n, P)
    gen = torch.Generator().manual_seed(37 * N + n + P + Cout)
    g = torch.randn((B, Cout, M, M), generator=gen, dtype=torch.float32)
    din = kst.kst_backward_input(g.to(DEV), w.to(DEV), N, P)
    dw = kst.kst_backward_weight(x.to(DEV), g.to(DEV), n, P)
    torch.cuda.synchronize()
    want_din = oracle.backward_input(g.numpy().astype(np.float64), wl.to_f64(w), N, P)
    want_dw = oracle.backward_weight(wl.to_f64(x), g.numpy().astype(np.float64), n, P)
    assert rel_err(din.cpu().numpy(), want_din) <= GRAD_TOL[dtype]
    assert rel_err(dw.cpu().numpy(), want_dw) <= GRAD_TOL[dtype]


def _seeded_forward_shapes(count, seed):
    """Forward layers over every kernel size up to 7, both operand types, padding factors 0-3 and
    channel counts on both sides of every path's limits."""
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        n = int(rng.integers(1, 8))
        N = int(rng.choice([1, 2, 3, 5, 8, 9, 16, 17, 31, 40, 64]))
        P = int(rng.integers(0, 4))
        if 2 * N + 2 * P - n < 1:
            continue
        Cin = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16, 24, 40, 64, 136]))
        Cout = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 32, 40, 132]))
        B = int(rng.integers(1, 4))
        dtype = "bf16" if rng.integers(0, 3) == 0 else "f32"
        if B * Cin * Cout * N * N * n * n > 3e8:
            continue
        shapes.append((B, Cin, Cout, N, n, P, dtype))
    return shapes


@pytest.mark.parametrize("B,Cin,Cout,N,n,P,dtype", _seeded_forward_shapes(40, 20260513))
def test_forward_seeded_shapes_on_every_path_that_takes_them(B, Cin, Cout, N, n, P, dtype):
    layer = wl.Layer("fwd_seeded", B, Cin, Cout, N, n, dtype, "normal", w_std=0.2)
    x, w = wl.make_tensors(layer, 9000 + 31 * N + 7 * n + P + Cin)
    xd, wd = x.to(DEV), w.to(DEV)
    w_seg = kst.kst_segregate_weights(wd)
    want = oracle.forward(wl.to_f64(x), wl.to_f64(w), P)
    ran = []
    for name, code in (("auto", kst.KST_PATH_AUTO), ("direct", kst.KST_PATH_DIRECT), ("igemm", kst.KST_PATH_IGEMM),
                       ("even", kst.KST_PATH_IGEMM_EVEN)):
        try:
            got = kst.kst_forward_seg_padded(xd, w_seg, Cout, n, P, path=code)
        except kst.KstError:
            assert name in ("igemm", "even"), name               # only the matrix-core paths may refuse a layer
            continue
        torch.cuda.synchronize()
        ran.append(name)
        e = rel_err(got.cpu().numpy(), want)
        assert e <= TOL[dtype], "%s: rel err %.3e" % (name, e)
    assert "auto" in ran and "direct" in ran


def _seeded_narrow_and_tap_major_shapes(count, seed):
    """fp32 layers aimed at the matrix-core kernels' tile choices: 8 to 64 output channels (tiles of 64
    channels), few wide tiles (a halved split), batches of layers with one to four output channels and
    32 k input channels (taps as the rows of the product), weights around the limit between position
    blocks and tiles -- every padding factor form, random bias and activation."""
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        kind = int(rng.integers(0, 3))
        n = int(rng.integers(2, 6))
        P = int(rng.integers(0, 5))
        if kind == 0:                                   # tiles of 64 output channels
            N = int(rng.choice([4, 8, 12, 16, 20, 32]))
            Cin = int(rng.choice([8, 16, 32, 64, 128]))
            Cout = int(rng.choice([8, 12, 16, 32, 48, 64]))
            B = int(rng.integers(1, 40))
        elif kind == 1:                                 # more than 64 output channels, few tiles
            N = int(rng.choice([4, 8, 16]))
            Cin = int(rng.choice([64, 128, 256]))
            Cout = int(rng.choice([128, 192, 256]))
            B = int(rng.integers(1, 24))
        else:                                           # taps as rows: at least 128 workgroups
            N = int(rng.choice([8, 16, 32, 48]))
            Cin = int(rng.choice([64, 96, 128]))
            Cout = int(rng.integers(1, 5))
            if n * n * Cout > 64:
                continue
            M = 2 * N + 2 * P - n
            B = int(rng.integers(1, 3)) * (128 // max(1, (M + 15) // 16) + 1)
        if 2 * N - 1 + 2 * P < n:
            continue
        if B * Cin * Cout * (2 * N + 2 * P) ** 2 * n * n > 6e9:
            continue
        shapes.append((B, Cin, Cout, N, n, P, int(rng.integers(0, 3)), bool(rng.integers(0, 2))))
    return shapes


@pytest.mark.parametrize("B,Cin,Cout,N,n,P,act,bias", _seeded_narrow_and_tap_major_shapes(36, 20261129))
def test_seeded_matrix_core_tile_choices_with_bias_and_activation(B, Cin, Cout, N, n, P, act, bias):
    layer = wl.Layer("tiles_seeded", B, Cin, Cout, N, n, "f32", "relu_normal", w_std=0.1)
    x, w = wl.make_tensors(layer, 9700 + 31 * N + 7 * n + P + Cin + Cout)
    gen = torch.Generator().manual_seed(N + n + P + Cout)
    bvec = torch.randn((Cout,), generator=gen, dtype=torch.float32) if bias else None
    b64 = None if bvec is None else bvec.numpy().astype(np.float64)
    xd, w_seg = x.to(DEV), kst.kst_segregate_weights(w.to(DEV))
    want = oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), b64, act, P)
    scale = max(1.0, np.abs(oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), b64, 0, P)).max())
    ran = []
    for name, code in (("auto", kst.KST_PATH_AUTO), ("direct", kst.KST_PATH_DIRECT), ("igemm", kst.KST_PATH_IGEMM),
                       ("even", kst.KST_PATH_IGEMM_EVEN)):
        o = torch.full(want.shape, float("nan"), dtype=torch.float32, device=DEV)
        try:
            kst.kst_forward_seg_epilogue(xd, w_seg, Cout, n, None if bvec is None else bvec.to(DEV), act, P, out=o, path=code)
        except kst.KstError:
            assert name in ("igemm", "even"), name
            continue
        torch.cuda.synchronize()
        ran.append(name)
        err = np.abs(o.cpu().numpy() - want).max()                       # (NaN where nothing was written)
        assert err <= 2e-5 * scale, "%s: abs err %.3e (scale %.3g)" % (name, err, scale)
    assert "auto" in ran and "direct" in ran and "igemm" in ran


def _seeded_frame_and_epilogue_shapes(count, seed):
    """fp32 layers aimed at the kernels that supply the zero frame themselves and shift their
    stores for odd padding factors -- the flat-output kernel (one or three input channels, maps
    that are multiples of 4), the multi-channel direct kernel, the pipelined matrix-core kernel
    (channel counts that are multiples of 4), the position-block kernel (64 and more input
    channels, few positions) -- each with a random bias and activation."""
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        kind = int(rng.integers(0, 4))
        n = int(rng.integers(2, 6))
        P = int(rng.integers(0, 6))
        act = int(rng.integers(0, 3))
        bias = bool(rng.integers(0, 2))
        if kind == 0:        # flat-output kernel
            Cin, Cout = int(rng.choice([1, 3])), int(rng.choice([1, 2, 3]))
            N = int(rng.choice([48, 52, 64, 100, 132]))
            B = int(rng.integers(1, 4)) if Cin == 1 else int(rng.choice([260, 300]))
            if Cin == 3 and N > 64:
                continue
        elif kind == 1:      # multi-channel direct kernel
            Cin, Cout = int(rng.choice([2, 5, 20, 33, 64, 100])), int(rng.choice([1, 2, 3, 4, 6]))
            N, B = int(rng.choice([5, 9, 16, 30, 37])), int(rng.integers(1, 4))
        elif kind == 2:      # pipelined matrix-core kernel
            Cin, Cout = int(rng.choice([8, 16, 32, 48])), int(rng.choice([16, 32, 64, 132]))
            N, B = int(rng.choice([4, 8, 12, 16, 20])), int(rng.choice([4, 8, 16]))
        else:                # position blocks of 16
            Cin, Cout = int(rng.choice([64, 96, 128, 256])), int(rng.choice([3, 16, 48, 64, 100]))
            N, B = int(rng.choice([2, 3, 4, 6, 8, 12])), int(rng.integers(1, 4))
        if 2 * N + 2 * P - n < 1 or B * Cin * Cout * (2 * N + 2 * P) ** 2 * n * n > 2.5e9:
            continue
        shapes.append((B, Cin, Cout, N, n, P, act, bias))
    return shapes


@pytest.mark.parametrize("B,Cin,Cout,N,n,P,act,bias", _seeded_frame_and_epilogue_shapes(48, 20261128))
def test_seeded_padded_layers_with_bias_and_activation(B, Cin, Cout, N, n, P, act, bias):
    layer = wl.Layer("frame_seeded", B, Cin, Cout, N, n, "f32", "normal", w_std=0.2)
    x, w = wl.make_tensors(layer, 9500 + 31 * N + 7 * n + P + Cin)
    gen = torch.Generator().manual_seed(N + n + P + Cout)
    bvec = torch.randn((Cout,), generator=gen, dtype=torch.float32) if bias else None
    xd, w_seg = x.to(DEV), kst.kst_segregate_weights(w.to(DEV))
    want = oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), None if bvec is None else bvec.numpy().astype(np.float64),
                                   act, P)
    scale = max(1.0, np.abs(oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w),
                                                    None if bvec is None else bvec.numpy().astype(np.float64), 0, P)).max())
    ran = []
    for name, code in (("auto", kst.KST_PATH_AUTO), ("direct", kst.KST_PATH_DIRECT), ("igemm", kst.KST_PATH_IGEMM)):
        try:
            got = kst.kst_forward_seg_epilogue(xd, w_seg, Cout, n, None if bvec is None else bvec.to(DEV), act, P, path=code)
        except kst.KstError:
            assert name == "igemm", name
            continue
        torch.cuda.synchronize()
        ran.append(name)
        assert got.shape == want.shape
        err = np.abs(got.cpu().numpy() - want).max()
        assert err <= 2e-5 * scale, "%s: abs err %.3e (scale %.3g)" % (name, err, scale)
    assert "auto" in ran and "direct" in ran


# ----------------------------------------------------------------------------
# Image layers with kernels of 4 x 4 and more at large batches (the flat-output kernel with three
# input channels, the multi-channel kernel with two or four)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("B,Cin,Cout,N,n,P,act,bias", [
    (90, 3, 1, 224, 5, 2, 1, True),      # Table 1's layer, 5 x 5 kernel, ReLU
    (86, 3, 1, 224, 4, 1, 0, False),     # ... 4 x 4 kernel, odd padding factor (the sub-kernels' roles swapped)
    (1024, 2, 2, 64, 4, 3, 2, True),     # small maps, two output channels, odd padding factor, tanh
    (300, 4, 1, 120, 5, 0, 0, False),    # no padding: odd map (M = 235), four input channels
    (70, 2, 3, 250, 7, 4, 0, True),      # 7 x 7 kernel, a map edge that is no multiple of 4, three output channels
    (260, 2, 2, 128, 6, 5, 1, False),    # 6 x 6 kernel, padding factor 5
])
def test_forward_of_image_layers_at_large_batches(B, Cin, Cout, N, n, P, act, bias):
    layer = wl.Layer("image_batches", B, Cin, Cout, N, n, "f32", "normal", w_std=0.2)
    x, w = wl.make_tensors(layer, 8100 + 3 * N + 7 * n + P)
    gen = torch.Generator().manual_seed(N + n + P + Cout)
    bvec = torch.randn((Cout,), generator=gen, dtype=torch.float32) if bias else None
    b64 = None if bvec is None else bvec.numpy().astype(np.float64)
    xd, w_seg = x.to(DEV), kst.kst_segregate_weights(w.to(DEV))
    want = oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), b64, act, P)
    scale = max(1.0, np.abs(oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), b64, 0, P)).max())
    assert kst.kst_workspace_bytes_padded(B, Cin, Cout, N, n, P, kst.KST_F32, kst.KST_PATH_AUTO) == 0
    for name, code in (("auto", kst.KST_PATH_AUTO), ("direct", kst.KST_PATH_DIRECT)):
        o = torch.full(want.shape, float("nan"), dtype=torch.float32, device=DEV)
        kst.kst_forward_seg_epilogue(xd, w_seg, Cout, n, None if bvec is None else bvec.to(DEV), act, P, out=o, path=code)
        torch.cuda.synchronize()
        err = np.abs(o.cpu().numpy() - want).max()                       # (NaN where nothing was written)
        assert err <= 2e-5 * scale, "%s: abs err %.3e (scale %.3g)" % (name, err, scale)


# ----------------------------------------------------------------------------
# Few output channels, many input channels, batched: the taps of all sub-kernels as the rows of
# one matrix product over the input channels (the generators' output layer of Table 3)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("B,Cin,Cout,N,n,P,act,bias", [
    (33, 64, 3, 32, 4, 2, 2, True),     # Table 3's output layer at half the channels: 48 rows, 16 output rows per workgroup, tanh
    (32, 96, 4, 32, 4, 0, 0, False),    # no padding, 64 rows (all four row blocks), three chunks of channels, M = 60: ragged last block
    (33, 64, 2, 32, 3, 1, 1, True),     # 3 x 3 kernel, odd padding factor, 18 rows, ReLU
    (33, 64, 1, 32, 5, 3, 0, True),     # 5 x 5 kernel, one output channel, odd map (M = 65): five row blocks, the last of one row
    (16, 64, 3, 64, 2, 2, 0, False),    # 2 x 2 kernel on the widest map the kernel takes: 8 output rows per workgroup
    (128, 64, 3, 8, 4, 2, 2, False),    # small maps: one workgroup per batch item
    (64, 64, 3, 16, 3, 9, 1, True),     # padding factor beyond the kernel: output rows that only the padding reaches (bias alone)
    (35, 128, 3, 28, 4, 2, 0, False),   # a map edge that is no multiple of 16: column blocks straddle rows; four chunks
    (32, 256, 4, 32, 4, 2, 1, True),    # the largest the kernel takes: 64 rows, 256 input channels (150 KB of LDS)
])
def test_tap_major_matrix_core_kernel(B, Cin, Cout, N, n, P, act, bias):
    layer = wl.Layer("tap_major", B, Cin, Cout, N, n, "f32", "relu_normal", w_std=0.1)
    x, w = wl.make_tensors(layer, 7300 + 13 * N + 5 * n + P + Cin)
    gen = torch.Generator().manual_seed(N + n + P + Cout)
    bvec = torch.randn((Cout,), generator=gen, dtype=torch.float32) if bias else None
    b64 = None if bvec is None else bvec.numpy().astype(np.float64)
    xd, w_seg = x.to(DEV), kst.kst_segregate_weights(w.to(DEV))
    want = oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), b64, act, P)
    scale = max(1.0, np.abs(oracle.forward_epilogue(wl.to_f64(x), wl.to_f64(w), b64, 0, P)).max())
    # the matrix-core path of such a layer needs no workspace (the tile kernels would: this is how the test knows
    # which kernel AUTO and the forced path run)
    assert kst.kst_workspace_bytes_padded(B, Cin, Cout, N, n, P, kst.KST_F32, kst.KST_PATH_IGEMM) == 0
    assert kst.kst_workspace_bytes_padded(B, Cin, Cout, N, n, P, kst.KST_F32, kst.KST_PATH_AUTO) == 0
    got = {}
    for name, code in (("auto", kst.KST_PATH_AUTO), ("igemm", kst.KST_PATH_IGEMM), ("direct", kst.KST_PATH_DIRECT)):
        o = kst.kst_forward_seg_epilogue(xd, w_seg, Cout, n, None if bvec is None else bvec.to(DEV), act, P, path=code)
        torch.cuda.synchronize()
        assert o.shape == want.shape
        err = np.abs(o.cpu().numpy() - want).max()
        assert err <= 2e-5 * scale, "%s: abs err %.3e (scale %.3g)" % (name, err, scale)
        got[name] = o
    assert torch.equal(got["auto"], got["igemm"])          # AUTO takes the matrix-core kernel for these layers


# ----------------------------------------------------------------------------
# Half-precision operands: the 16-bit kernels with the other multiply
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("B,Cin,Cout,N,n,paths", [
    (2, 48, 32, 22, 3, ("igemm", "forward", "direct")),      # row-strip kernel
    (1, 17, 33, 50, 1, ("igemm", "forward", "direct")),      # ... n = 1, ragged channels
    (2, 48, 64, 32, 2, ("igemm", "forward", "direct")),      # LDS-ring kernel
    (1, 64, 64, 64, 3, ("igemm", "forward", "direct")),      # ... the ring wraps
    (4, 32, 256, 64, 3, ("igemm", "forward")),               # persistent wide-tile kernel
    (29, 112, 128, 32, 2, ("igemm", "forward")),             # ... seven chunks
    (2, 24, 40, 9, 5, ("igemm", "forward", "direct")),       # the plain 16-bit matrix-core kernel
    (1, 3, 2, 20, 4, ("direct", "forward", "zero_insert")),  # few channels
    (2, 1, 1, 33, 5, ("direct", "forward", "zero_insert")),  # one channel
])
def test_half_precision_forward(B, Cin, Cout, N, n, paths):
    layer = wl.Layer("f16", B, Cin, Cout, N, n, "f16", "relu_normal", w_std=0.1)
    check_layer(layer, paths=paths, seed=N * 11 + n)


def test_half_precision_wide_kernel_is_exact_on_integers():
    """Small integers are exact in half precision and in the fp32 accumulators."""
    layer = wl.Layer("wide_int_f16", 5, 32, 256, 64, 3, "f16", "integer")
    x, w = wl.make_tensors(layer, 14)
    out = kst.kst_forward_seg(x.to(DEV), kst.kst_segregate_weights(w.to(DEV)), layer.Cout, layer.n, path=kst.KST_PATH_IGEMM)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().astype(np.float64), oracle.forward(wl.to_f64(x), wl.to_f64(w)))


@pytest.mark.parametrize("B,Cin,Cout,N,n,P,dtype", [s[:6] + ("f16",) for s in _seeded_forward_shapes(16, 20260514)])
def test_half_precision_forward_seeded_shapes(B, Cin, Cout, N, n, P, dtype):
    test_forward_seeded_shapes_on_every_path_that_takes_them(B, Cin, Cout, N, n, P, dtype)


@pytest.mark.parametrize("B,Cin,Cout,N,n,P,dtype", [s[:6] + ("f16",) for s in _seeded_few_channel_shapes(12, 20260515)] +
                         [(2, 64, 32, 8, 4, 2, "f16"), (1, 128, 3, 8, 4, 2, "f16")])
def test_half_precision_gradients(B, Cin, Cout, N, n, P, dtype):
    test_gradients_of_few_channel_layers_seeded_shapes(B, Cin, Cout, N, n, P, dtype)
