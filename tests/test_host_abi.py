"""Host-side checks of libkst.so that need no GPU: the library loads, exports
every symbol the headers under include/ declare, and rejects bad arguments before any
launch."""
import ctypes
import os
import re

import pytest

from paper_2209_03704_amd import binding as kst

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    """Every function the headers under include/ declare (kst.h: the product's interface;
    kst_yardstick.h: the benchmark's measuring aids)."""
    import glob
    names = set()
    for path in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        text = open(path).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(kst_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_are_exported_and_bound():
    names = declared_symbols()
    assert "kst_forward" in names and "kst_segregate_weights" in names
    l = kst.lib()
    for name in names:
        assert hasattr(l, name), name
        assert name in kst.SIGNATURES, "binding lacks " + name
        assert hasattr(kst, name), "binding lacks a wrapper for " + name
    assert sorted(kst.SIGNATURES) == names


def test_version_and_strings():
    assert kst.kst_version() >= 100
    assert kst.kst_status_string(0) == "ok"
    assert all(kst.kst_status_string(s) for s in range(0, 9))


@pytest.mark.parametrize("N,n", [(4, 3), (32, 3), (512, 5), (16, 4), (8, 5), (64, 3)])
def test_out_size(N, n):
    assert kst.kst_out_size(N, n) == 2 * N - n          # Section 1
    assert kst.kst_out_size_padded(N, n, 0) == 2 * N - n


def test_out_size_padded():
    # Table 1 shapes (224 x 224 inputs, padding factor 2) and DCGAN's 4 -> 8 layer of Table 3
    assert kst.kst_out_size_padded(224, 5, 2) == 447
    assert kst.kst_out_size_padded(224, 4, 2) == 448
    assert kst.kst_out_size_padded(224, 3, 2) == 449
    assert kst.kst_out_size_padded(4, 4, 2) == 8


@pytest.mark.parametrize("n", range(1, 10))
def test_subkernel_shapes_partition_the_kernel(n):
    """Section 3.2: sizes ceil x ceil, ceil x floor, floor x ceil, floor x floor."""
    ce, fl = (n + 1) // 2, n // 2
    shapes = [kst.kst_subkernel_shape(n, p) for p in range(4)]
    assert shapes == [(ce, ce), (ce, fl), (fl, ce), (fl, fl)]
    assert sum(a * b for a, b in shapes) == n * n
    # fp32 segregation is a permutation: same element count, class offsets are prefix sums
    Cin, Cout = 5, 7
    assert kst.kst_segregated_elems(Cin, Cout, n, kst.KST_F32) == Cin * Cout * n * n
    run = 0
    for p, (a, b) in enumerate(shapes):
        assert kst.kst_segregated_offset(Cin, Cout, n, p, kst.KST_F32) == run * Cin * Cout
        assert kst.kst_segregated_offset(Cin, Cout, n, p, kst.KST_BF16) == run * 8 * Cout
        run += a * b
    assert kst.kst_segregated_elems(Cin, Cout, n, kst.KST_BF16) == 8 * Cout * n * n


def test_subkernel_shape_errors():
    with pytest.raises(kst.KstError):
        kst.kst_subkernel_shape(0, 0)
    with pytest.raises(kst.KstError):
        kst.kst_subkernel_shape(3, 4)


def test_argument_errors_are_statuses_not_crashes():
    l = kst.lib()
    one = ctypes.c_void_p(16)          # non-null, aligned, never dereferenced: checks fail first
    # null pointers
    assert l.kst_forward(None, one, one, 1, 1, 1, 4, 3, 0, None) == 1
    assert l.kst_forward_seg(one, None, one, None, 0, 1, 1, 1, 4, 3, 0, 0, None) == 1
    assert l.kst_segregate_weights(None, one, 1, 1, 3, 0, None) == 1
    assert l.kst_forward_zero_insert(one, one, None, one, 1, 1, 1, 4, 3, 0, None) == 1
    # dtype
    assert l.kst_forward(one, one, one, 1, 1, 1, 4, 3, 7, None) == 3
    assert l.kst_segregate_weights(one, one, 1, 1, 3, 3, None) == 3
    # shapes: a size < 1, kernel larger than the up-sampled map, tensors of 2^31 elements
    assert l.kst_forward(one, one, one, 0, 1, 1, 4, 3, 0, None) == 2
    assert l.kst_forward(one, one, one, 1, 1, 1, 2, 5, 0, None) == 2
    assert l.kst_forward(one, one, one, 1, 1, 1, 4, 0, 0, None) == 2
    assert l.kst_forward(one, one, one, 4096, 64, 64, 512, 3, 0, None) == 2
    assert l.kst_forward_seg(one, one, one, None, 0, 1, 1, 1, 4, 9, 0, 0, None) == 2
    # unknown path; matrix-core path asked for a kernel size it does not cover
    assert l.kst_forward_seg(one, one, one, None, 0, 1, 8, 16, 8, 3, 0, 9, None) == 6
    assert l.kst_forward_seg(one, one, one, None, 0, 1, 8, 16, 8, 9, 0, 2, None) == 6
    # the forced even-share launch exists for fp32 layers with Cin and Cout multiples of 4 only
    assert l.kst_forward_seg(one, one, one, None, 0, 1, 8, 16, 8, 3, 1, 3, None) == 6      # bf16
    assert l.kst_forward_seg(one, one, one, None, 0, 1, 10, 16, 8, 3, 0, 3, None) == 6     # Cin = 10
    assert l.kst_forward_seg(one, one, one, None, 0, 1, 8, 18, 8, 3, 0, 3, None) == 6      # Cout = 18
    assert l.kst_forward_seg(one, one, one, None, 0, 1, 8, 16, 8, 3, 0, 3, None) == 4      # fine, but no workspace
    # (two workgroups, two slots each, of one tile's accumulators: 128 positions x 64 channels -- the half-width tile of
    # layers with up to 64 output channels -- x 4 classes)
    assert kst.kst_workspace_bytes(1, 8, 16, 8, 3, kst.KST_F32, kst.KST_PATH_IGEMM_EVEN) == 2 * 2 * 128 * 64 * 4 * 4
    # alignment
    odd = ctypes.c_void_p(20)
    assert l.kst_forward(odd, one, one, 1, 1, 1, 4, 3, 0, None) == 7
    # workspace: the split matrix-core plan needs scratch
    need = kst.kst_workspace_bytes(64, 1024, 512, 8, 5, kst.KST_F32, kst.KST_PATH_IGEMM)
    assert need > 0
    assert l.kst_forward_seg(one, one, one, None, 0, 64, 1024, 512, 8, 5, 0, 2, None) == 4
    assert l.kst_forward_seg(one, one, one, one, need - 1, 64, 1024, 512, 8, 5, 0, 2, None) == 4
    # sizes helpers return 0 on illegal input
    assert kst.kst_segregated_elems(0, 1, 3, 0) == 0
    assert kst.kst_workspace_bytes(1, 1, 1, 2, 5, 0, 0) == 0
    assert kst.kst_workspace_bytes(1, 1, 1, 32, 3, kst.KST_F32, kst.KST_PATH_DIRECT) == 0
    # padding factor: negative P, an output edge below 1, a missing or short workspace
    assert l.kst_forward_seg_padded(one, one, one, one, 1 << 20, 1, 1, 1, 4, 3, -1, 0, 0, None) == 2
    assert l.kst_forward_seg_padded(one, one, one, one, 1 << 20, 1, 1, 1, 1, 9, 2, 0, 0, None) == 2
    assert l.kst_forward_padded(one, one, one, 1, 1, 1, 1, 9, 2, 0, None) == 2
    assert l.kst_forward_seg_padded(one, None, one, one, 1 << 20, 1, 1, 1, 4, 3, 2, 0, 0, None) == 1
    # (a single-channel layer is served through a framed copy of the input)
    need = kst.kst_workspace_bytes_padded(2, 1, 4, 8, 3, 2, kst.KST_F32)
    assert need >= 2 * 1 * 10 * 10 * 4
    assert l.kst_forward_seg_padded(one, one, one, None, 0, 2, 1, 4, 8, 3, 2, 0, 0, None) == 4
    assert l.kst_forward_seg_padded(one, one, one, one, need - 1, 2, 1, 4, 8, 3, 2, 0, 0, None) == 4
    assert kst.kst_workspace_bytes_padded(1, 1, 1, 1, 9, 2, 0) == 0
    # odd P also holds the wider output
    assert kst.kst_workspace_bytes_padded(2, 1, 4, 8, 3, 3, kst.KST_F32) >= 2 * 1 * 12 * 12 * 4 + 2 * 4 * 21 * 21 * 4
    assert l.kst_forward_seg_padded(one, one, one, None, 0, 2, 1, 4, 8, 3, 3, 0, 0, None) == 4
    # several input channels on the direct path: the kernel supplies the zero frame itself and, for an
    # odd P, stores its quads one row and column earlier: no workspace at all
    assert kst.kst_workspace_bytes_padded(2, 3, 4, 8, 3, 2, kst.KST_F32) == 0
    assert kst.kst_workspace_bytes_padded(2, 3, 4, 8, 3, 3, kst.KST_F32) == 0
    # large single-channel maps (the flat-output kernel keeps the frame in LDS): none either
    assert kst.kst_workspace_bytes_padded(2, 1, 1, 64, 5, 2, kst.KST_F32) == 0
    assert kst.kst_workspace_bytes_padded(2, 1, 1, 64, 5, 3, kst.KST_F32) == 0
    # fp32 matrix cores: frame supplied while staging, odd P stored shifted: only the split reduction's partial sums
    # (no more than the even padding factor above it, which has the same frame and larger planes)
    assert 0 < kst.kst_workspace_bytes_padded(64, 512, 256, 8, 4, 3, kst.KST_F32) <= kst.kst_workspace_bytes_padded(
        64, 512, 256, 8, 4, 4, kst.KST_F32)


def test_gradient_workspaces_follow_the_kernels_that_run():
    """Byte counts depend on the shape only; what they hold is stated in the header."""
    f32 = kst.KST_F32
    # no padding factor, one workgroup's worth of positions: nothing to copy, nothing to add up
    assert kst.kst_backward_input_workspace_bytes(1, 2, 2, 8, 3, 0, f32) == 0
    # kernels up to 7 x 7 visit the unframed positions: an even P needs no copy for the input
    # gradient, an odd P only the one-pixel frame around g
    assert kst.kst_backward_input_workspace_bytes(2, 3, 1, 8, 3, 2, f32) == 0
    M = kst.kst_out_size_padded(8, 3, 3)                 # 19; framed by one pixel: 21
    need = kst.kst_backward_input_workspace_bytes(2, 3, 1, 8, 3, 3, f32)
    assert 2 * 1 * (M + 2) * (M + 2) * 4 <= need < 2 * 1 * (M + 2) * (M + 2) * 4 + 256
    # beyond 7 x 7 the plain kernels work on a framed problem: the framed result is held too
    assert kst.kst_backward_input_workspace_bytes(1, 2, 2, 8, 9, 2, f32) >= 1 * 2 * 10 * 10 * 4
    # kernel gradient, few channels, many positions: partial results of the sliced position range only
    need = kst.kst_backward_weight_workspace_bytes(16, 3, 1, 224, 5, 2, f32)
    assert 0 < need <= 1024 * 3 * 25 * 4 + 256
    # matrix cores: the zero-framed copy of g plus partial sums
    Mg = kst.kst_out_size_padded(16, 4, 2)               # 32; framed by n - 1 = 3
    need = kst.kst_backward_weight_workspace_bytes(64, 256, 128, 16, 4, 2, f32)
    assert need >= 64 * 128 * (Mg + 6) * (Mg + 6) * 4
    # 16-bit operands on the matrix cores: the fp32 kernels after an exact widening of w (input
    # gradient) or in (kernel gradient) into the workspace
    for dt in (kst.KST_BF16, kst.KST_F16):
        assert (kst.kst_backward_input_workspace_bytes(64, 256, 128, 16, 4, 2, dt)
                == kst.kst_backward_input_workspace_bytes(64, 256, 128, 16, 4, 2, f32) + 128 * 256 * 16 * 4)
        assert (kst.kst_backward_weight_workspace_bytes(64, 256, 128, 16, 4, 2, dt)
                == kst.kst_backward_weight_workspace_bytes(64, 256, 128, 16, 4, 2, f32) + 64 * 256 * 16 * 16 * 4)
    # illegal shapes give 0
    assert kst.kst_backward_weight_workspace_bytes(1, 1, 1, 1, 9, 0, f32) == 0
    assert kst.kst_backward_input_workspace_bytes(0, 1, 1, 8, 3, 0, f32) == 0
