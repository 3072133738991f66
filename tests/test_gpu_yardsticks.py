"""The measurement yardsticks: the streaming copy copies, the matrix-core loop runs and refuses
arguments it cannot serve.  They are no part of the method, so there is no oracle for them."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kst():
    from paper_2209_03704_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("elems", [4, 4 * 1000 + 4, 4 * (1 << 20) + 12])
def test_copy_is_bit_exact(kst, elems):
    g = torch.Generator(device="cpu").manual_seed(elems)
    src = torch.randint(-2**31, 2**31 - 1, (elems,), generator=g, dtype=torch.int32).cuda()
    dst = torch.zeros(elems + 8, dtype=torch.int32, device="cuda")
    kst.kst_yardstick_copy(src, dst[:elems])
    torch.cuda.synchronize()
    assert torch.equal(dst[:elems], src)
    assert int(dst[elems:].abs().max()) == 0          # nothing behind the range is written


def test_copy_rejects_ragged_and_misaligned(kst):
    a = torch.zeros(64, dtype=torch.uint8, device="cuda")
    b = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(kst.KstError):
        kst.kst_yardstick_copy(a[:24], b[:24])        # not a multiple of 16 bytes
    with pytest.raises(kst.KstError):
        kst.kst_yardstick_copy(a[4:36], b[:32])       # source not aligned to 16 bytes


@pytest.mark.parametrize("dtype_name", ["KST_F32", "KST_BF16"])
def test_mfma_loop_runs_and_counts(kst, dtype_name):
    dt = getattr(kst, dtype_name)
    need = kst.kst_yardstick_mfma_sink_elems()
    sink = torch.full((need + 4,), float("nan"), dtype=torch.float32, device="cuda")
    kst.kst_yardstick_mfma(dt, 3, sink)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink[:need]).all())    # every lane of the grid wrote its sum
    assert bool(torch.isnan(sink[need:]).all())
    per = 2 * 32 * 32 * (16 if dtype_name == "KST_BF16" else 2)
    assert kst.kst_yardstick_mfma_flops(dt, 3) == per * 4 * 3 * (need // 64)
    assert kst.kst_yardstick_mfma_flops(dt, 0) == 0.0
    with pytest.raises(kst.KstError):
        kst.kst_yardstick_mfma(dt, 3, sink[: need - 1])
    with pytest.raises(kst.KstError):
        kst.kst_yardstick_mfma(dt, 0, sink)
