"""GPU parity of the comparison implementations (the paper's scheme 1 with materialised
intermediates and a vendor batched multiply, its scheme 2 as a flat loop with atomic
accumulation, and the framework's grouped convolution) against the CPU oracle.  They are
measured next to the implicit-GEMM kernels, so they must compute the same operator."""
import numpy as np
import pytest

from oracle import capsconv
from paper_2104_02621_amd import capscaps as cc
from paper_2104_02621_amd import comparisons as cmp
from paper_2104_02621_amd import workloads as wl
from tests.gpu_util import check, shape_args, to_device
from tests.test_gpu_parity import SMALL_SHAPES, small

pytestmark = pytest.mark.gpu


def run_scheme2(w, i_dev, k_dev):
    import torch
    args = shape_args(w)
    nbytes = cc.capscaps_scheme2_index_bytes(*args)
    assert nbytes > 0
    index = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    assert cc.capscaps_scheme2_build_index(index.data_ptr(), nbytes, *args, st) == cc.OK
    out = torch.full(w.out_shape, float("nan"), dtype=torch.float32, device="cuda")
    rc = cc.capscaps_scheme2_fwd(i_dev.data_ptr(), k_dev.data_ptr(), out.data_ptr(),
                                 index.data_ptr(), nbytes, *args, st)
    assert rc == cc.OK, cc.capscaps_strerror(rc)
    return out


def compare_all(w):
    i_st, k_st, i32, k32 = wl.generate(w)
    ref, S = capsconv.conv_fwd(i32, k32, w.stride, w.pad, with_abs_sum=True)
    i_dev, k_dev = to_device(i_st, w.dtype), to_device(k_st, w.dtype)
    check(w, run_scheme2(w, i_dev, k_dev).cpu().numpy(), ref, S, "scheme 2")
    check(w, cmp.scheme1_fwd(i_dev, k_dev, w.stride, w.pad, max_batch_elems=1 << 16).cpu().numpy(),
          ref, S, "scheme 1")
    # the framework's convolution algorithms may leave rounding noise instead of an exact zero
    # where a window lies entirely in the padding (S = 0): hold those to the overall scale
    S_fw = np.where(S == 0, np.abs(ref).max(), S)
    check(w, cmp.framework_conv_fwd(i_dev, k_dev, w.stride, w.pad).cpu().numpy(), ref, S_fw,
          "framework conv")


@pytest.mark.parametrize("dtype", [wl.FP32, wl.BF16, wl.FP16], ids=["fp32", "bf16", "fp16"])
@pytest.mark.parametrize("shape", SMALL_SHAPES, ids=[s[0] for s in SMALL_SHAPES])
def test_small_shapes_match_oracle(shape, dtype):
    compare_all(small(shape[0], dtype, *shape[1:], seed=len(shape[0]) + 90))


@pytest.mark.parametrize("number", [1, 4])
def test_benchmark_configs(number):
    compare_all(wl.config(number))


def test_benchmark_config_2_two_images():
    """Configuration 2's layer on two of its 64 images: scheme 1 needs 2.8e7 small products per
    image there and runs them as 14 batched multiplies per image (blocks of 75 output pixels)."""
    w = wl.config(2).with_batch(2)
    assert w.Ho * w.Wo * w.M * w.kh * w.kw * w.C * w.D0 > 6 * cmp.MAX_BMM_BATCH
    i_st, k_st, i32, k32 = wl.generate(w)
    ref, S = capsconv.conv_fwd(i32, k32, w.stride, w.pad, with_abs_sum=True)
    i_dev, k_dev = to_device(i_st, w.dtype), to_device(k_st, w.dtype)
    check(w, cmp.scheme1_fwd(i_dev, k_dev, w.stride, w.pad).cpu().numpy(), ref, S, "scheme 1")


def test_scheme2_integer_data_is_exact():
    """Every partial sum is exact in fp32, so the unordered atomic additions cannot show."""
    w = wl.integer_variant(small("sq4", wl.FP32, 3, 9, 10, 5, 6, 3, 3, 1, 1, 1, 4, 4, 4))
    i_st, k_st, i32, k32 = wl.generate(w)
    ref = capsconv.conv_fwd(i32, k32, w.stride, w.pad)
    got = run_scheme2(w, to_device(i_st, w.dtype), to_device(k_st, w.dtype)).cpu().numpy()
    assert np.array_equal(got.astype(np.float64), ref)


def test_scheme2_refuses_small_index_buffer():
    import torch
    w = small("sq4", wl.FP32, 3, 9, 10, 5, 6, 3, 3, 1, 1, 1, 4, 4, 4)
    args = shape_args(w)
    nbytes = cc.capscaps_scheme2_index_bytes(*args)
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p, st = buf.data_ptr(), torch.cuda.current_stream().cuda_stream
    assert cc.capscaps_scheme2_build_index(p, nbytes - 1, *args, st) == cc.EWORKSPACE
    assert cc.capscaps_scheme2_fwd(p, p, p, p, nbytes - 1, *args, st) == cc.EWORKSPACE
    assert cc.capscaps_scheme2_fwd(p, p, p, 0, nbytes, *args, st) == cc.EINVAL


@pytest.mark.parametrize("dtype", [wl.FP32, wl.BF16, wl.FP16], ids=["fp32", "bf16", "fp16"])
def test_mfma_yardstick_computes_what_it_counts(dtype):
    """The measurement aid's arithmetic is checked too: with all-ones operands every accumulator
    element of a wave ends at iters * (K per instruction group), so a lane's sum over its 16
    tiles x 16 registers is known exactly."""
    import torch
    n_elem = 8 * 64 * (4 if dtype == wl.FP32 else 8)
    st, _ = wl.to_storage(np.ones(n_elem, dtype=np.float32), dtype)
    seed = to_device(st, dtype)
    blocks, iters = 3, 5
    sink = torch.full((blocks * 256,), float("nan"), dtype=torch.float32, device="cuda")
    rc = cc.capscaps_mfma_yardstick(seed.data_ptr(), sink.data_ptr(), dtype, blocks, iters,
                                    torch.cuda.current_stream().cuda_stream)
    assert rc == cc.OK
    k_per_iter = 8 if dtype == wl.FP32 else 16      # contracted values per accumulator and iteration
    assert bool((sink == 256.0 * iters * k_per_iter).all())
