"""GPU parity of the forward pass with 16-bit output (capscaps_conv_fwd_out16): the fp32
accumulator rounded to nearest even once, at the store.  Two checks: against the same library's
fp32 output rounded on the host (bit for bit where both calls sum in the same order: same kernel,
one rounding), and against the CPU oracle within half a 16-bit unit plus the fp32 summation
error."""
import numpy as np
import pytest

from oracle import capsconv
from paper_2104_02621_amd import capscaps as cc
from paper_2104_02621_amd import workloads as wl
from tests.gpu_util import run_gpu, shape_args, to_device
from tests.test_gpu_parity import SMALL_SHAPES, TUNED_SHAPES, small

pytestmark = pytest.mark.gpu

# relative size of one unit in the last place of the 16-bit types (8 and 11 significand bits)
ULP16 = {wl.BF16: 2.0 ** -7, wl.FP16: 2.0 ** -10}


def run_out16(w, i_dev, k_dev):
    import torch
    tdt = torch.bfloat16 if w.dtype == wl.BF16 else torch.float16
    out = torch.full(w.out_shape, float("nan"), dtype=tdt, device="cuda")
    need = cc.capscaps_conv_fwd_out16_workspace_bytes(*shape_args(w))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    rc = cc.capscaps_conv_fwd_out16(i_dev.data_ptr(), k_dev.data_ptr(), out.data_ptr(),
                                    *shape_args(w), ws.data_ptr(), ws.numel(),
                                    torch.cuda.current_stream().cuda_stream)
    assert rc == cc.OK, f"{w.name}: status {rc} ({cc.capscaps_strerror(rc)})"
    return out


def to_bits(t):
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def round_on_host(x32, dtype):
    if dtype == wl.BF16:
        return wl.round_to_bf16_bits(x32)
    return x32.astype(np.float16).view(np.uint16)


def bits_to_f64(bits, dtype):
    if dtype == wl.BF16:
        return wl.bf16_bits_to_f32(bits).astype(np.float64)
    return bits.view(np.float16).astype(np.float64)


def check_out16(w, ref=None, S=None, sample=None, exact_order=True):
    i_st, k_st, i32, k32 = wl.generate(w)
    i_dev, k_dev = to_device(i_st, w.dtype), to_device(k_st, w.dtype)
    got_bits = to_bits(run_out16(w, i_dev, k_dev))
    # (1) one rounding of the very same fp32 result.  On large problems the fp32 call may add
    # up the last tiles' K loop in pieces (another summation order, last bits differ): there a
    # few values near a rounding tie may land on the neighbouring 16-bit number.
    out32 = run_gpu(w, i_dev, k_dev, cc.PATH_AUTO).cpu().numpy()
    same = got_bits == round_on_host(out32, w.dtype)
    if not exact_order:
        off = ~same
        assert off.mean() < 1e-3, w.name
        g = bits_to_f64(got_bits[off], w.dtype)
        # half a 16-bit unit, plus what two fp32 summation orders can differ by
        noise = 1e-6 * np.abs(out32).max()
        assert (np.abs(g - out32[off]) <= 0.51 * ULP16[w.dtype] * np.abs(out32[off]) + noise).all()
    else:
        assert same.all(), w.name
    # (2) the oracle: half a unit of the 16-bit type, the fp32 summation error, and the
    # absolute spacing of the type's smallest numbers
    got = bits_to_f64(got_bits, w.dtype)
    if sample is not None:
        which = sample
        ref, S = capsconv.conv_fwd_subset(i32, k32, which, w.stride, w.pad, with_abs_sum=True)
        got = got[which[:, 0], which[:, 1], which[:, 2], which[:, 3]]
    elif ref is None:
        ref, S = capsconv.conv_fwd(i32, k32, w.stride, w.pad, with_abs_sum=True)
    bound = 0.5 * ULP16[w.dtype] * np.abs(ref) * 1.0001 + 1e-5 * S + 1e-7
    worst = (np.abs(got - ref) / bound).max()
    print(f"{w.name}: max error / bound = {worst:.3f}", flush=True)
    assert worst <= 1.0, w.name


# enough rows for the lane-per-row kernel to be the library's choice: 4x4 capsules (channels
# paired by a pre-pass), non-square capsules, and square ones on 384 columns
LANE_PER_ROW_SHAPES = [
    #        N  H   W   C   M  kh kw s  p D0  D1  D2  D3
    ("o4x4", 12, 40, 40, 8, 8, 3, 3, 1, 1, 1, 4, 4, 4),
    ("o4x8", 12, 40, 40, 6, 5, 3, 3, 1, 1, 1, 4, 8, 16),
    ("o384", 6, 40, 40, 8, 48, 3, 3, 1, 1, 1, 8, 8, 8),
    # ... 64 and 128 columns (two and four 32-column tiles per wave)
    ("o4x4c64", 12, 40, 40, 8, 16, 3, 3, 1, 1, 1, 4, 4, 4),
    ("o4x4c128", 12, 40, 40, 8, 32, 3, 3, 1, 1, 1, 4, 4, 4),
]
SHAPES = SMALL_SHAPES + TUNED_SHAPES + LANE_PER_ROW_SHAPES


@pytest.mark.parametrize("dtype", [wl.BF16, wl.FP16], ids=["bf16", "fp16"])
@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_small_shapes(shape, dtype):
    w = small(shape[0], dtype, *shape[1:], seed=len(shape[0]) + 120)
    if shape in LANE_PER_ROW_SHAPES:
        assert cc.capscaps_select_path(*shape_args(w)) == cc.PATH_MFMA_TUNED32
    check_out16(w)


@pytest.mark.parametrize("number", [3, 5])
def test_benchmark_configs_full_size_sampled(number):
    """Full size, the tuned kernel's 16-bit-output variant; the oracle on sampled capsules."""
    w = wl.config(number)
    assert cc.capscaps_select_path(*shape_args(w)) == cc.PATH_MFMA_TUNED16
    check_out16(w, sample=wl.sample_capsules(w, 1500, seed=77 + number), exact_order=False)


def test_fp32_operands_are_refused():
    import torch
    w = small("f32", wl.FP32, 1, 6, 6, 4, 4, 3, 3, 1, 1, 1, 4, 4, 4)
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    assert cc.capscaps_conv_fwd_out16_workspace_bytes(*shape_args(w)) == 0
    assert cc.capscaps_conv_fwd_out16(p, p, p, *shape_args(w), p, buf.numel(), None) == cc.EINVAL
