"""GPU parity of the backward pass: the HIP library's input and kernel gradients, called
through the C ABI, against the CPU oracle's, element by element on the same seeded inputs.
Needs an MI355X."""
import dataclasses
import functools

import numpy as np
import pytest

from oracle import capsconv
from paper_2104_02621_amd import capscaps as cc
from paper_2104_02621_amd import workloads as wl
from tests.gpu_util import check, shape_args, to_device
from tests.test_gpu_parity import SMALL_SHAPES, small

pytestmark = pytest.mark.gpu


def run_bwd_input(w, g_dev, k_dev):
    import torch
    din = torch.full(w.input_shape, float("nan"), dtype=torch.float32, device="cuda")
    need = cc.capscaps_conv_bwd_input_workspace_bytes(*shape_args(w))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    rc = cc.capscaps_conv_bwd_input(g_dev.data_ptr(), k_dev.data_ptr(), din.data_ptr(),
                                    *shape_args(w), ws.data_ptr(), ws.numel(),
                                    torch.cuda.current_stream().cuda_stream)
    assert rc == cc.OK, f"{w.name}: status {rc} ({cc.capscaps_strerror(rc)}; {cc.capscaps_last_hip_error()})"
    return din


def run_bwd_kernel(w, i_dev, g_dev):
    import torch
    dk = torch.full(w.kernel_shape, float("nan"), dtype=torch.float32, device="cuda")
    need = cc.capscaps_conv_bwd_kernel_workspace_bytes(*shape_args(w))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    rc = cc.capscaps_conv_bwd_kernel(i_dev.data_ptr(), g_dev.data_ptr(), dk.data_ptr(),
                                     *shape_args(w), ws.data_ptr(), ws.numel(),
                                     torch.cuda.current_stream().cuda_stream)
    assert rc == cc.OK, f"{w.name}: status {rc} ({cc.capscaps_strerror(rc)}; {cc.capscaps_last_hip_error()})"
    return dk


@functools.lru_cache(maxsize=2)
def oracle_bwd(w):
    """Inputs, the oracle's two gradients and, as the error scale of each gradient element,
    the same sums taken over absolute values."""
    i_st, k_st, i32, k32 = wl.generate(w)
    g_st, g32 = wl.generate_dout(w)
    hw, khw = (w.H, w.W), (w.kh, w.kw)
    dI = capsconv.conv_bwd_input(g32, k32, hw, w.stride, w.pad)
    dK = capsconv.conv_bwd_kernel(i32, g32, khw, w.stride, w.pad)
    SI = capsconv.conv_bwd_input(np.abs(g32), np.abs(k32), hw, w.stride, w.pad)
    SK = capsconv.conv_bwd_kernel(np.abs(i32), np.abs(g32), khw, w.stride, w.pad)
    return i_st, k_st, g_st, dI, dK, SI, SK


def both_gradients(w):
    i_st, k_st, g_st, dI, dK, SI, SK = oracle_bwd(w)
    i_dev, k_dev, g_dev = (to_device(a, w.dtype) for a in (i_st, k_st, g_st))
    got_i = run_bwd_input(w, g_dev, k_dev).cpu().numpy()
    got_k = run_bwd_kernel(w, i_dev, g_dev).cpu().numpy()
    # an input pixel no window reaches has dI = 0 and scale 0: compare those exactly
    dead = SI == 0
    assert (got_i[dead] == 0).all()
    check(w, got_i, dI, np.where(dead, 1.0, SI), "dinput")
    dead = SK == 0
    assert (got_k[dead] == 0).all()
    check(w, got_k, dK, np.where(dead, 1.0, SK), "dkernel")
    return got_i, got_k, dI, dK


# the forward pass's small shapes (strides 1..4, non-square windows and capsules, degenerate
# geometries) plus stride-1 cases that exercise the convolution route on several tiles
BWD_SHAPES = SMALL_SHAPES + [
    #          N  H   W   C   M  kh kw s  p D0  D1  D2  D3
    ("deeppad", 2, 5, 5, 3, 4, 3, 3, 1, 4, 1, 4, 4, 4),     # pad > k-1: no flipped-kernel form
    ("s1wide", 3, 12, 12, 24, 20, 3, 3, 1, 1, 1, 8, 8, 8),
    ("s1d16", 2, 9, 8, 16, 12, 3, 3, 1, 1, 1, 16, 16, 16),
    ("s1nonsq", 2, 10, 7, 6, 9, 2, 2, 1, 0, 2, 3, 5, 4),
    ("s1k5", 1, 11, 11, 8, 8, 5, 5, 1, 2, 1, 4, 4, 4),
    # for the 16-bit kernel-gradient kernel (D1 in {8, 16}): ragged rows and columns with a
    # leading capsule index, window taps that never meet the image, several row and column
    # tiles at stride 3, many images (the contraction split over image ranges)
    ("wg_rag", 3, 7, 6, 5, 3, 3, 3, 2, 1, 2, 8, 5, 4),
    ("wg_empty", 2, 1, 1, 3, 2, 5, 5, 1, 2, 1, 8, 4, 4),
    ("wg_d16s3", 2, 10, 9, 20, 18, 3, 3, 3, 1, 1, 16, 16, 16),
    ("wg_many", 70, 5, 5, 4, 4, 2, 2, 1, 0, 1, 16, 8, 8),
    # capsule widths that are multiples of 8 are read in place (no transposed copies): ragged
    # row and column tiles with a leading capsule index, and widths of 24 and 8 under 16 rows
    ("wg_own_rag", 3, 7, 6, 37, 35, 3, 3, 2, 1, 2, 8, 8, 16),
    ("wg_own_d24", 2, 5, 6, 3, 5, 2, 3, 1, 1, 1, 16, 24, 8),
    # for the fp32 kernel-gradient kernel: capsule heights of 6 and 12 floats (two and four
    # chunks of 3), several row and column tiles with ragged ends
    ("wg32_d6", 2, 6, 6, 3, 5, 3, 3, 1, 1, 2, 6, 4, 3),
    ("wg32_d12", 2, 5, 5, 2, 3, 2, 2, 2, 0, 1, 12, 5, 4),
    ("wg32_rows", 2, 6, 6, 40, 30, 3, 3, 1, 1, 1, 4, 8, 8),
    # ... and square capsules, which that kernel reads without transposed copies: 3x3x3 with a
    # leading capsule index (config 2's kind), several row and column tiles of 4x4 capsules,
    # heights of two and four chunks of 3, and 3x3 capsules on more columns than one tile
    # (which go the transposed way again)
    ("wg32n_d3", 3, 7, 6, 10, 9, 3, 3, 1, 1, 3, 3, 3, 3),
    ("wg32n_d4t", 2, 6, 6, 70, 40, 3, 3, 1, 1, 1, 4, 4, 4),
    ("wg32n_d6", 2, 6, 6, 5, 7, 3, 3, 1, 1, 2, 6, 6, 6),
    ("wg32n_d12", 2, 5, 5, 3, 3, 2, 2, 2, 0, 1, 12, 12, 12),
    ("wg32n_d3t", 2, 6, 6, 20, 50, 3, 3, 2, 1, 1, 3, 3, 3),
    # large enough for the strided input gradient to run as interleaved phase convolutions
    # (16-bit): stride 2; stride 3 with a 2x2 window (one phase of pixels no window reaches);
    # a non-square window with padding beyond its reach and a leading capsule index
    ("ph_s2", 3, 80, 80, 4, 8, 3, 3, 2, 1, 1, 8, 8, 8),
    ("ph_s3", 3, 120, 118, 4, 8, 2, 2, 3, 0, 1, 8, 4, 8),
    ("ph_ns", 2, 90, 61, 3, 4, 4, 3, 2, 3, 2, 16, 8, 16),
    # ... and for fp32 on the tuned fp32 kernel (which wants 256 tiles of 256 rows per phase):
    # 8x8 capsules at stride 2, and 3x3x3 capsules (12-byte rows, a leading capsule index) at
    # stride 3 with a 4x4 window, whose phases have 2 or 1 taps a side and different paddings
    # 4x4 capsules on enough pixels for the 16-bit input gradient to run on the lane-per-row
    # kernel (the output gradient's channels paired)
    ("p4big", 12, 40, 40, 8, 8, 3, 3, 1, 1, 1, 4, 4, 4),
    # 4-row capsules with widths of 8 and 16: the 16-bit kernel gradient reads them in place
    ("wg4_inpl", 3, 9, 8, 5, 6, 3, 3, 1, 1, 1, 4, 8, 16),
    ("wg4_wide", 2, 7, 7, 3, 3, 2, 2, 2, 0, 2, 4, 16, 8),
    # vector capsules (one or two rows): every lane of the 16-bit kernel gradient follows a pixel
    # of its own; strides, a leading capsule index, many images (the contraction split over image
    # ranges), a 1x1 image under a 5x5 window (taps that never meet it), rectangles narrower than
    # a stage
    ("wgv1", 3, 9, 8, 5, 6, 3, 3, 1, 1, 1, 1, 8, 16),
    ("wgv2", 2, 7, 7, 3, 3, 2, 2, 2, 0, 2, 2, 16, 8),
    ("wgv1many", 40, 5, 5, 4, 4, 2, 2, 1, 0, 1, 1, 8, 8),
    ("wgv1tiny", 2, 1, 1, 3, 2, 5, 5, 1, 2, 1, 1, 8, 8),
    ("wgv2wide", 1, 3, 70, 2, 35, 3, 3, 3, 1, 1, 2, 8, 8),
    ("ph32_s2", 7, 80, 78, 4, 8, 3, 3, 2, 1, 1, 8, 8, 8),
    # ... and for 16-bit layers the 256x256-tile kernel does not take: 4x4 capsules, and 8-row
    # capsules on too few channels for its stages
    ("ph16_d4", 14, 80, 78, 4, 8, 3, 3, 2, 1, 1, 4, 4, 4),
    ("ph16_ns", 10, 60, 62, 6, 4, 3, 3, 2, 1, 1, 8, 16, 8),
    ("ph32_d3", 8, 100, 97, 5, 6, 4, 4, 3, 2, 3, 3, 3, 3),
    # at most 128 rows (c, d2): the 16-bit kernel gradient puts several window taps into a tile.  A 5x5
    # window with padding 2 (25 taps: the last pair has one; neighbouring taps' pixel ranges
    # differ by up to two), stride 3 with a leading capsule index and 16-row capsules, an image
    # narrower than the window (the next row's first tap lies before the previous row's last),
    # a 1x1 image (pairs of which one or no tap meets it), channel-paired 4x4 capsules, and
    # exactly 128 rows under a 1x2 window
    ("wgp_k5", 2, 6, 7, 3, 5, 5, 5, 1, 2, 1, 8, 8, 8),
    ("wgp_s3", 2, 10, 9, 4, 3, 3, 2, 3, 1, 2, 16, 16, 8),
    ("wgp_thin", 3, 2, 2, 2, 3, 5, 5, 1, 2, 1, 8, 8, 8),
    ("wgp_1x1", 2, 1, 1, 3, 2, 5, 5, 1, 2, 1, 4, 8, 8),
    ("wgp_44", 3, 9, 8, 6, 4, 3, 3, 2, 1, 1, 4, 4, 4),
    ("wgp_128", 2, 7, 7, 16, 3, 1, 2, 1, 0, 1, 8, 8, 8),
    # (the shapes above with at most 64 rows take four taps per tile.)  Two taps per tile with
    # 65 .. 128 rows: 96 rows at stride 2, 80 rows of 16-wide capsules under a 5x5 window, a 1x1
    # image, and a two-tap window on few rows
    ("wgp_r96", 2, 8, 7, 12, 5, 3, 3, 2, 1, 1, 8, 8, 8),
    ("wgp_r80k5", 2, 6, 7, 5, 3, 5, 5, 1, 2, 1, 8, 16, 8),
    ("wgp_1x1b", 2, 1, 1, 9, 2, 5, 5, 1, 2, 1, 4, 8, 8),
    ("wgq_1x2", 2, 7, 7, 4, 3, 1, 2, 1, 0, 1, 8, 8, 8),
    # four taps per tile: 9 taps in tiles of 4, 4 and 1; 25 taps at stride 2 with a leading
    # capsule index and 16-row capsules; channel-paired 4x4 capsules; a three-tap window; many
    # images (pixel ranges that begin inside an image)
    ("wgq_k3", 3, 9, 8, 4, 5, 3, 3, 1, 1, 1, 8, 8, 8),
    ("wgq_k5s2", 2, 9, 10, 2, 3, 5, 5, 2, 2, 2, 16, 16, 8),
    ("wgq_44", 3, 9, 8, 8, 4, 3, 3, 1, 1, 1, 4, 4, 4),
    ("wgq_1x3", 2, 6, 9, 3, 4, 1, 3, 1, 1, 1, 8, 8, 8),
    ("wgq_many", 90, 7, 6, 4, 4, 3, 3, 1, 1, 1, 8, 8, 8),
]


@pytest.mark.parametrize("dtype", [wl.FP32, wl.BF16, wl.FP16], ids=["fp32", "bf16", "fp16"])
@pytest.mark.parametrize("shape", BWD_SHAPES, ids=[s[0] for s in BWD_SHAPES])
def test_gradients_match_oracle(shape, dtype):
    both_gradients(small(shape[0], dtype, *shape[1:], seed=len(shape[0]) + 50))


@pytest.mark.parametrize("dtype", [wl.FP32, wl.BF16, wl.FP16], ids=["fp32", "bf16", "fp16"])
@pytest.mark.parametrize("shape", BWD_SHAPES, ids=[s[0] for s in BWD_SHAPES])
def test_integer_data_is_bit_exact(shape, dtype):
    """Small-integer operands: every partial sum is exact in fp32, so both gradients must equal
    the oracle's bit for bit whatever the summation order."""
    w = wl.integer_variant(small(shape[0], dtype, *shape[1:], seed=len(shape[0]) + 60))
    got_i, got_k, dI, dK = both_gradients(w)
    assert np.abs(dI).max() < 2 ** 24 and np.abs(dK).max() < 2 ** 24
    assert np.array_equal(got_i.astype(np.float64), dI)
    assert np.array_equal(got_k.astype(np.float64), dK)


def test_fig2_example_gradients():
    """The worked example's geometry (Fig. 2: 5x5 image of 3x3x3 capsules, 4x4 window)."""
    w = small("fig2", wl.FP32, 1, 5, 5, 1, 1, 4, 4, 1, 0, 3, 3, 3, 3, seed=77)
    both_gradients(w)


@pytest.mark.parametrize("number", [1, 2, 3, 4, 5])
def test_benchmark_configs_reduced_batch(number):
    """The five benchmark shapes with the batch (and, for the largest, the image) cut to what
    the oracle finishes in seconds."""
    full = wl.config(number)
    w = full.with_batch(2)
    if w.flops_nominal() > 5e10:
        w = dataclasses.replace(w, N=1, H=8, W=8)
    both_gradients(w)


@pytest.mark.parametrize("number", [1, 2, 3, 4, 5])
def test_benchmark_configs_full_size_sampled(number):
    """Full benchmark sizes.  dI[n,:,:,c] depends only on image n of the gradient and channel c
    of the kernel, dK[:,:,c,m] only on channel c of the input and channel m of the gradient, so
    the oracle computes sampled slices exactly from sliced operands."""
    w = wl.config(number)
    i_st, k_st, i32, k32 = wl.generate(w)
    g_st, g32 = wl.generate_dout(w)
    i_dev, k_dev, g_dev = (to_device(a, w.dtype) for a in (i_st, k_st, g_st))
    got_i = run_bwd_input(w, g_dev, k_dev)
    got_k = run_bwd_kernel(w, i_dev, g_dev)
    rng = np.random.default_rng(900 + number)
    hw, khw = (w.H, w.W), (w.kh, w.kw)
    for _ in range(3):
        n, c, m = int(rng.integers(w.N)), int(rng.integers(w.C)), int(rng.integers(w.M))
        gs, ks = g32[n:n + 1], np.ascontiguousarray(k32[:, :, c:c + 1])
        ref = capsconv.conv_bwd_input(gs, ks, hw, w.stride, w.pad)
        S = capsconv.conv_bwd_input(np.abs(gs), np.abs(ks), hw, w.stride, w.pad)
        sub = dataclasses.replace(w, name=f"{w.name} dI[{n},:,:,{c}]")
        check(sub, got_i[n:n + 1, :, :, c:c + 1].cpu().numpy(), ref, np.maximum(S, 1e-30))
        isl = np.ascontiguousarray(i32[:, :, :, c:c + 1])
        gsl = np.ascontiguousarray(g32[:, :, :, m:m + 1])
        ref = capsconv.conv_bwd_kernel(isl, gsl, khw, w.stride, w.pad)
        S = capsconv.conv_bwd_kernel(np.abs(isl), np.abs(gsl), khw, w.stride, w.pad)
        sub = dataclasses.replace(w, name=f"{w.name} dK[:,:,{c},{m}]")
        check(sub, got_k[:, :, c:c + 1, m:m + 1].cpu().numpy(), ref, np.maximum(S, 1e-30))
    assert bool(got_i.isfinite().all()) and bool(got_k.isfinite().all())


def test_workspace_too_small_is_refused():
    import torch
    # enough pixels for the kernel gradient to cut its contraction into ranges (partial sums)
    w = small("s1", wl.FP16, 40, 6, 6, 4, 4, 3, 3, 1, 1, 1, 8, 8, 8)
    args = shape_args(w)
    need_i = cc.capscaps_conv_bwd_input_workspace_bytes(*args)
    need_k = cc.capscaps_conv_bwd_kernel_workspace_bytes(*args)
    assert need_i > 0 and need_k > 0
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    p = buf.data_ptr()
    assert cc.capscaps_conv_bwd_input(p, p, p, *args, p, need_i - 1, st) == cc.EWORKSPACE
    assert cc.capscaps_conv_bwd_kernel(p, p, p, *args, 0, 0, st) == cc.EWORKSPACE
    assert cc.capscaps_conv_bwd_input(0, p, p, *args, p, need_i, st) == cc.EINVAL
    # a non-square window takes the gather kernel for dI, which needs no scratch
    # (its kernel gradient: capsule widths of 4 elements go through transposed copies)
    nonsq = small("ns", wl.FP16, 2, 6, 6, 4, 4, 3, 2, 1, 1, 1, 8, 8, 4)
    assert cc.capscaps_conv_bwd_input_workspace_bytes(*shape_args(nonsq)) == 0
    assert cc.capscaps_conv_bwd_kernel_workspace_bytes(*shape_args(nonsq)) > 0
