"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle, element by
element on the same seeded inputs.  Needs an MI355X."""
import dataclasses
import functools

import numpy as np
import pytest

from oracle import capsconv
from paper_2104_02621_amd import capscaps as cc
from paper_2104_02621_amd import workloads as wl
from tests.gpu_util import check, run_gpu, shape_args, to_device

pytestmark = pytest.mark.gpu

PATHS = {"direct": cc.PATH_DIRECT, "mfma": cc.PATH_MFMA, "auto": cc.PATH_AUTO,
         "generic": cc.PATH_MFMA_GENERIC, "tuned16": cc.PATH_MFMA_TUNED16,
         "tuned32": cc.PATH_MFMA_TUNED32, "small": cc.PATH_MFMA_SMALL}


def small(name, dtype, N, H, W, C, M, kh, kw, s, p, D0, D1, D2, D3, dist="normal", seed=0):
    return wl.Workload(name, dtype, N, H, W, C, M, kh, kw, s, p, D0, D1, D2, D3, dist, dist, 1.0,
                       3000 + seed, 4000 + seed)


@functools.lru_cache(maxsize=4)
def oracle_full(w):
    """Inputs and the oracle's full result for a workload (cached across path variants)."""
    i_st, k_st, i32, k32 = wl.generate(w)
    ref, S = capsconv.conv_fwd(i32, k32, w.stride, w.pad, with_abs_sum=True)
    return i_st, k_st, ref, S


def full_compare(w, path):
    i_st, k_st, ref, S = oracle_full(w)
    got = run_gpu(w, to_device(i_st, w.dtype), to_device(k_st, w.dtype), path).cpu().numpy()
    return check(w, got, ref, S, f"path={path}")


# shapes chosen to span several tiles with ragged tails in rows, columns and K, non-square
# capsules (D1 != D2 != D3), leading capsule dimension, strides, padding, 1x1 and wide windows
SMALL_SHAPES = [
    #      N  H   W   C   M  kh kw s  p D0  D1  D2  D3
    ("sq4", 3, 9, 10, 5, 6, 3, 3, 1, 1, 1, 4, 4, 4),
    ("d3x3", 2, 8, 7, 6, 5, 3, 3, 1, 1, 3, 3, 3, 3),
    ("nonsq", 2, 7, 9, 3, 4, 2, 3, 2, 1, 2, 2, 3, 5),
    ("tall", 2, 6, 6, 4, 3, 3, 2, 1, 0, 1, 5, 8, 4),
    ("wide", 1, 12, 11, 8, 9, 3, 3, 2, 2, 1, 8, 8, 8),
    ("d16", 1, 6, 7, 4, 5, 3, 3, 1, 1, 1, 16, 16, 16),
    ("mix16", 2, 5, 6, 3, 7, 1, 1, 1, 0, 2, 4, 16, 8),
    ("k1", 2, 9, 9, 16, 12, 1, 1, 3, 0, 1, 4, 4, 4),
    ("fc", 5, 4, 3, 6, 7, 4, 3, 1, 0, 1, 4, 4, 4),
    ("odd", 1, 10, 9, 7, 3, 5, 4, 1, 2, 1, 3, 5, 7),
    ("manyrows", 4, 20, 20, 4, 20, 3, 3, 1, 1, 1, 8, 8, 8),
    # capsule rows that are half a 16-byte chunk, or an odd number of halves (the any-shape
    # kernel's 8-byte loads): 2 and 6 floats, 12 halves
    ("d2two", 2, 6, 7, 5, 4, 3, 3, 1, 1, 1, 3, 2, 4),
    ("d2twelve", 1, 6, 6, 3, 4, 3, 3, 1, 1, 1, 4, 12, 4),
    # degenerate geometries: a single pixel, a window equal to the padded input, a stride
    # larger than the window, padding wider than the window's reach, scalar capsules
    ("pixel", 1, 1, 1, 3, 2, 1, 1, 1, 0, 1, 2, 3, 2),
    ("whole", 2, 2, 3, 2, 3, 4, 5, 1, 1, 2, 3, 4, 2),
    ("jump", 1, 9, 9, 2, 2, 2, 2, 4, 0, 1, 4, 4, 4),
    ("farpad", 1, 3, 3, 2, 2, 3, 3, 2, 3, 1, 4, 8, 4),
    ("scalar", 2, 6, 6, 5, 7, 3, 3, 1, 1, 1, 1, 1, 1),
]


@pytest.mark.parametrize("dtype", [wl.FP32, wl.BF16, wl.FP16], ids=["fp32", "bf16", "fp16"])
@pytest.mark.parametrize("path", ["direct", "mfma", "generic", "small"])
@pytest.mark.parametrize("shape", SMALL_SHAPES, ids=[s[0] for s in SMALL_SHAPES])
def test_small_shapes_match_oracle(shape, path, dtype):
    w = small(shape[0], dtype, *shape[1:], seed=len(shape[0]))
    full_compare(w, PATHS[path])


# extra shapes for the fp32 kernel with direct-to-LDS copies: partial last channel group
# (C*D2/CW not a multiple of 4), capsule rows of 6 and 12 floats, many rows (4-wave tiles),
# wide column extents (several column tiles), padding wider than the window reach
TUNED32_SHAPES = SMALL_SHAPES + [
    #        N  H   W   C   M  kh kw s  p D0  D1  D2  D3
    ("c5d3", 2, 6, 6, 5, 4, 3, 3, 1, 1, 1, 3, 3, 3),
    ("d6", 1, 7, 6, 3, 5, 2, 2, 1, 0, 2, 4, 6, 3),
    ("d12", 1, 5, 5, 2, 3, 3, 3, 2, 1, 1, 2, 12, 4),
    ("rows", 6, 24, 24, 3, 40, 3, 3, 1, 1, 3, 3, 3, 3),
    ("cols", 2, 10, 10, 4, 70, 3, 3, 1, 2, 1, 4, 4, 4),
]


@pytest.mark.parametrize("shape", TUNED32_SHAPES, ids=[s[0] for s in TUNED32_SHAPES])
def test_tuned_fp32_kernel_matches_oracle(shape):
    if shape[12] % 3 and shape[12] % 4:
        pytest.skip("capsule rows of 1, 2, 5, 7 ... floats are served by the generic kernel")
    w = small(shape[0], wl.FP32, *shape[1:], seed=len(shape[0]) + 70)
    full_compare(w, PATHS["tuned32"])
    wi = small(shape[0] + "_int", wl.FP32, *shape[1:], dist="int", seed=71)
    i_st, k_st, i32, k32 = wl.generate(wi)
    ref = capsconv.conv_fwd(i32, k32, wi.stride, wi.pad)
    got = run_gpu(wi, to_device(i_st, wl.FP32), to_device(k_st, wl.FP32), PATHS["tuned32"])
    assert np.array_equal(got.cpu().numpy().astype(np.float64), ref), wi.name


# 16-bit capsule rows of 4 elements with an even number of channels run on the same lane-per-row
# kernel after a pre-pass has paired the channels: capsules 4x4 (the matrix-capsule shape) and
# non-square, one and many channel pairs (a ragged last stage), a leading capsule index, strides,
# padding, several column tiles, many rows (four-wave tiles), a 1x1 window and an FC layer
PAIRED16_SHAPES = [
    #        N  H   W   C   M  kh kw s  p D0  D1  D2  D3
    ("p4a", 3, 9, 10, 6, 5, 3, 3, 1, 1, 1, 4, 4, 4),
    ("p4b", 2, 8, 7, 2, 3, 3, 3, 2, 1, 2, 4, 4, 4),
    ("p4c", 2, 7, 9, 10, 4, 2, 3, 2, 1, 1, 3, 4, 5),
    ("p4d", 1, 6, 6, 14, 40, 3, 2, 1, 0, 3, 8, 4, 8),
    ("p4rows", 5, 24, 24, 4, 12, 3, 3, 1, 1, 1, 4, 4, 4),
    ("p4k1", 2, 9, 9, 16, 12, 1, 1, 3, 0, 1, 4, 4, 4),
    ("p4fc", 5, 4, 3, 6, 7, 4, 3, 1, 0, 1, 4, 4, 4),
    ("p4pad", 1, 3, 3, 2, 2, 3, 3, 2, 3, 1, 4, 4, 4),
    # ... and rows of 8, 16 and 32 elements, which it takes as they lie in memory: square and
    # non-square capsules, vector capsules (one row), odd channel counts
    ("r8sq", 1, 12, 11, 8, 9, 3, 3, 2, 2, 1, 8, 8, 8),
    ("r16sq", 1, 6, 7, 4, 5, 3, 3, 1, 1, 1, 16, 16, 16),
    ("r16mix", 2, 5, 6, 3, 7, 1, 1, 1, 0, 2, 4, 16, 8),
    ("r8tall", 2, 6, 6, 5, 3, 3, 2, 1, 0, 1, 5, 8, 4),
    ("r8vec", 2, 9, 8, 7, 5, 3, 3, 1, 1, 1, 1, 8, 16),
    ("r32", 1, 5, 6, 3, 4, 2, 2, 1, 0, 1, 2, 32, 4),
    ("r8rows", 4, 20, 20, 4, 20, 3, 3, 1, 1, 1, 8, 8, 8),
]


@pytest.mark.parametrize("dtype", [wl.BF16, wl.FP16], ids=["bf16", "fp16"])
@pytest.mark.parametrize("shape", PAIRED16_SHAPES, ids=[s[0] for s in PAIRED16_SHAPES])
def test_lane_per_row_kernel_on_16bit_operands(shape, dtype):
    w = small(shape[0], dtype, *shape[1:], seed=len(shape[0]) + 75)
    full_compare(w, PATHS["tuned32"])
    wi = small(shape[0] + "_int", dtype, *shape[1:], dist="int", seed=76)
    i_st, k_st, i32, k32 = wl.generate(wi)
    ref = capsconv.conv_fwd(i32, k32, wi.stride, wi.pad)
    got = run_gpu(wi, to_device(i_st, dtype), to_device(k_st, dtype), PATHS["tuned32"])
    assert np.array_equal(got.cpu().numpy().astype(np.float64), ref), wi.name


# shapes the 256x256-tile 16-bit kernel accepts (D1 = D2 in {8, 16}, C*D2 a multiple of 64):
# ragged row tiles, tiles that straddle images, several column tiles with a ragged last one,
# leading capsule dimension, strides, padding wider than the window reach, D3 != D1
TUNED_SHAPES = [
    #        N  H   W   C   M  kh kw s  p D0  D1  D2  D3
    ("t16a", 2, 9, 7, 4, 5, 3, 3, 1, 1, 1, 16, 16, 16),
    ("t16b", 3, 6, 5, 8, 20, 2, 3, 2, 2, 2, 16, 16, 4),
    ("t16c", 1, 20, 20, 4, 3, 1, 1, 1, 0, 1, 16, 16, 8),
    ("t8a", 2, 11, 9, 8, 9, 3, 3, 1, 1, 1, 8, 8, 8),
    ("t8b", 5, 5, 4, 16, 40, 3, 2, 2, 1, 3, 8, 8, 12),
    ("t8c", 1, 30, 30, 8, 4, 3, 3, 1, 3, 1, 8, 8, 4),
]


@pytest.mark.parametrize("dtype", [wl.BF16, wl.FP16], ids=["bf16", "fp16"])
@pytest.mark.parametrize("shape", TUNED_SHAPES, ids=[s[0] for s in TUNED_SHAPES])
def test_tuned_16bit_kernel_matches_oracle(shape, dtype):
    w = small(shape[0], dtype, *shape[1:], seed=len(shape[0]) + 50)
    full_compare(w, PATHS["tuned16"])
    wi = small(shape[0] + "_int", dtype, *shape[1:], dist="int", seed=61)
    i_st, k_st, i32, k32 = wl.generate(wi)
    ref = capsconv.conv_fwd(i32, k32, wi.stride, wi.pad)
    got = run_gpu(wi, to_device(i_st, dtype), to_device(k_st, dtype), PATHS["tuned16"]).cpu().numpy()
    assert np.array_equal(got.astype(np.float64), ref), wi.name


@pytest.mark.parametrize("dtype", [wl.BF16, wl.FP16], ids=["bf16", "fp16"])
@pytest.mark.parametrize("shape", [
    #        N   H   W   C   M  kh kw s  p D0  D1  D2  D3
    ("h16", 3, 30, 30, 4, 16, 3, 3, 1, 1, 1, 16, 16, 16),   # 169 tiles of 256 rows, 338 of 128
    ("h8", 5, 61, 59, 8, 20, 3, 3, 2, 2, 1, 8, 8, 12),      # ragged last tile and columns
], ids=["h16", "h8"])
def test_tuned_16bit_kernel_half_height_tiles(shape, dtype):
    """Problems that fill the chip with 128-row tiles but not with 256-row ones take the tuned
    kernel's half-height variant (two workgroups per CU) on the library's own choice."""
    w = small(shape[0], dtype, *shape[1:], seed=len(shape[0]) + 70)
    assert cc.capscaps_select_path(*shape_args(w)) == cc.PATH_MFMA_TUNED16
    rows = w.N * w.Ho * w.Wo * w.D1
    assert (rows + 255) // 256 * ((w.M * w.D3 + 255) // 256) < 256 <= (rows + 127) // 128 * ((w.M * w.D3 + 255) // 256)
    full_compare(w, cc.PATH_AUTO)
    wi = small(shape[0] + "_int", dtype, *shape[1:], dist="int", seed=71)
    i_st, k_st, i32, k32 = wl.generate(wi)
    ref = capsconv.conv_fwd(i32, k32, wi.stride, wi.pad)
    got = run_gpu(wi, to_device(i_st, dtype), to_device(k_st, dtype), cc.PATH_AUTO).cpu().numpy()
    assert np.array_equal(got.astype(np.float64), ref), wi.name


@pytest.mark.parametrize("dtype", [wl.BF16, wl.FP16], ids=["bf16", "fp16"])
def test_tuned_16bit_kernel_short_k_loop(dtype):
    """A K loop of few stages takes the half-height tiles even where 256-row tiles would fill the
    chip (18 stages here); each XCD then works on a contiguous range of tiles."""
    shape = ("hk", 8, 32, 32, 8, 32, 3, 3, 1, 1, 1, 8, 8, 8)
    w = small(shape[0], dtype, *shape[1:], seed=77)
    assert cc.capscaps_select_path(*shape_args(w)) == cc.PATH_MFMA_TUNED16
    rows = w.N * w.Ho * w.Wo * w.D1
    assert rows // 256 >= 256 and w.kh * w.kw * w.C * w.D2 // 32 <= 96
    full_compare(w, cc.PATH_AUTO)
    wi = small(shape[0] + "_int", dtype, *shape[1:], dist="int", seed=78)
    i_st, k_st, i32, k32 = wl.generate(wi)
    ref = capsconv.conv_fwd(i32, k32, wi.stride, wi.pad)
    got = run_gpu(wi, to_device(i_st, dtype), to_device(k_st, dtype), cc.PATH_AUTO).cpu().numpy()
    assert np.array_equal(got.astype(np.float64), ref), wi.name


def test_window_of_64_taps_leaves_the_tuned_kernel():
    """The tuned 16-bit kernel keeps one bit of a 64-bit mask per window tap and one bit free:
    63 taps run on it, 64 go to the generic kernel."""
    import torch
    for kh, kw, tuned in ((7, 9, True), (8, 8, False)):
        w = small(f"taps{kh * kw}", wl.BF16, 64, 15, 16, 8, 4, kh, kw, 1, 0, 1, 8, 8, 8, seed=79)
        assert (cc.capscaps_select_path(*shape_args(w)) == cc.PATH_MFMA_TUNED16) == tuned, w.name
        if tuned:
            full_compare(w, cc.PATH_AUTO)
            continue
        I = torch.zeros(w.input_shape, dtype=torch.bfloat16, device="cuda")
        K = torch.zeros(w.kernel_shape, dtype=torch.bfloat16, device="cuda")
        out = torch.zeros(w.out_shape, device="cuda")
        ws = torch.empty(1 << 24, dtype=torch.uint8, device="cuda")
        rc = cc.capscaps_conv_fwd_path(I.data_ptr(), K.data_ptr(), out.data_ptr(),
                                       *shape_args(w)[:13], w.dtype, cc.PATH_MFMA_TUNED16,
                                       ws.data_ptr(), ws.numel(), None)
        assert rc == cc.EUNSUPPORTED
        full_compare(w, cc.PATH_AUTO)


def test_tuned_kernel_refuses_other_shapes():
    import torch
    w = small("no", wl.FP32, 1, 6, 6, 4, 4, 3, 3, 1, 1, 1, 16, 16, 16)
    I = torch.zeros(w.input_shape, device="cuda")
    K = torch.zeros(w.kernel_shape, device="cuda")
    out = torch.zeros(w.out_shape, device="cuda")
    ws = torch.empty(1 << 22, dtype=torch.uint8, device="cuda")
    rc = cc.capscaps_conv_fwd_path(I.data_ptr(), K.data_ptr(), out.data_ptr(), *shape_args(w)[:13],
                                   w.dtype, cc.PATH_MFMA_TUNED16, ws.data_ptr(), ws.numel(), None)
    assert rc == cc.EUNSUPPORTED


@pytest.mark.parametrize("path", ["direct", "mfma", "auto"])
def test_paper_worked_example_on_gpu(path):
    """Fig. 2: all-ones 5x5 input of 3x3x3 capsules, all-ones 4x4 kernel -> 2x2 of 48s."""
    import torch
    w = small("fig2", wl.FP32, 1, 5, 5, 1, 1, 4, 4, 1, 0, 3, 3, 3, 3)
    I = torch.ones(w.input_shape, device="cuda")
    K = torch.ones(w.kernel_shape, device="cuda")
    got = run_gpu(w, I, K, PATHS[path]).cpu().numpy()
    assert got.shape == (1, 2, 2, 1, 3, 3, 3) and np.all(got == 48.0)


@pytest.mark.parametrize("dtype", [wl.FP32, wl.BF16, wl.FP16], ids=["fp32", "bf16", "fp16"])
@pytest.mark.parametrize("path", ["direct", "mfma", "generic", "small"])
def test_small_integer_inputs_are_bit_exact(path, dtype):
    """Integer inputs in [-3,3]: every partial sum is exact in fp32, so any summation order
    must give exactly the oracle's result -- sharp against tile-edge, halo and split errors."""
    for shape in (SMALL_SHAPES[0], SMALL_SHAPES[2], SMALL_SHAPES[4], SMALL_SHAPES[8]):
        w = small(shape[0], dtype, *shape[1:], dist="int", seed=11)
        i_st, k_st, i32, k32 = wl.generate(w)
        ref = capsconv.conv_fwd(i32, k32, w.stride, w.pad)
        got = run_gpu(w, to_device(i_st, dtype), to_device(k_st, dtype), PATHS[path]).cpu().numpy()
        assert np.array_equal(got.astype(np.float64), ref), f"{w.name} {path}"


@pytest.mark.parametrize("num", [1, 4])
@pytest.mark.parametrize("path", ["direct", "mfma", "auto", "generic", "tuned32", "small"])
def test_benchmark_configs_full_tensor(num, path):
    full_compare(wl.config(num), PATHS[path])


@pytest.mark.parametrize("path", ["direct", "generic", "tuned16", "tuned32"])
@pytest.mark.parametrize("num,batch,hw", [(2, 2, 32), (3, 2, 28), (5, 2, 6)])
def test_benchmark_configs_reduced_full_tensor(num, batch, hw, path):
    """Configs 2, 3, 5 with fewer images (config 5 also with a smaller image, to keep the
    oracle's run to seconds): every pixel, channel and border, whole tensor compared."""
    w = wl.config(num)
    w = dataclasses.replace(w, N=batch, H=hw, W=hw, name=f"{w.name}[N={batch},HW={hw}]")
    if path == "tuned16" and w.dtype == wl.FP32:
        pytest.skip("the tuned 16-bit kernel is for 16-bit element types")
    full_compare(w, PATHS[path])


@functools.lru_cache(maxsize=1)
def full_size_run(num):
    """A benchmark configuration at full size in the launch configuration the bench times: its
    fp32 inputs and the GPU's output (kept on the device), shared by the checks below."""
    import torch
    w = wl.config(num)
    i_st, k_st, i32, k32 = wl.generate(w)
    out = run_gpu(w, to_device(i_st, w.dtype), to_device(k_st, w.dtype), cc.PATH_AUTO)
    torch.cuda.synchronize()
    return w, i32, k32, out


# (configuration, part): 12000 / 12000 / 10000 sampled output capsules (a quarter of them on
# image borders) plus finiteness of the whole tensor; for the two 16-bit configurations also the
# first and the last image whole -- every border, tile edge and tile tail of an image, and the
# last tiles of the launch
FULL_SIZE_PARTS = [(2, "sampled"), (3, "sampled"), (3, "first image"), (3, "last image"),
                   (5, "sampled"), (5, "first image"), (5, "last image")]


@pytest.mark.parametrize("num,part", FULL_SIZE_PARTS,
                         ids=[f"config{n}-{p.replace(' ', '-')}" for n, p in FULL_SIZE_PARTS])
def test_benchmark_configs_full_size(num, part):
    import torch
    w, i32, k32, out = full_size_run(num)
    if part == "sampled":
        assert bool(torch.isfinite(out).all())
        which = wl.sample_capsules(w, {2: 12000, 3: 12000, 5: 10000}[num], seed=77 + num)
        ref, S = capsconv.conv_fwd_subset(i32, k32, which, w.stride, w.pad, with_abs_sum=True)
        idx = torch.from_numpy(which.astype(np.int64)).cuda()
        got = out[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy()
        check(w, got, ref, S, "sampled")
        return
    n = 0 if part == "first image" else w.N - 1
    ref, S = capsconv.conv_fwd(i32[n:n + 1], k32, w.stride, w.pad, with_abs_sum=True)
    check(w, out[n:n + 1].cpu().numpy(), ref, S, part)


@pytest.mark.parametrize("num", [3, 5])
def test_full_size_integer_data_every_output(num):
    """Configs 3 and 5 at full size on small-integer data, where every partial sum is exact in
    fp32: EVERY output element is compared with the generic kernel's (bit for bit) and with the
    framework's grouped convolution (an independent implementation of the same operator, itself
    checked against the oracle in test_gpu_comparisons.py and on the CPU), and sampled capsules
    with the oracle, exactly.  A wrong tile edge, halo or stage anywhere in the tensor shows as
    a difference of at least 1."""
    import torch
    from paper_2104_02621_amd import comparisons as cmp
    w = wl.integer_variant(wl.config(num))
    i_st, k_st, i32, k32 = wl.generate(w)
    i_dev, k_dev = to_device(i_st, w.dtype), to_device(k_st, w.dtype)
    out = run_gpu(w, i_dev, k_dev, cc.PATH_AUTO)
    which = wl.sample_capsules(w, 1500, seed=91 + num)
    ref = capsconv.conv_fwd_subset(i32, k32, which, w.stride, w.pad)
    assert np.abs(ref).max() < 2 ** 24
    idx = torch.from_numpy(which.astype(np.int64)).cuda()
    got = out[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy()
    assert np.array_equal(got.astype(np.float64), ref)
    # a second kernel of this library with other tiles and addressing: identical everywhere
    generic = run_gpu(w, i_dev, k_dev, cc.PATH_MFMA_GENERIC)
    assert bool(torch.equal(out, generic))
    del generic
    other = cmp.framework_conv_fwd(i_dev, k_dev, w.stride, w.pad)   # fp32 arithmetic
    assert other.shape == out.shape
    # Where the two differ by more than rounding noise of a transform-based algorithm (the exact
    # results are integers), the oracle decides who is right.  (Seen on MI355X: the framework's
    # result for config 5 is off by up to 3 in a few thousand elements of the last image.)
    differ = torch.nonzero((out - other).abs() > 0.25)
    print(f"{w.name}: {differ.shape[0]} of {out.numel()} outputs differ from the framework's")
    if differ.shape[0] > 0:
        caps = np.unique(differ[:100000, :4].cpu().numpy(), axis=0)[:200].astype(np.int32)
        ref = capsconv.conv_fwd_subset(i32, k32, caps, w.stride, w.pad)
        cidx = torch.from_numpy(caps.astype(np.int64)).cuda()
        mine = out[cidx[:, 0], cidx[:, 1], cidx[:, 2], cidx[:, 3]].cpu().numpy()
        assert np.array_equal(mine.astype(np.float64), ref)
        assert differ.shape[0] < out.numel() // 1000, "the two implementations disagree widely"


def test_offsets_beyond_4GB():
    """A config-5-like layer whose input (5.4 GB) and output (10.7 GB) exceed 32-bit byte
    offsets: output capsules sampled from the last images, where every address is past 4 GB."""
    import torch
    w = dataclasses.replace(wl.config(5), N=160, name="large_caps_fp16[N=160]")
    rng = np.random.default_rng(99)
    # seeded inputs of the workload's distributions, drawn image by image to bound host memory
    I = torch.empty(w.input_shape, dtype=torch.float16, device="cuda")
    per_image = int(np.prod(w.input_shape[1:]))
    tail = {}
    for n in range(w.N):
        img = rng.standard_normal(per_image, dtype=np.float32).astype(np.float16)
        I[n] = torch.from_numpy(img).cuda().view(w.input_shape[1:])
        if n >= w.N - 2:
            tail[n] = img.reshape(w.input_shape[1:])
    k16 = (rng.standard_normal(w.kernel_shape, dtype=np.float32) * np.float32(w.kernel_sigma)) \
        .astype(np.float16)
    K = torch.from_numpy(k16).cuda()
    out = run_gpu(w, I, K, cc.PATH_AUTO)
    assert bool(torch.isfinite(out[-2:]).all())
    # oracle on the last two images only (same values, re-indexed as a 2-image problem)
    i2 = np.stack([tail[w.N - 2], tail[w.N - 1]]).astype(np.float32)
    w2 = dataclasses.replace(w, N=2)
    which = wl.sample_capsules(w2, 400, seed=5)
    ref, S = capsconv.conv_fwd_subset(i2, k16.astype(np.float32), which, w.stride, w.pad,
                                      with_abs_sum=True)
    idx = torch.from_numpy(which.astype(np.int64)).cuda()
    got = out[idx[:, 0] + (w.N - 2), idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy()
    check(w, got, ref, S, "last images of a >4 GB tensor")


def test_split_reduction_is_deterministic():
    """Config 4 splits its K loop over many blocks; partial sums are reduced in a fixed order."""
    import torch
    w = wl.config(4)
    i_st, k_st, _, _ = wl.generate(w)
    I, K = to_device(i_st, w.dtype), to_device(k_st, w.dtype)
    for path in (cc.PATH_MFMA, cc.PATH_MFMA_GENERIC, cc.PATH_MFMA_SMALL):
        a = run_gpu(w, I, K, path)
        b = run_gpu(w, I, K, path)
        assert torch.equal(a, b), path


def test_plain_entry_point_allocates_its_own_scratch():
    """capscaps_conv_fwd (the paper's pad-free operator, stream-ordered scratch)."""
    import torch
    w = wl.config(1)
    i_st, k_st, i32, k32 = wl.generate(w)
    I, K = to_device(i_st, w.dtype), to_device(k_st, w.dtype)
    out = torch.full(w.out_shape, float("nan"), dtype=torch.float32, device="cuda")
    rc = cc.capscaps_conv_fwd(I.data_ptr(), K.data_ptr(), out.data_ptr(), w.N, w.H, w.W, w.C, w.M,
                              w.kh, w.kw, w.stride, w.D0, w.D1, w.D2, w.D3, w.dtype,
                              torch.cuda.current_stream().cuda_stream)
    assert rc == cc.OK
    ref, S = capsconv.conv_fwd(i32, k32, w.stride, 0, with_abs_sum=True)
    check(w, out.cpu().numpy(), ref, S, "plain entry point")


def test_torch_wrapper_and_side_stream():
    import torch
    w = small("wrap", wl.FP16, 2, 8, 8, 8, 8, 3, 3, 1, 1, 1, 8, 8, 8)
    i_st, k_st, i32, k32 = wl.generate(w)
    I, K = to_device(i_st, w.dtype), to_device(k_st, w.dtype)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        out = cc.conv_fwd(I, K, stride=1, pad=1)
    s.synchronize()
    ref, S = capsconv.conv_fwd(i32, k32, 1, 1, with_abs_sum=True)
    check(w, out.cpu().numpy(), ref, S, "wrapper")


GRAPH_CASES = {
    # split-K path: repack, MFMA kernel, reduction; and both gradients
    "config4": lambda: wl.config(4),
    # a strided 16-bit layer of 4x4 capsules: channel-pairing pre-passes, the input gradient as four
    # phase convolutions through output views, the kernel gradient with two taps per tile and a
    # reduction over pixel ranges
    "strided4x4": lambda: small("g4x4", wl.BF16, 14, 80, 78, 4, 8, 3, 3, 2, 1, 1, 4, 4, 4, seed=31),
    # stride 3 under a 2x2 window: one phase of input pixels no window reaches (zeroed by a kernel)
    "stride3": lambda: small("gs3", wl.FP16, 3, 120, 118, 4, 8, 2, 2, 3, 0, 1, 8, 4, 8, seed=32),
}


@pytest.mark.parametrize("case", list(GRAPH_CASES))
def test_calls_can_be_captured_in_a_graph(case):
    """With caller-provided scratch the library only enqueues kernels on the stream it is given
    (no allocation, no memset, no synchronisation), so a call can be captured in a HIP graph.
    Replays, with eager work and synchronisations between them, must reproduce the eager
    result every time."""
    import torch
    w = GRAPH_CASES[case]()
    i_st, k_st, _, _ = wl.generate(w)
    g_st, _ = wl.generate_dout(w)
    I, K, G = (to_device(a, w.dtype) for a in (i_st, k_st, g_st))
    args = shape_args(w)
    out = torch.zeros(w.out_shape, dtype=torch.float32, device="cuda")
    din = torch.zeros(w.input_shape, dtype=torch.float32, device="cuda")
    dk = torch.zeros(w.kernel_shape, dtype=torch.float32, device="cuda")
    half = w.dtype != wl.FP32  # 16-bit operands: the 16-bit input gradient as well
    din16 = torch.zeros(w.input_shape, dtype=I.dtype, device="cuda") if half else None
    ws = [torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
          for n in (cc.capscaps_conv_fwd_workspace_bytes(*args),
                    cc.capscaps_conv_bwd_input_workspace_bytes(*args),
                    cc.capscaps_conv_bwd_kernel_workspace_bytes(*args),
                    cc.capscaps_conv_bwd_input_out16_workspace_bytes(*args) if half else 0)]

    def step(st):
        assert cc.capscaps_conv_fwd_ex(I.data_ptr(), K.data_ptr(), out.data_ptr(), *args,
                                       ws[0].data_ptr(), ws[0].numel(), st) == cc.OK
        assert cc.capscaps_conv_bwd_input(G.data_ptr(), K.data_ptr(), din.data_ptr(), *args,
                                          ws[1].data_ptr(), ws[1].numel(), st) == cc.OK
        assert cc.capscaps_conv_bwd_kernel(I.data_ptr(), G.data_ptr(), dk.data_ptr(), *args,
                                           ws[2].data_ptr(), ws[2].numel(), st) == cc.OK
        if half:
            assert cc.capscaps_conv_bwd_input_out16(G.data_ptr(), K.data_ptr(), din16.data_ptr(),
                                                    *args, ws[3].data_ptr(), ws[3].numel(),
                                                    st) == cc.OK

    results = (out, din, dk) + ((din16,) if half else ())
    step(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    eager = [t.clone() for t in results]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(side.cuda_stream)
    for k in range(4):
        for t in results:
            t.fill_(float(k))            # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, e in zip(results, eager):
            assert torch.equal(t, e), f"replay {k}"
    assert all(bool(e.isfinite().all()) for e in eager)


def test_workspace_too_small_is_refused_before_any_launch():
    import torch
    w = wl.config(1)
    I = torch.zeros(w.input_shape, device="cuda")
    K = torch.zeros(w.kernel_shape, device="cuda")
    out = torch.full(w.out_shape, 7.0, device="cuda")
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    rc = cc.capscaps_conv_fwd_path(I.data_ptr(), K.data_ptr(), out.data_ptr(), *shape_args(w)[:13],
                                   w.dtype, cc.PATH_MFMA_GENERIC, ws.data_ptr(), 256, None)
    assert rc == cc.EWORKSPACE
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
