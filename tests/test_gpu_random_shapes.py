"""GPU parity on seeded random layer shapes: forward pass (the library's own path choice) and
both gradients against the CPU oracle.  The hand-picked shapes of the other files aim at
known tile edges; these reach combinations nobody thought of (capsule shapes, windows wider
than high, strides up to 3, paddings up to the window, one to many channels).  Needs an MI355X."""
import numpy as np
import pytest

from paper_2104_02621_amd import workloads as wl
from tests.test_gpu_bwd_parity import both_gradients
from tests.test_gpu_parity import full_compare, small
from paper_2104_02621_amd import capscaps as cc

pytestmark = pytest.mark.gpu

CAPSULE_DIMS = [1, 2, 3, 4, 5, 6, 8, 12, 16]


def random_shape(seed):
    """A layer small enough for the oracle to take well under a second."""
    rng = np.random.default_rng(90000 + seed)
    while True:
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        s = int(rng.integers(1, 4))
        p = int(rng.integers(0, max(kh, kw) + 1))
        H, W = int(rng.integers(1, 20)), int(rng.integers(1, 20))
        if kh > H + 2 * p or kw > W + 2 * p:
            continue
        N = int(rng.integers(1, 6))
        C, M = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        D0 = int(rng.choice([1, 1, 1, 2, 3]))
        if rng.random() < 0.5:  # square capsules, the kind the tuned kernels take
            D1 = D2 = D3 = int(rng.choice([3, 4, 8, 16]))
        else:
            D1, D2, D3 = (int(rng.choice(CAPSULE_DIMS)) for _ in range(3))
        Ho, Wo = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
        flops = 2.0 * N * Ho * Wo * M * D0 * D1 * D3 * kh * kw * C * D2
        if flops <= 3e8:
            return (N, H, W, C, M, kh, kw, s, p, D0, D1, D2, D3)


def random_medium_shape(seed):
    """A layer with enough rows for the tuned kernels' 256-row tiles to fill the chip (or nearly):
    square capsules of the element type's kind, a few seconds of oracle."""
    rng = np.random.default_rng(95000 + seed)
    dtype = [wl.FP32, wl.BF16, wl.FP16][seed % 3]
    while True:
        D = int(rng.choice([3, 4, 6, 8] if dtype == wl.FP32 else [4, 8, 16]))
        D0 = int(rng.choice([1, 1, 2, 3])) if dtype == wl.FP32 else 1
        kh, kw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        s = int(rng.integers(1, 3))
        p = int(rng.integers(0, 3))
        H, W = int(rng.integers(12, 41)), int(rng.integers(12, 41))
        N = int(rng.integers(4, 33))
        C, M = 8 * int(rng.integers(1, 9)), 8 * int(rng.integers(1, 9))
        Ho, Wo = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
        rows = N * Ho * Wo * D
        flops = 2.0 * rows * M * D0 * D * kh * kw * C * D
        if rows >= 200 * 256 and flops <= 8e9:
            return dtype, (N, H, W, C, M, kh, kw, s, p, D0, D, D, D)


def random_mixed16_shape(seed):
    """A 16-bit layer of non-square, vector (one or two rows) or 4-row capsules with enough rows for
    the lane-per-row kernel's 256-row tiles and the in-place kernel-gradient kernel."""
    rng = np.random.default_rng(97000 + seed)
    dtype = [wl.BF16, wl.FP16][seed % 2]
    while True:
        D1 = int(rng.choice([1, 2, 4, 8, 16]))
        D2 = int(rng.choice([4, 8, 16, 32]))
        D3 = int(rng.choice([4, 8, 16]))
        kh, kw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        s = int(rng.integers(1, 3))
        p = int(rng.integers(0, 3))
        H, W = int(rng.integers(12, 49)), int(rng.integers(12, 49))
        N = int(rng.integers(4, 49))
        C, M = 2 * int(rng.integers(1, 25)), 2 * int(rng.integers(1, 25))
        Ho, Wo = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
        rows = N * Ho * Wo * D1
        flops = 2.0 * rows * M * D3 * kh * kw * C * D2
        if rows >= 260 * 256 and flops <= 8e9:
            return dtype, (N, H, W, C, M, kh, kw, s, p, 1, D1, D2, D3)


def random_few_rows_shape(seed):
    """A 16-bit layer with at most 128 rows (c, d2), for the kernel gradient's tiles of two or four
    window taps: windows up to 5x5, strides up to 3, paddings up to 3, one to many images (pixel
    ranges that begin inside an image), 4x4 capsules with paired channels among them."""
    rng = np.random.default_rng(99000 + seed)
    while True:
        if rng.random() < 0.25:
            D1 = D2 = D3 = 4
            C, M = 2 * int(rng.integers(1, 17)), 2 * int(rng.integers(1, 9))
        else:
            D1, D2, D3 = int(rng.choice([4, 8, 16])), int(rng.choice([8, 16, 24])), int(rng.choice([8, 16]))
            C, M = int(rng.integers(1, 128 // D2 + 1)), int(rng.integers(1, 12))
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        s, p = int(rng.integers(1, 4)), int(rng.integers(0, 4))
        H, W = int(rng.integers(1, 15)), int(rng.integers(1, 15))
        if kh > H + 2 * p or kw > W + 2 * p:
            continue
        N = int(rng.choice([1, 2, 3, 7, 40, 130]))
        D0 = int(rng.choice([1, 1, 2]))
        Ho, Wo = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
        if 2.0 * N * Ho * Wo * M * D0 * D1 * D3 * kh * kw * C * D2 <= 4e8:
            return [wl.BF16, wl.FP16][seed % 2], (N, H, W, C, M, kh, kw, s, p, D0, D1, D2, D3)


SEEDS = list(range(60))
MEDIUM_SEEDS = list(range(15))
MIXED16_SEEDS = list(range(14))


@pytest.mark.parametrize("seed", SEEDS)
def test_random_layer_forward_and_gradients(seed):
    shape = random_shape(seed)
    dtype = [wl.FP32, wl.BF16, wl.FP16][seed % 3]
    w = small("rand%d_" % seed + "x".join(map(str, shape)), dtype, *shape, seed=700 + seed)
    print(w.name, flush=True)
    full_compare(w, cc.PATH_AUTO)
    both_gradients(w)


@pytest.mark.parametrize("seed", MEDIUM_SEEDS)
def test_random_medium_layer_forward_and_gradients(seed):
    dtype, shape = random_medium_shape(seed)
    w = small("randm%d_" % seed + "x".join(map(str, shape)), dtype, *shape, seed=800 + seed)
    print(w.name, cc.capscaps_select_path(*shape, dtype), flush=True)
    full_compare(w, cc.PATH_AUTO)
    both_gradients(w)


@pytest.mark.parametrize("seed", MIXED16_SEEDS)
def test_random_mixed_16bit_layer_forward_and_gradients(seed):
    dtype, shape = random_mixed16_shape(seed)
    w = small("randx%d_" % seed + "x".join(map(str, shape)), dtype, *shape, seed=900 + seed)
    print(w.name, cc.capscaps_select_path(*shape, dtype), flush=True)
    full_compare(w, cc.PATH_AUTO)
    both_gradients(w)


@pytest.mark.parametrize("seed", list(range(40)))
def test_random_few_rows_16bit_layer_gradients(seed):
    dtype, shape = random_few_rows_shape(seed)
    w = small("randr%d_" % seed + "x".join(map(str, shape)), dtype, *shape, seed=950 + seed)
    print(w.name, flush=True)
    both_gradients(w)
