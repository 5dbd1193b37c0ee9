"""Seeded synthetic inputs for the capsule-convolution forward pass.

This module holds shapes, seeds, value distributions and storage-type rounding only: none
of the operator's arithmetic.  It is the one module both the GPU tests/bench and the CPU
oracle's callers draw inputs from, so that both sides see bit-identical operands.

The paper names no dataset and its sample network's figure carries no shapes, so the five
workloads below (the benchmark configurations of this build) stand in for its layers.
Tensors use the library's dense layouts:
    input  [N][H][W][C][D0][D1][D2]      kernel [kh][kw][C][M][D0][D2][D3]
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

FP32, BF16, FP16 = 0, 1, 2
DTYPE_NAMES = {FP32: "fp32", BF16: "bf16", FP16: "fp16"}


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: int
    N: int
    H: int
    W: int
    C: int
    M: int
    kh: int
    kw: int
    stride: int
    pad: int
    D0: int
    D1: int
    D2: int
    D3: int
    input_dist: str      # "uniform" (U[-1,1]) | "normal" (N(0,1)) | "int" (integers in [-3,3])
    kernel_dist: str     # "uniform" | "normal" | "int"
    kernel_sigma: float  # std-dev for "normal" kernels
    seed_input: int
    seed_kernel: int

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def input_shape(self):
        return (self.N, self.H, self.W, self.C, self.D0, self.D1, self.D2)

    @property
    def kernel_shape(self):
        return (self.kh, self.kw, self.C, self.M, self.D0, self.D2, self.D3)

    @property
    def out_shape(self):
        return (self.N, self.Ho, self.Wo, self.M, self.D0, self.D1, self.D3)

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == FP32 else 2

    def flops_nominal(self) -> int:
        """2 * (multiply-adds), padding taps counted."""
        return (2 * self.N * self.Ho * self.Wo * self.M * self.D0 * self.D1 * self.D3
                * self.kh * self.kw * self.C * self.D2)

    def flops_tap_exact(self) -> int:
        """2 * (multiply-adds) against in-range input pixels only."""
        def in_range(extent, out_extent, k):
            cnt = 0
            for o in range(out_extent):
                for t in range(k):
                    i = o * self.stride - self.pad + t
                    cnt += 0 <= i < extent
            return cnt
        taps = in_range(self.H, self.Ho, self.kh) * in_range(self.W, self.Wo, self.kw)
        return 2 * self.N * taps * self.M * self.D0 * self.D1 * self.D3 * self.C * self.D2

    def compulsory_bytes(self) -> int:
        """Input once + kernel once + fp32 output once."""
        n_in = int(np.prod(self.input_shape))
        n_k = int(np.prod(self.kernel_shape))
        n_out = int(np.prod(self.out_shape))
        return (n_in + n_k) * self.elem_bytes + n_out * 4

    def with_batch(self, N: int) -> "Workload":
        return replace(self, N=N, name=f"{self.name}[N={N}]")


def _w(name, dtype, N, HW, C, M, k, stride, pad, D0, D, idist, kdist, sigma, num):
    return Workload(name, dtype, N, HW, HW, C, M, k, k, stride, pad, D0, D, D, D, idist, kdist,
                    sigma, 1000 + num, 2000 + num)


CONFIGS = (
    _w("caps_conv_fp32_small", FP32, 8, 16, 4, 4, 3, 1, 0, 1, 4, "uniform", "uniform", 1.0, 1),
    _w("pcapsnet_3d_fp32", FP32, 64, 32, 32, 32, 3, 1, 1, 3, 3, "uniform", "normal",
       1.0 / np.sqrt(9 * 32 * 3), 2),
    _w("strided_bf16", BF16, 128, 28, 64, 64, 3, 2, 1, 1, 8, "normal", "normal",
       1.0 / np.sqrt(9 * 64 * 8), 3),
    _w("fc_caps_fp32", FP32, 256, 6, 32, 10, 6, 1, 0, 1, 4, "uniform", "normal", 0.02, 4),
    _w("large_caps_fp16", FP16, 64, 32, 64, 64, 3, 1, 1, 1, 16, "normal", "normal",
       1.0 / np.sqrt(9 * 64 * 16), 5),
)


def net5(N: int = 64, dtype: int = BF16):
    """A five-layer stack of capsule convolutions (the paper's experiment, Sec. 3, is a
    five-layer convolutional CapsNet; the figure with its shapes is not available, so these are
    stand-ins of the benchmark configurations' kind): 8x8 capsules, 32x32 images, two strided
    layers, a fully-connected last layer.  Layer k's output (in the operands' 16-bit type) is
    layer k+1's input; kernels N(0, 1/fan-in) keep the activations at unit scale."""
    #          HW   C   M  k  s  p
    layers = ((32, 16, 32, 3, 1, 1),
              (32, 32, 32, 3, 2, 1),
              (16, 32, 64, 3, 1, 1),
              (16, 64, 64, 3, 2, 1),
              (8, 64, 10, 8, 1, 0))
    D = 8
    return tuple(
        Workload(f"net5_layer{k + 1}", dtype, N, hw, hw, c, m, ksz, ksz, s_, p_, 1, D, D, D,
                 "normal", "normal", 1.0 / float(np.sqrt(ksz * ksz * c * D)), 5000 + k, 6000 + k)
        for k, (hw, c, m, ksz, s_, p_) in enumerate(layers))


def config(number: int) -> Workload:
    """Benchmark configuration 1..5."""
    return CONFIGS[number - 1]


# ----------------------------------------------------------------------------- rounding
def round_to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b16: np.ndarray) -> np.ndarray:
    return (b16.astype(np.uint32) << 16).view(np.float32)


def to_storage(x32: np.ndarray, dtype: int):
    """Round float32 values once to the run's storage type.

    Returns (storage, widened): `storage` is what is uploaded to the GPU (float32, uint16
    holding bf16 bits, or float16); `widened` is the same values as float32 (exact)."""
    if dtype == FP32:
        x = np.ascontiguousarray(x32, dtype=np.float32)
        return x, x
    if dtype == BF16:
        bits = round_to_bf16_bits(x32)
        return bits, bf16_bits_to_f32(bits)
    if dtype == FP16:
        h = np.ascontiguousarray(x32, dtype=np.float32).astype(np.float16)
        return h, h.astype(np.float32)
    raise ValueError(f"unknown dtype {dtype}")


# ----------------------------------------------------------------------------- generators
def _draw(rng, shape, dist, sigma):
    if dist == "uniform":
        x = rng.random(shape, dtype=np.float32)
        x *= 2.0
        x -= 1.0
        return x
    if dist == "normal":
        x = rng.standard_normal(shape, dtype=np.float32)
        if sigma != 1.0:
            x *= np.float32(sigma)
        return x
    if dist == "int":
        return rng.integers(-3, 4, size=shape).astype(np.float32)
    raise ValueError(f"unknown distribution {dist}")


def generate(w: Workload):
    """Returns (input_storage, kernel_storage, input_f32, kernel_f32) for a workload."""
    xi = _draw(np.random.default_rng(w.seed_input), w.input_shape, w.input_dist, 1.0)
    xk = _draw(np.random.default_rng(w.seed_kernel), w.kernel_shape, w.kernel_dist,
               w.kernel_sigma)
    i_st, i_32 = to_storage(xi, w.dtype)
    k_st, k_32 = to_storage(xk, w.dtype)
    return i_st, k_st, i_32, k_32


def generate_dout(w: Workload):
    """Output gradient dL/dO for the backward pass of a workload: (storage, f32) in the
    workload's element type, drawn like the input (its own seed)."""
    xg = _draw(np.random.default_rng(w.seed_input + 7000), w.out_shape, w.input_dist, 1.0)
    return to_storage(xg, w.dtype)


def integer_variant(w: Workload) -> Workload:
    """Same shape, small-integer values: every partial sum is exact in fp32, so any correct
    implementation must reproduce the exact result bit for bit in any summation order."""
    return replace(w, name=w.name + "[int]", input_dist="int", kernel_dist="int",
                   seed_input=w.seed_input + 500, seed_kernel=w.seed_kernel + 500)


def sample_capsules(w: Workload, count: int, seed: int, border_share: float = 0.25):
    """`count` output capsules (n, x, y, m) drawn with a fixed seed: a share of them on the
    image border (where padding taps fall), the rest uniform.  int32 array [count, 4]."""
    rng = np.random.default_rng(seed)
    Ho, Wo = w.Ho, w.Wo
    n = rng.integers(0, w.N, size=count)
    x = rng.integers(0, Ho, size=count)
    y = rng.integers(0, Wo, size=count)
    m = rng.integers(0, w.M, size=count)
    nb = int(count * border_share)
    side = rng.integers(0, 4, size=nb)
    x[:nb] = np.where(side == 0, 0, np.where(side == 1, Ho - 1, x[:nb]))
    y[:nb] = np.where(side == 2, 0, np.where(side == 3, Wo - 1, y[:nb]))
    return np.stack([n, x, y, m], axis=1).astype(np.int32)
