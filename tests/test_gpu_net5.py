"""GPU parity of the chained five-layer stack: layers 1-4 through the 16-bit-output entry point
(each layer's output is the next one's input, no conversion pass), layer 5 to fp32, against the
oracle applied layer by layer with the same rounding of the activations to the 16-bit type."""
import numpy as np
import pytest

from oracle import capsconv
from paper_2104_02621_amd import capscaps as cc
from paper_2104_02621_amd import workloads as wl
from tests.gpu_util import to_device

pytestmark = pytest.mark.gpu


def oracle_stack(layers, x32):
    for k, w in enumerate(layers):
        _, _, _, k32 = wl.generate(w)
        y = capsconv.conv_fwd(x32, k32, w.stride, w.pad)
        if k + 1 < len(layers):  # the activation as the next layer reads it
            _, x32 = wl.to_storage(y.astype(np.float32), w.dtype)
    return y


def gpu_stack(layers, x_dev):
    x = x_dev
    for k, w in enumerate(layers):
        k_st = wl.generate(w)[1]
        x = cc.conv_fwd(x, to_device(k_st, w.dtype), w.stride, w.pad, out16=k + 1 < len(layers))
    return x


@pytest.mark.parametrize("dtype", [wl.BF16, wl.FP16], ids=["bf16", "fp16"])
def test_five_layer_stack_matches_oracle(dtype):
    layers = wl.net5(N=2, dtype=dtype)
    i_st, _, i32, _ = wl.generate(layers[0])
    for a, b in zip(layers, layers[1:]):  # shapes chain
        assert a.out_shape[:4] == (b.N, b.H, b.W, b.C) and (a.D1, a.D3) == (b.D1, b.D2)
    ref = oracle_stack(layers, i32)
    got = gpu_stack(layers, to_device(i_st, dtype)).cpu().numpy()
    assert got.shape == ref.shape == (2, 1, 1, 10, 1, 8, 8)
    err = np.abs(got - ref).max() / np.abs(ref).max()
    print(f"net5 {wl.DTYPE_NAMES[dtype]}: max|g-r|/max|r| = {err:.3e}", flush=True)
    # each layer's activations are rounded to the 16-bit type on both sides, but from sums taken
    # in different precision (fp32 vs fp64), so a few activations land on neighbouring 16-bit
    # values; what that leaves after four more layers is far below the 16-bit tolerance
    assert err <= 2e-2
