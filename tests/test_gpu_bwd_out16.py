"""GPU parity of the input gradient with 16-bit output (capscaps_conv_bwd_input_out16): the fp32
sum rounded to nearest even once, at the store.  Two checks, as for the forward pass's 16-bit
output: against the same library's fp32 gradient rounded on the host (bit for bit: same kernels,
same summation order, one rounding), and against the CPU oracle within half a 16-bit unit plus
the fp32 summation error.  Needs an MI355X."""
import dataclasses

import numpy as np
import pytest

from oracle import capsconv
from paper_2104_02621_amd import capscaps as cc
from paper_2104_02621_amd import workloads as wl
from tests.gpu_util import shape_args, to_device
from tests.test_gpu_bwd_parity import BWD_SHAPES, run_bwd_input
from tests.test_gpu_out16 import ULP16, bits_to_f64, round_on_host, to_bits
from tests.test_gpu_parity import small

pytestmark = pytest.mark.gpu


def run_bwd_input_out16(w, g_dev, k_dev):
    import torch
    tdt = torch.bfloat16 if w.dtype == wl.BF16 else torch.float16
    din = torch.full(w.input_shape, float("nan"), dtype=tdt, device="cuda")
    need = cc.capscaps_conv_bwd_input_out16_workspace_bytes(*shape_args(w))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    rc = cc.capscaps_conv_bwd_input_out16(g_dev.data_ptr(), k_dev.data_ptr(), din.data_ptr(),
                                          *shape_args(w), ws.data_ptr(), ws.numel(),
                                          torch.cuda.current_stream().cuda_stream)
    assert rc == cc.OK, f"{w.name}: status {rc} ({cc.capscaps_strerror(rc)}; {cc.capscaps_last_hip_error()})"
    return din


def within_bound(w, got, ref, S):
    """Half a unit of the 16-bit type, the fp32 summation error, and the absolute spacing of the
    type's smallest numbers."""
    bound = 0.5 * ULP16[w.dtype] * np.abs(ref) * 1.0001 + 1e-5 * S + 1e-7
    worst = (np.abs(got - ref) / bound).max()
    print(f"{w.name}: max error / bound = {worst:.3f}", flush=True)
    assert worst <= 1.0, w.name


@pytest.mark.parametrize("dtype", [wl.BF16, wl.FP16], ids=["bf16", "fp16"])
@pytest.mark.parametrize("shape", BWD_SHAPES, ids=[s[0] for s in BWD_SHAPES])
def test_small_shapes(shape, dtype):
    w = small(shape[0], dtype, *shape[1:], seed=len(shape[0]) + 50)
    i_st, k_st, i32, k32 = wl.generate(w)
    g_st, g32 = wl.generate_dout(w)
    dI = capsconv.conv_bwd_input(g32, k32, (w.H, w.W), w.stride, w.pad)
    SI = capsconv.conv_bwd_input(np.abs(g32), np.abs(k32), (w.H, w.W), w.stride, w.pad)
    k_dev, g_dev = to_device(k_st, w.dtype), to_device(g_st, w.dtype)
    got_bits = to_bits(run_bwd_input_out16(w, g_dev, k_dev))
    din32 = run_bwd_input(w, g_dev, k_dev).cpu().numpy()
    assert np.array_equal(got_bits, round_on_host(din32, w.dtype)), w.name
    got = bits_to_f64(got_bits, w.dtype)
    assert (got[SI == 0] == 0).all()  # pixels no window reaches
    within_bound(w, got, dI, SI)


@pytest.mark.parametrize("number", [3, 5])
def test_benchmark_configs_full_size_sampled(number):
    """Full size.  dI[n,:,:,c] depends only on image n of the gradient and channel c of the
    kernel, so the oracle computes sampled slices from sliced operands."""
    w = wl.config(number)
    i_st, k_st, i32, k32 = wl.generate(w)
    g_st, g32 = wl.generate_dout(w)
    k_dev, g_dev = to_device(k_st, w.dtype), to_device(g_st, w.dtype)
    got16 = run_bwd_input_out16(w, g_dev, k_dev)
    din32 = run_bwd_input(w, g_dev, k_dev)
    import torch
    assert bool(got16.isfinite().all())
    # one rounding of the very same fp32 result (torch rounds to nearest even as well); where
    # the fp32 call adds up its last tiles' K loop in pieces, a few values near a rounding tie
    # may land on the neighbouring 16-bit number
    assert float((got16 != din32.to(got16.dtype)).float().mean()) < 1e-3
    rng = np.random.default_rng(950 + number)
    hw = (w.H, w.W)
    for _ in range(3):
        n, c = int(rng.integers(w.N)), int(rng.integers(w.C))
        gs, ks = g32[n:n + 1], np.ascontiguousarray(k32[:, :, c:c + 1])
        ref = capsconv.conv_bwd_input(gs, ks, hw, w.stride, w.pad)
        S = capsconv.conv_bwd_input(np.abs(gs), np.abs(ks), hw, w.stride, w.pad)
        sub = dataclasses.replace(w, name=f"{w.name} dI[{n},:,:,{c}]")
        got = bits_to_f64(to_bits(got16[n:n + 1, :, :, c:c + 1].contiguous()), w.dtype)
        within_bound(sub, got, ref, S)


def test_fp32_operands_and_small_workspaces_are_refused():
    import torch
    w = small("f32", wl.FP32, 1, 6, 6, 4, 4, 3, 3, 1, 1, 1, 4, 4, 4)
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    assert cc.capscaps_conv_bwd_input_out16_workspace_bytes(*shape_args(w)) == 0
    assert cc.capscaps_conv_bwd_input_out16(p, p, p, *shape_args(w), p, buf.numel(), None) == cc.EINVAL
    h = small("s1", wl.FP16, 2, 6, 6, 4, 4, 3, 3, 1, 1, 1, 8, 8, 8)
    need = cc.capscaps_conv_bwd_input_out16_workspace_bytes(*shape_args(h))
    assert need > 0
    assert cc.capscaps_conv_bwd_input_out16(p, p, p, *shape_args(h), p, need - 1, None) == cc.EWORKSPACE
