"""The entry point that allocates nothing (capscaps_conv_fwd_static, scratch in a fixed device
array) against capscaps_conv_fwd_ex (scratch from the caller), through the C ABI: same kernels,
so the same bits; and both against the oracle.  Two calls in a row, the second with a smaller
input, so that what the first call left in the shared array cannot leak into the second."""
import numpy as np
import pytest

from oracle import capsconv
from paper_2104_02621_amd import capscaps as cc
from paper_2104_02621_amd import workloads as wl
from tests.gpu_util import check, shape_args, to_device

pytestmark = pytest.mark.gpu


def _both(w, with_oracle=True):
    import torch
    i_st, k_st, i32, k32 = wl.generate(w)
    I, K = to_device(i_st, w.dtype), to_device(k_st, w.dtype)
    stream = torch.cuda.current_stream().cuda_stream
    args = shape_args(w)
    need = cc.capscaps_conv_fwd_workspace_bytes(*args)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    ref_out = torch.full(w.out_shape, float("nan"), dtype=torch.float32, device="cuda")
    rc = cc.capscaps_conv_fwd_ex(I.data_ptr(), K.data_ptr(), ref_out.data_ptr(), *args,
                                 ws.data_ptr(), ws.numel(), stream)
    assert rc == cc.OK, cc.capscaps_strerror(rc)
    out = torch.full(w.out_shape, float("nan"), dtype=torch.float32, device="cuda")
    rc = cc.capscaps_conv_fwd_static(I.data_ptr(), K.data_ptr(), out.data_ptr(), *args, stream)
    assert rc == cc.OK, f"{cc.capscaps_strerror(rc)} ({cc.capscaps_last_hip_error()})"
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out), f"{w.name}: differs from capscaps_conv_fwd_ex"
    if not with_oracle:
        return
    if w.flops_nominal() < 2e10:
        ref, S = capsconv.conv_fwd(i32, k32, w.stride, w.pad, with_abs_sum=True)
        check(w, out.cpu().numpy(), ref, S, "static scratch")
    else:   # the oracle on sampled output capsules (a quarter of them on image borders)
        which = wl.sample_capsules(w, 1500, seed=907)
        ref, S = capsconv.conv_fwd_subset(i32, k32, which, w.stride, w.pad, with_abs_sum=True)
        idx = torch.from_numpy(which.astype(np.int64)).cuda()
        got = out[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy()
        check(w, got, ref, S, "static scratch, sampled")


@pytest.mark.parametrize("dtype", [wl.FP32, wl.BF16, wl.FP16], ids=["fp32", "bf16", "fp16"])
def test_static_scratch_two_calls_second_smaller(dtype):
    # a kernel repack plus a split reduction's partial sums in the scratch (few tiles, long K
    # loop), then a smaller problem of the same kind; then shapes of the tuned kernels
    D = 4 if dtype == wl.FP32 else 8
    big = wl.Workload("static_big", dtype, 6, 9, 9, 16, 10, 3, 3, 1, 1, 1, D, D, D, "normal",
                      "normal", 0.1, 901, 902)
    small = wl.Workload("static_small", dtype, 2, 5, 6, 8, 3, 3, 3, 1, 1, 1, D, D, D, "normal",
                        "normal", 0.1, 903, 904)
    _both(big)
    _both(small)
    # one of the benchmark configurations' kind at reduced batch (tuned kernels), then smaller
    k = {wl.FP32: 2, wl.BF16: 3, wl.FP16: 5}[dtype]
    _both(wl.config(k).with_batch(2))
    _both(wl.config(k).with_batch(1))


def test_static_scratch_holds_the_largest_benchmark_scratch():
    # configuration 3 at full size needs the most scratch of the five (repacked kernel plus the
    # partial sums of its last round of tiles, 72 MB); compared with the caller-workspace call only
    _both(wl.config(3), with_oracle=False)
    _both(wl.config(1))


def test_static_scratch_rejects_what_does_not_fit():
    import torch
    # a repacked kernel beyond the fixed array: 3x3 window, C = M = 160, 16x16 capsules, fp16
    w = wl.Workload("static_toobig", wl.FP16, 1, 34, 34, 160, 160, 3, 3, 1, 1, 1, 16, 16, 16,
                    "normal", "normal", 0.1, 905, 906)
    args = shape_args(w)
    assert cc.capscaps_conv_fwd_workspace_bytes(*args) > cc.STATIC_SCRATCH_BYTES
    t = torch.zeros(64, dtype=torch.float32, device="cuda")   # never touched: refused first
    rc = cc.capscaps_conv_fwd_static(t.data_ptr(), t.data_ptr(), t.data_ptr(), *args,
                                     torch.cuda.current_stream().cuda_stream)
    assert rc == cc.ESCRATCH
    assert "scratch" in cc.capscaps_strerror(rc)
