"""Helpers shared by the GPU parity tests: upload seeded inputs, call the C ABI through the
binding, bring results back, and the error measures the tolerances are stated in."""
import numpy as np

from paper_2104_02621_amd import capscaps as cc
from paper_2104_02621_amd import workloads as wl

# Tolerances.  The target is max|g-r| / max|r| <= 1e-5 for fp32 and <= 2e-2 for 16-bit inputs
# with fp32 accumulation.  16-bit products are exact in fp32, so for every dtype the only
# error source is the order of fp32 additions; against the scale S = sum|I*K| of each output
# that error is bounded by about (number of terms) * 2^-24 in the worst case and is of order
# sqrt(terms) * 2^-24 for random data, so a second, much sharper check err/S <= 1e-5 is made
# for all dtypes (terms <= 9216 in every test here: worst-case bound 5.5e-4, typical 6e-6).
TOL_PRIMARY = {wl.FP32: 1e-5, wl.BF16: 2e-2, wl.FP16: 2e-2}
TOL_VS_ABS_SUM = 1e-5


def to_device(storage: np.ndarray, dtype: int):
    import torch
    if dtype == wl.BF16:
        return torch.from_numpy(storage.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(storage).cuda()


def shape_args(w: wl.Workload):
    return (w.N, w.H, w.W, w.C, w.M, w.kh, w.kw, w.stride, w.pad, w.D0, w.D1, w.D2, w.D3, w.dtype)


def run_gpu(w: wl.Workload, i_dev, k_dev, path=cc.PATH_AUTO, out=None, workspace=None):
    """One call through capscaps_conv_fwd_path on torch's current stream -> device tensor."""
    import torch
    if out is None:
        # poison the output so that an element the kernel fails to write cannot pass
        out = torch.full(w.out_shape, float("nan"), dtype=torch.float32, device="cuda")
    need = cc.capscaps_conv_fwd_workspace_bytes(*shape_args(w))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    rc = cc.capscaps_conv_fwd_path(i_dev.data_ptr(), k_dev.data_ptr(), out.data_ptr(), w.N, w.H,
                                   w.W, w.C, w.M, w.kh, w.kw, w.stride, w.pad, w.D0, w.D1, w.D2,
                                   w.D3, w.dtype, path, workspace.data_ptr(), workspace.numel(),
                                   torch.cuda.current_stream().cuda_stream)
    assert rc == cc.OK, f"{w.name}: status {rc} ({cc.capscaps_strerror(rc)}; {cc.capscaps_last_hip_error()})"
    return out


def errors(got: np.ndarray, ref: np.ndarray, abs_sum: np.ndarray):
    """(max|g-r| / max|r|,  max(|g-r| / S))."""
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite values (or unwritten outputs) in the GPU result"
    diff = np.abs(got.astype(np.float64) - ref)
    primary = diff.max() / max(np.abs(ref).max(), 1e-300)
    secondary = (diff / np.maximum(abs_sum, 1e-300)).max()
    return float(primary), float(secondary)


def check(w: wl.Workload, got, ref, abs_sum, label=""):
    primary, secondary = errors(got, ref, abs_sum)
    msg = f"{w.name} {label}: rel-to-max {primary:.3e}, rel-to-abs-sum {secondary:.3e}"
    print(msg, flush=True)
    assert primary <= TOL_PRIMARY[w.dtype], msg
    assert secondary <= TOL_VS_ABS_SUM, msg
    return primary, secondary
