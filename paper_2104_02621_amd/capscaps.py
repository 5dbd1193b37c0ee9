"""ctypes binding of ``libcapscaps.so`` (C ABI in ``include/capscaps.h``).

Argument marshalling only: every step of the capsule convolution runs in the HIP library.
Functions carry the C names; ``conv_fwd`` is a convenience wrapper that takes torch tensors
(torch is used for device memory and streams only).  There is no CPU fallback: if the
library is missing or no GPU is present, calls fail.
"""
from __future__ import annotations

import ctypes
import os
from pathlib import Path

FP32, BF16, FP16 = 0, 1, 2
PATH_AUTO, PATH_DIRECT, PATH_MFMA, PATH_MFMA_GENERIC, PATH_MFMA_TUNED16 = 0, 1, 2, 3, 4
PATH_MFMA_TUNED32 = 5
PATH_MFMA_SMALL = 6
OK, EINVAL, EWORKSPACE, EUNSUPPORTED, EHIP, ESCRATCH = 0, -1, -2, -3, -4, -5
STATIC_SCRATCH_BYTES = 80 << 20

# CAPSCAPS_SANITIZE=1 selects the build whose host code is instrumented (see build.py)
_LIB_PATH = Path(__file__).resolve().parent / (
    "libcapscaps.san.so" if os.environ.get("CAPSCAPS_SANITIZE") == "1" else "libcapscaps.so")
_lib = None


class CapscapsError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        detail = f" ({capscaps_last_hip_error()})" if status == EHIP else ""
        super().__init__(f"capscaps status {status}: {capscaps_strerror(status)}{detail}")


def library_path() -> Path:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not _LIB_PATH.exists():
        raise FileNotFoundError(
            f"{_LIB_PATH} is not built; run `python -m paper_2104_02621_amd.build`")
    # One HIP runtime per process: PyTorch ships its own libamdhip64 under the same soname as
    # ROCm's.  Importing torch first makes the dynamic loader resolve this library's dependency
    # to the copy torch already mapped, so streams and device pointers are shared.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(str(_LIB_PATH))
    i, p, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    ip = ctypes.POINTER(ctypes.c_int)
    lib.capscaps_out_shape.argtypes = [i] * 6 + [ip, ip]
    lib.capscaps_out_shape.restype = i
    lib.capscaps_conv_fwd.argtypes = [p, p, p] + [i] * 13 + [p]
    lib.capscaps_conv_fwd.restype = i
    lib.capscaps_conv_fwd_ex.argtypes = [p, p, p] + [i] * 14 + [p, sz, p]
    lib.capscaps_conv_fwd_ex.restype = i
    lib.capscaps_conv_fwd_static.argtypes = [p, p, p] + [i] * 14 + [p]
    lib.capscaps_conv_fwd_static.restype = i
    lib.capscaps_conv_fwd_out16_workspace_bytes.argtypes = [i] * 14
    lib.capscaps_conv_fwd_out16_workspace_bytes.restype = sz
    lib.capscaps_conv_fwd_out16.argtypes = [p, p, p] + [i] * 14 + [p, sz, p]
    lib.capscaps_conv_fwd_out16.restype = i
    lib.capscaps_conv_fwd_path.argtypes = [p, p, p] + [i] * 15 + [p, sz, p]
    lib.capscaps_conv_fwd_path.restype = i
    lib.capscaps_conv_fwd_workspace_bytes.argtypes = [i] * 14
    lib.capscaps_conv_fwd_workspace_bytes.restype = sz
    lib.capscaps_select_path.argtypes = [i] * 14
    lib.capscaps_select_path.restype = i
    for name in ("capscaps_conv_bwd_input", "capscaps_conv_bwd_kernel"):
        getattr(lib, name).argtypes = [p, p, p] + [i] * 14 + [p, sz, p]
        getattr(lib, name).restype = i
        getattr(lib, name + "_workspace_bytes").argtypes = [i] * 14
        getattr(lib, name + "_workspace_bytes").restype = sz
    lib.capscaps_conv_bwd_input_out16.argtypes = [p, p, p] + [i] * 14 + [p, sz, p]
    lib.capscaps_conv_bwd_input_out16.restype = i
    lib.capscaps_conv_bwd_input_out16_workspace_bytes.argtypes = [i] * 14
    lib.capscaps_conv_bwd_input_out16_workspace_bytes.restype = sz
    lib.capscaps_scheme2_index_bytes.argtypes = [i] * 14
    lib.capscaps_scheme2_index_bytes.restype = sz
    lib.capscaps_scheme2_build_index.argtypes = [p, sz] + [i] * 14 + [p]
    lib.capscaps_scheme2_build_index.restype = i
    lib.capscaps_scheme2_fwd.argtypes = [p, p, p, p, sz] + [i] * 14 + [p]
    lib.capscaps_scheme2_fwd.restype = i
    lib.capscaps_mfma_yardstick.argtypes = [p, p, i, i, i, p]
    lib.capscaps_mfma_yardstick.restype = i
    lib.capscaps_mfma_yardstick_flops.argtypes = [i, i, i]
    lib.capscaps_mfma_yardstick_flops.restype = ctypes.c_double
    lib.capscaps_strerror.argtypes = [i]
    lib.capscaps_strerror.restype = ctypes.c_char_p
    lib.capscaps_last_hip_error.argtypes = []
    lib.capscaps_last_hip_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


# ------------------------------------------------------------------ C ABI, same names
def capscaps_strerror(status: int) -> str:
    return _load().capscaps_strerror(int(status)).decode()


def capscaps_last_hip_error() -> str:
    return _load().capscaps_last_hip_error().decode()


def capscaps_out_shape(H, W, kh, kw, stride, pad):
    """Returns (status, Ho, Wo)."""
    ho, wo = ctypes.c_int(0), ctypes.c_int(0)
    rc = _load().capscaps_out_shape(H, W, kh, kw, stride, pad, ctypes.byref(ho), ctypes.byref(wo))
    return rc, ho.value, wo.value


def capscaps_conv_fwd(input, kernel, out, N, H, W, C, M, kh, kw, stride, D0, D1, D2, D3, dtype,
                      stream=None) -> int:
    """Device pointers as ints; returns the status code."""
    return _load().capscaps_conv_fwd(input, kernel, out, N, H, W, C, M, kh, kw, stride, D0, D1,
                                     D2, D3, dtype, stream)


def capscaps_conv_fwd_ex(input, kernel, out, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3,
                         dtype, workspace, workspace_bytes, stream=None) -> int:
    return _load().capscaps_conv_fwd_ex(input, kernel, out, N, H, W, C, M, kh, kw, stride, pad,
                                        D0, D1, D2, D3, dtype, workspace, workspace_bytes, stream)


def capscaps_conv_fwd_static(input, kernel, out, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3,
                             dtype, stream=None) -> int:
    return _load().capscaps_conv_fwd_static(input, kernel, out, N, H, W, C, M, kh, kw, stride, pad,
                                            D0, D1, D2, D3, dtype, stream)


def capscaps_conv_fwd_out16_workspace_bytes(N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3,
                                            dtype) -> int:
    return int(_load().capscaps_conv_fwd_out16_workspace_bytes(N, H, W, C, M, kh, kw, stride, pad,
                                                               D0, D1, D2, D3, dtype))


def capscaps_conv_fwd_out16(input, kernel, out, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3,
                            dtype, workspace, workspace_bytes, stream=None) -> int:
    return _load().capscaps_conv_fwd_out16(input, kernel, out, N, H, W, C, M, kh, kw, stride, pad,
                                           D0, D1, D2, D3, dtype, workspace, workspace_bytes,
                                           stream)


def capscaps_conv_fwd_path(input, kernel, out, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2,
                           D3, dtype, path, workspace, workspace_bytes, stream=None) -> int:
    return _load().capscaps_conv_fwd_path(input, kernel, out, N, H, W, C, M, kh, kw, stride, pad,
                                          D0, D1, D2, D3, dtype, path, workspace,
                                          workspace_bytes, stream)


def capscaps_conv_fwd_workspace_bytes(N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3,
                                      dtype) -> int:
    return int(_load().capscaps_conv_fwd_workspace_bytes(N, H, W, C, M, kh, kw, stride, pad, D0,
                                                         D1, D2, D3, dtype))


def capscaps_select_path(N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype) -> int:
    return int(_load().capscaps_select_path(N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3,
                                            dtype))


def capscaps_conv_bwd_input(dout, kernel, dinput, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2,
                            D3, dtype, workspace, workspace_bytes, stream=None) -> int:
    return _load().capscaps_conv_bwd_input(dout, kernel, dinput, N, H, W, C, M, kh, kw, stride,
                                           pad, D0, D1, D2, D3, dtype, workspace, workspace_bytes,
                                           stream)


def capscaps_conv_bwd_input_out16(dout, kernel, dinput, N, H, W, C, M, kh, kw, stride, pad, D0, D1,
                                  D2, D3, dtype, workspace, workspace_bytes, stream=None) -> int:
    return _load().capscaps_conv_bwd_input_out16(dout, kernel, dinput, N, H, W, C, M, kh, kw,
                                                 stride, pad, D0, D1, D2, D3, dtype, workspace,
                                                 workspace_bytes, stream)


def capscaps_conv_bwd_input_out16_workspace_bytes(N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2,
                                                  D3, dtype) -> int:
    return int(_load().capscaps_conv_bwd_input_out16_workspace_bytes(N, H, W, C, M, kh, kw, stride,
                                                                     pad, D0, D1, D2, D3, dtype))


def capscaps_conv_bwd_kernel(input, dout, dkernel, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2,
                             D3, dtype, workspace, workspace_bytes, stream=None) -> int:
    return _load().capscaps_conv_bwd_kernel(input, dout, dkernel, N, H, W, C, M, kh, kw, stride,
                                            pad, D0, D1, D2, D3, dtype, workspace,
                                            workspace_bytes, stream)


def capscaps_conv_bwd_input_workspace_bytes(N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3,
                                            dtype) -> int:
    return int(_load().capscaps_conv_bwd_input_workspace_bytes(N, H, W, C, M, kh, kw, stride, pad,
                                                               D0, D1, D2, D3, dtype))


def capscaps_conv_bwd_kernel_workspace_bytes(N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3,
                                             dtype) -> int:
    return int(_load().capscaps_conv_bwd_kernel_workspace_bytes(N, H, W, C, M, kh, kw, stride,
                                                                pad, D0, D1, D2, D3, dtype))


def capscaps_scheme2_index_bytes(N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype) -> int:
    return int(_load().capscaps_scheme2_index_bytes(N, H, W, C, M, kh, kw, stride, pad, D0, D1,
                                                    D2, D3, dtype))


def capscaps_scheme2_build_index(index, index_bytes, N, H, W, C, M, kh, kw, stride, pad, D0, D1,
                                 D2, D3, dtype, stream=None) -> int:
    return _load().capscaps_scheme2_build_index(index, index_bytes, N, H, W, C, M, kh, kw, stride,
                                                pad, D0, D1, D2, D3, dtype, stream)


def capscaps_scheme2_fwd(input, kernel, out, index, index_bytes, N, H, W, C, M, kh, kw, stride,
                         pad, D0, D1, D2, D3, dtype, stream=None) -> int:
    return _load().capscaps_scheme2_fwd(input, kernel, out, index, index_bytes, N, H, W, C, M, kh,
                                        kw, stride, pad, D0, D1, D2, D3, dtype, stream)


def capscaps_mfma_yardstick(seed, sink, dtype, blocks, iters, stream=None) -> int:
    return _load().capscaps_mfma_yardstick(seed, sink, dtype, blocks, iters, stream)


def capscaps_mfma_yardstick_flops(dtype, blocks, iters) -> float:
    return float(_load().capscaps_mfma_yardstick_flops(dtype, blocks, iters))


# ------------------------------------------------------------------ torch convenience
def _torch_dtype_code(t):
    import torch
    return {torch.float32: FP32, torch.bfloat16: BF16, torch.float16: FP16}[t.dtype]


def conv_fwd(input, kernel, stride=1, pad=0, path=PATH_AUTO, out=None, workspace=None,
             out16=False):
    """input [N,H,W,C,D0,D1,D2], kernel [kh,kw,C,M,D0,D2,D3] (contiguous device tensors of one
    dtype: float32, bfloat16 or float16) -> float32 [N,H',W',M,D0,D1,D3] (with `out16`: of the
    operands' 16-bit type, library's own path choice).  Enqueues on torch's current stream; does
    not synchronise."""
    import torch
    if not (input.is_cuda and kernel.is_cuda):
        raise ValueError("capscaps runs on the GPU only: pass device tensors")
    if input.dtype != kernel.dtype or input.dim() != 7 or kernel.dim() != 7:
        raise ValueError("input and kernel must be 7-D tensors of one dtype")
    if not (input.is_contiguous() and kernel.is_contiguous()):
        raise ValueError("input and kernel must be contiguous")
    N, H, W, C, D0, D1, D2 = input.shape
    kh, kw, Ck, M, D0k, D2k, D3 = kernel.shape
    if (Ck, D0k, D2k) != (C, D0, D2):
        raise ValueError(f"kernel {tuple(kernel.shape)} does not match input {tuple(input.shape)}")
    dt = _torch_dtype_code(input)
    rc, Ho, Wo = capscaps_out_shape(H, W, kh, kw, stride, pad)
    if rc != OK:
        raise CapscapsError(rc)
    if out is None:
        out = torch.empty((N, Ho, Wo, M, D0, D1, D3),
                          dtype=input.dtype if out16 else torch.float32, device=input.device)
    need = (capscaps_conv_fwd_out16_workspace_bytes if out16 else
            capscaps_conv_fwd_workspace_bytes)(N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dt)
    if workspace is None or workspace.numel() * workspace.element_size() < need:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=input.device)
    stream = torch.cuda.current_stream(input.device).cuda_stream
    if out16:
        rc = capscaps_conv_fwd_out16(input.data_ptr(), kernel.data_ptr(), out.data_ptr(), N, H, W,
                                     C, M, kh, kw, stride, pad, D0, D1, D2, D3, dt,
                                     workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), stream)
    else:
        rc = capscaps_conv_fwd_path(input.data_ptr(), kernel.data_ptr(), out.data_ptr(), N, H, W,
                                    C, M, kh, kw, stride, pad, D0, D1, D2, D3, dt, path,
                                    workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), stream)
    if rc != OK:
        raise CapscapsError(rc)
    return out


def _bwd_common(a, b):
    if not (a.is_cuda and b.is_cuda):
        raise ValueError("capscaps runs on the GPU only: pass device tensors")
    if a.dtype != b.dtype or a.dim() != 7 or b.dim() != 7:
        raise ValueError("operands must be 7-D tensors of one dtype")
    if not (a.is_contiguous() and b.is_contiguous()):
        raise ValueError("operands must be contiguous")


def conv_bwd_input(dout, kernel, input_hw, stride=1, pad=0, out16=False):
    """dout [N,H',W',M,D0,D1,D3], kernel [kh,kw,C,M,D0,D2,D3] (one dtype), input_hw = (H, W) of
    the forward input -> float32 dinput [N,H,W,C,D0,D1,D2] (with `out16`: of the operands' 16-bit
    type)."""
    import torch
    _bwd_common(dout, kernel)
    N, Ho, Wo, M, D0, D1, D3 = dout.shape
    kh, kw, C, Mk, D0k, D2, D3k = kernel.shape
    H, W = input_hw
    rc, ho, wo = capscaps_out_shape(H, W, kh, kw, stride, pad)
    if rc != OK:
        raise CapscapsError(rc)
    if (Mk, D0k, D3k, ho, wo) != (M, D0, D3, Ho, Wo):
        raise ValueError("dout, kernel and input_hw do not describe one convolution")
    dt = _torch_dtype_code(dout)
    shape = (N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dt)
    need = (capscaps_conv_bwd_input_out16_workspace_bytes if out16 else
            capscaps_conv_bwd_input_workspace_bytes)(*shape)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dout.device)
    din = torch.empty((N, H, W, C, D0, D1, D2), dtype=dout.dtype if out16 else torch.float32,
                      device=dout.device)
    call = capscaps_conv_bwd_input_out16 if out16 else capscaps_conv_bwd_input
    rc = call(dout.data_ptr(), kernel.data_ptr(), din.data_ptr(), *shape, ws.data_ptr(), ws.numel(),
              torch.cuda.current_stream(dout.device).cuda_stream)
    if rc != OK:
        raise CapscapsError(rc)
    return din


def conv_bwd_kernel(input, dout, kernel_hw, stride=1, pad=0):
    """input [N,H,W,C,D0,D1,D2], dout [N,H',W',M,D0,D1,D3] (one dtype), kernel_hw = (kh, kw)
    -> float32 dkernel [kh,kw,C,M,D0,D2,D3]."""
    import torch
    _bwd_common(input, dout)
    N, H, W, C, D0, D1, D2 = input.shape
    Ng, Ho, Wo, M, D0g, D1g, D3 = dout.shape
    kh, kw = kernel_hw
    rc, ho, wo = capscaps_out_shape(H, W, kh, kw, stride, pad)
    if rc != OK:
        raise CapscapsError(rc)
    if (Ng, D0g, D1g, ho, wo) != (N, D0, D1, Ho, Wo):
        raise ValueError("input, dout and kernel_hw do not describe one convolution")
    dt = _torch_dtype_code(input)
    shape = (N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dt)
    need = capscaps_conv_bwd_kernel_workspace_bytes(*shape)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=input.device)
    dk = torch.empty((kh, kw, C, M, D0, D2, D3), dtype=torch.float32, device=input.device)
    rc = capscaps_conv_bwd_kernel(input.data_ptr(), dout.data_ptr(), dk.data_ptr(), *shape,
                                  ws.data_ptr(), ws.numel(),
                                  torch.cuda.current_stream(input.device).cuda_stream)
    if rc != OK:
        raise CapscapsError(rc)
    return dk
