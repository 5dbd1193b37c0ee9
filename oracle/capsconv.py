"""ctypes front end of the C oracle (``capsconv_oracle.c``).  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file (paper Sec. 1.2, Algorithm 2, Fig. 2); this module only
builds it with gcc, checks shapes and marshals numpy arrays.  It shares no code with the GPU
library and never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "capsconv_oracle.c"
# CAPSCAPS_SANITIZE=1: a second build with AddressSanitizer and UndefinedBehaviorSanitizer (clang,
# shared runtime), for running the CPU tests under the sanitizers; the process must then preload
# clang's libclang_rt.asan-x86_64.so.
_SANITIZE = os.environ.get("CAPSCAPS_SANITIZE") == "1"
_LIB = _HERE / ("libcapsconv_oracle.san.so" if _SANITIZE else "libcapsconv_oracle.so")
_CLANG = os.environ.get("CAPSCAPS_CLANG", "/opt/rocm/lib/llvm/bin/clang")
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, OpenMP).  Rebuilds if the source is newer."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-o", str(tmp), str(_SRC)]
        if _SANITIZE:
            cmd = [_CLANG, "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall",
                   "-Wextra", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                   "-fno-omit-frame-pointer", "-shared-libsan", "-o", str(tmp), str(_SRC)]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        i, ll, p = ctypes.c_int, ctypes.c_longlong, ctypes.c_void_p
        lib.capsconv_oracle_out_shape.argtypes = [i] * 6 + [ctypes.POINTER(i)] * 2
        lib.capsconv_oracle_out_shape.restype = i
        lib.capsconv_oracle_fwd.argtypes = [p, p, p, p] + [i] * 13
        lib.capsconv_oracle_fwd.restype = i
        lib.capsconv_oracle_fwd_subset.argtypes = [p, p, p, p] + [i] * 13 + [p, ll]
        lib.capsconv_oracle_fwd_subset.restype = i
        lib.capsconv_oracle_bwd_input.argtypes = [p, p, p] + [i] * 13
        lib.capsconv_oracle_bwd_input.restype = i
        lib.capsconv_oracle_bwd_kernel.argtypes = [p, p, p] + [i] * 13
        lib.capsconv_oracle_bwd_kernel.restype = i
        lib.capsconv_oracle_threads.argtypes = []
        lib.capsconv_oracle_threads.restype = i
        _lib = lib
    return _lib


def threads() -> int:
    """Number of host threads the oracle's loops use."""
    return int(_load().capsconv_oracle_threads())


def out_shape(H, W, kh, kw, stride, pad):
    ho, wo = ctypes.c_int(), ctypes.c_int()
    rc = _load().capsconv_oracle_out_shape(H, W, kh, kw, stride, pad, ctypes.byref(ho),
                                           ctypes.byref(wo))
    if rc:
        raise ValueError("invalid geometry")
    return ho.value, wo.value


def _as_f32(a, ndim, name):
    a = np.asarray(a)
    if a.ndim != ndim:
        raise ValueError(f"{name} must have {ndim} dimensions, got {a.ndim}")
    b = np.ascontiguousarray(a, dtype=np.float32)
    if a.dtype != np.float32 and not np.array_equal(b.astype(np.float64), a.astype(np.float64)):
        raise ValueError(f"{name} holds values that are not exactly representable in float32")
    return b


def _dims(I, K, stride, pad):
    N, H, W, C, D0, D1, D2 = I.shape
    kh, kw, Ck, M, D0k, D2k, D3 = K.shape
    if (Ck, D0k, D2k) != (C, D0, D2):
        raise ValueError(f"kernel {K.shape} does not match input {I.shape}")
    Ho, Wo = out_shape(H, W, kh, kw, stride, pad)
    return (N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3), (Ho, Wo)


def conv_fwd(I, K, stride=1, pad=0, with_abs_sum=False):
    """Full output.  I: [N,H,W,C,D0,D1,D2], K: [kh,kw,C,M,D0,D2,D3] -> float64
    O: [N,H',W',M,D0,D1,D3] (and S, the sum of |products|, if requested)."""
    I = _as_f32(I, 7, "I")
    K = _as_f32(K, 7, "K")
    dims, (Ho, Wo) = _dims(I, K, stride, pad)
    N, _, _, _, M, _, _, _, _, D0, D1, _, D3 = dims
    O = np.empty((N, Ho, Wo, M, D0, D1, D3), dtype=np.float64)
    S = np.empty_like(O) if with_abs_sum else None
    rc = _load().capsconv_oracle_fwd(I.ctypes.data, K.ctypes.data, O.ctypes.data,
                                     S.ctypes.data if with_abs_sum else None, *dims)
    if rc:
        raise ValueError(f"oracle rejected the dimensions (rc={rc})")
    return (O, S) if with_abs_sum else O


def conv_fwd_subset(I, K, which, stride=1, pad=0, with_abs_sum=False):
    """Listed output capsules only.  which: int array [count, 4] of (n, x, y, m).
    Returns float64 [count, D0, D1, D3] (and S)."""
    I = _as_f32(I, 7, "I")
    K = _as_f32(K, 7, "K")
    dims, _ = _dims(I, K, stride, pad)
    D0, D1, D3 = dims[9], dims[10], dims[12]
    which = np.ascontiguousarray(which, dtype=np.int32).reshape(-1, 4)
    O = np.empty((which.shape[0], D0, D1, D3), dtype=np.float64)
    S = np.empty_like(O) if with_abs_sum else None
    rc = _load().capsconv_oracle_fwd_subset(I.ctypes.data, K.ctypes.data, O.ctypes.data,
                                            S.ctypes.data if with_abs_sum else None, *dims,
                                            which.ctypes.data, which.shape[0])
    if rc:
        raise ValueError(f"oracle rejected the request (rc={rc})")
    return (O, S) if with_abs_sum else O


def conv_bwd_input(G, K, input_hw, stride=1, pad=0):
    """dL/dI from G = dL/dO [N,H',W',M,D0,D1,D3] and K [kh,kw,C,M,D0,D2,D3]; input_hw = (H, W).
    Returns float64 [N,H,W,C,D0,D1,D2]."""
    G = _as_f32(G, 7, "G")
    K = _as_f32(K, 7, "K")
    H, W = input_hw
    N, Ho, Wo, M, D0, D1, D3 = G.shape
    kh, kw, C, Mk, D0k, D2, D3k = K.shape
    if (Mk, D0k, D3k) != (M, D0, D3) or out_shape(H, W, kh, kw, stride, pad) != (Ho, Wo):
        raise ValueError(f"G {G.shape}, K {K.shape} and input {H}x{W} do not fit together")
    dI = np.empty((N, H, W, C, D0, D1, D2), dtype=np.float64)
    rc = _load().capsconv_oracle_bwd_input(G.ctypes.data, K.ctypes.data, dI.ctypes.data, N, H, W, C,
                                           M, kh, kw, stride, pad, D0, D1, D2, D3)
    if rc:
        raise ValueError(f"oracle rejected the dimensions (rc={rc})")
    return dI


def conv_bwd_kernel(I, G, kernel_hw, stride=1, pad=0):
    """dL/dK from I [N,H,W,C,D0,D1,D2] and G = dL/dO [N,H',W',M,D0,D1,D3]; kernel_hw = (kh, kw).
    Returns float64 [kh,kw,C,M,D0,D2,D3]."""
    I = _as_f32(I, 7, "I")
    G = _as_f32(G, 7, "G")
    kh, kw = kernel_hw
    N, H, W, C, D0, D1, D2 = I.shape
    Ng, Ho, Wo, M, D0g, D1g, D3 = G.shape
    if (Ng, D0g, D1g) != (N, D0, D1) or out_shape(H, W, kh, kw, stride, pad) != (Ho, Wo):
        raise ValueError(f"I {I.shape}, G {G.shape} and window {kh}x{kw} do not fit together")
    dK = np.empty((kh, kw, C, M, D0, D2, D3), dtype=np.float64)
    rc = _load().capsconv_oracle_bwd_kernel(I.ctypes.data, G.ctypes.data, dK.ctypes.data, N, H, W,
                                            C, M, kh, kw, stride, pad, D0, D1, D2, D3)
    if rc:
        raise ValueError(f"oracle rejected the dimensions (rc={rc})")
    return dK
