"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, computes output extents, and refuses bad arguments before touching the GPU."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_2104_02621_amd import capscaps as cc
from paper_2104_02621_amd import workloads as wl

ROOT = Path(__file__).resolve().parent.parent


def declared_symbols():
    text = (ROOT / "include" / "capscaps.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(capscaps_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(str(cc.library_path()))
    names = declared_symbols()
    assert "capscaps_conv_fwd" in names and len(names) >= 7
    for name in names:
        assert hasattr(lib, name), name


def test_binding_has_the_same_names():
    for name in declared_symbols():
        assert callable(getattr(cc, name)), name


def test_out_shape_matches_paper_figures_and_configs():
    assert cc.capscaps_out_shape(5, 5, 4, 4, 1, 0) == (cc.OK, 2, 2)       # Fig. 1 and Fig. 2
    for w in wl.CONFIGS:
        assert cc.capscaps_out_shape(w.H, w.W, w.kh, w.kw, w.stride, w.pad) == (cc.OK, w.Ho, w.Wo)
    assert cc.capscaps_out_shape(7, 7, 2, 2, 3, 2)[1:] == (4, 4)


@pytest.mark.parametrize("bad", [
    dict(H=0), dict(W=-1), dict(kh=0), dict(stride=0), dict(pad=-1), dict(kh=6, pad=0, H=5),
    dict(kw=8, pad=1, W=5),
])
def test_out_shape_rejects(bad):
    a = dict(H=5, W=5, kh=3, kw=3, stride=1, pad=0)
    a.update(bad)
    assert cc.capscaps_out_shape(a["H"], a["W"], a["kh"], a["kw"], a["stride"], a["pad"])[0] \
        == cc.EINVAL


def _args(**over):
    a = dict(N=2, H=6, W=6, C=3, M=4, kh=3, kw=3, stride=1, pad=1, D0=1, D1=4, D2=4, D3=4,
             dtype=cc.FP32)
    a.update(over)
    return [a[k] for k in ("N", "H", "W", "C", "M", "kh", "kw", "stride", "pad", "D0", "D1", "D2",
                           "D3", "dtype")]


FAKE = 0x10000  # a 16-byte aligned non-null "pointer"; never dereferenced on these error paths


@pytest.mark.parametrize("over", [dict(N=0), dict(C=-3), dict(M=0), dict(D0=0), dict(D1=0),
                                  dict(D2=-1), dict(D3=0), dict(stride=0), dict(pad=-1),
                                  dict(kh=9), dict(dtype=3), dict(dtype=-1)])
def test_compute_entry_points_reject_bad_shapes(over):
    a = _args(**over)
    assert cc.capscaps_conv_fwd_ex(FAKE, FAKE, FAKE, *a, FAKE, 1 << 30, None) == cc.EINVAL
    assert cc.capscaps_conv_fwd_path(FAKE, FAKE, FAKE, *a, cc.PATH_AUTO, FAKE, 1 << 30, None) \
        == cc.EINVAL
    assert cc.capscaps_select_path(*a) == cc.EINVAL
    assert cc.capscaps_conv_fwd_workspace_bytes(*a) == 0
    if over.get("pad", 0) == 0 or "pad" not in over:
        b = a[:8] + a[9:]
        if "pad" not in over and "kh" not in over:
            assert cc.capscaps_conv_fwd(FAKE, FAKE, FAKE, *b, None) == cc.EINVAL


def test_null_and_misaligned_pointers_and_bad_path():
    a = _args()
    for ptrs in ((None, FAKE, FAKE), (FAKE, None, FAKE), (FAKE, FAKE, None), (FAKE + 4, FAKE, FAKE),
                 (FAKE, FAKE + 8, FAKE), (FAKE, FAKE, FAKE + 2)):
        assert cc.capscaps_conv_fwd_ex(*ptrs, *a, FAKE, 1 << 30, None) == cc.EINVAL
        assert cc.capscaps_conv_fwd(*ptrs, *(a[:8] + a[9:]), None) == cc.EINVAL
    assert cc.capscaps_conv_fwd_path(FAKE, FAKE, FAKE, *a, 9, FAKE, 1 << 30, None) == cc.EINVAL
    # workspace checks come before any launch
    need = cc.capscaps_conv_fwd_workspace_bytes(*a)
    assert need > 0
    generic = cc.PATH_MFMA_GENERIC   # a forced kernel is held to the size the query reports
    assert cc.capscaps_conv_fwd_path(FAKE, FAKE, FAKE, *a, generic, None, 0, None) \
        == cc.EWORKSPACE
    assert cc.capscaps_conv_fwd_path(FAKE, FAKE, FAKE, *a, generic, FAKE, need - 1, None) \
        == cc.EWORKSPACE
    assert cc.capscaps_conv_fwd_path(FAKE, FAKE, FAKE, *a, generic, FAKE + 4, need, None) \
        == cc.EINVAL


def test_path_selection_and_workspace_sizes():
    for w in wl.CONFIGS:
        a = (w.N, w.H, w.W, w.C, w.M, w.kh, w.kw, w.stride, w.pad, w.D0, w.D1, w.D2, w.D3, w.dtype)
        assert cc.capscaps_select_path(*a) in (cc.PATH_MFMA_SMALL, cc.PATH_MFMA_TUNED16,
                                               cc.PATH_MFMA_TUNED32)
        kernel_bytes = w.kh * w.kw * w.C * w.M * w.D0 * w.D2 * w.D3 * w.elem_bytes
        assert cc.capscaps_conv_fwd_workspace_bytes(*a) >= kernel_bytes
    # the Fig. 2 example has 3 output columns and K = 48: measured, 16-column matrix-core tiles
    # still finish before the wavefront-level path; that path takes contractions of up to 24 values
    assert cc.capscaps_select_path(1, 5, 5, 1, 1, 4, 4, 1, 0, 3, 3, 3, 3, cc.FP32) == cc.PATH_MFMA_SMALL
    # ... the same layer on 256 images of 20x20: throughput counts, 3-element rows: wavefront-level
    assert cc.capscaps_select_path(256, 20, 20, 1, 1, 4, 4, 1, 0, 3, 3, 3, 3, cc.FP32) == cc.PATH_DIRECT
    assert cc.capscaps_select_path(256, 20, 20, 2, 4, 4, 4, 1, 0, 3, 3, 3, 3, cc.FP32) != cc.PATH_DIRECT
    assert cc.capscaps_select_path(64, 32, 32, 1, 8, 2, 2, 1, 0, 1, 4, 4, 4, cc.FP32) == cc.PATH_DIRECT
    assert cc.capscaps_select_path(2, 6, 6, 5, 7, 1, 1, 1, 0, 1, 1, 1, 1, cc.FP32) == cc.PATH_DIRECT
    # problems too small to fill the chip with the tuned kernels' tiles take the generic kernel's
    # small tiles, the smallest ones the single-launch small-problem kernel
    assert cc.capscaps_select_path(*_args(M=64, D3=16, D1=16, D2=16, C=64, dtype=cc.FP16)) \
        == cc.PATH_MFMA_GENERIC
    assert cc.capscaps_select_path(*_args(M=8, C=8, dtype=cc.FP16)) == cc.PATH_MFMA_SMALL
    picks = [cc.capscaps_select_path(w.N, w.H, w.W, w.C, w.M, w.kh, w.kw, w.stride, w.pad, w.D0,
                                     w.D1, w.D2, w.D3, w.dtype) for w in wl.CONFIGS]
    assert picks == [cc.PATH_MFMA_SMALL, cc.PATH_MFMA_TUNED32, cc.PATH_MFMA_TUNED16,
                     cc.PATH_MFMA_SMALL, cc.PATH_MFMA_TUNED16]
    # the small-problem kernel reads the kernel tensor in place: configuration 1 needs no scratch
    # on the library's own choice (the size query covers every forced path)
    w = wl.CONFIGS[0]
    a = (w.N, w.H, w.W, w.C, w.M, w.kh, w.kw, w.stride, w.pad, w.D0, w.D1, w.D2, w.D3, w.dtype)
    assert cc.capscaps_conv_fwd_ex(None, FAKE, FAKE, *a, None, 0, None) == cc.EINVAL


def test_strerror():
    assert cc.capscaps_strerror(cc.OK) == "success"
    for code in (cc.EINVAL, cc.EWORKSPACE, cc.EUNSUPPORTED, cc.EHIP, -99):
        assert cc.capscaps_strerror(code)


@pytest.mark.parametrize("over", [dict(N=0), dict(M=0), dict(D2=-1), dict(stride=0), dict(pad=-1),
                                  dict(kh=9), dict(dtype=3)])
def test_backward_comparison_and_out16_entry_points_reject_bad_shapes(over):
    a = _args(**over)
    big = 1 << 30
    assert cc.capscaps_conv_bwd_input(FAKE, FAKE, FAKE, *a, FAKE, big, None) == cc.EINVAL
    assert cc.capscaps_conv_bwd_kernel(FAKE, FAKE, FAKE, *a, FAKE, big, None) == cc.EINVAL
    assert cc.capscaps_conv_bwd_input_workspace_bytes(*a) == 0
    assert cc.capscaps_conv_bwd_kernel_workspace_bytes(*a) == 0
    assert cc.capscaps_scheme2_index_bytes(*a) == 0
    assert cc.capscaps_scheme2_build_index(FAKE, big, *a, None) == cc.EINVAL
    assert cc.capscaps_scheme2_fwd(FAKE, FAKE, FAKE, FAKE, big, *a, None) == cc.EINVAL
    a16 = _args(**{**over, "dtype": over.get("dtype", cc.FP16)})
    assert cc.capscaps_conv_fwd_out16(FAKE, FAKE, FAKE, *a16, FAKE, big, None) == cc.EINVAL
    assert cc.capscaps_conv_fwd_out16_workspace_bytes(*a16) == 0
    assert cc.capscaps_conv_bwd_input_out16(FAKE, FAKE, FAKE, *a16, FAKE, big, None) == cc.EINVAL
    assert cc.capscaps_conv_bwd_input_out16_workspace_bytes(*a16) == 0


def test_backward_pointer_and_workspace_checks():
    # (enough images for the kernel gradient to cut its contraction: partial sums in the scratch)
    a = _args(N=40, dtype=cc.FP16, D1=8, D2=8, D3=8)
    need_i = cc.capscaps_conv_bwd_input_workspace_bytes(*a)
    need_k = cc.capscaps_conv_bwd_kernel_workspace_bytes(*a)
    assert need_i > 0 and need_k > 0 and need_i % 256 == 0
    for fn, need in ((cc.capscaps_conv_bwd_input, need_i), (cc.capscaps_conv_bwd_kernel, need_k)):
        assert fn(0, FAKE, FAKE, *a, FAKE, need, None) == cc.EINVAL
        assert fn(FAKE, FAKE + 4, FAKE, *a, FAKE, need, None) == cc.EINVAL
        assert fn(FAKE, FAKE, FAKE, *a, FAKE, need - 1, None) == cc.EWORKSPACE
        assert fn(FAKE, FAKE, FAKE, *a, 0, 0, None) == cc.EWORKSPACE
        assert fn(FAKE, FAKE, FAKE, *a, FAKE + 8, need, None) == cc.EINVAL
    # 16-bit output is for 16-bit operands only
    assert cc.capscaps_conv_fwd_out16(FAKE, FAKE, FAKE, *_args(), FAKE, 1 << 30, None) == cc.EINVAL
    assert cc.capscaps_conv_fwd_out16_workspace_bytes(*_args()) == 0


def test_16bit_input_gradient_checks():
    # fp32 operands are refused; for 16-bit ones the same pointer and workspace rules hold
    assert cc.capscaps_conv_bwd_input_out16(FAKE, FAKE, FAKE, *_args(), FAKE, 1 << 30, None) == cc.EINVAL
    assert cc.capscaps_conv_bwd_input_out16_workspace_bytes(*_args()) == 0
    a = _args(dtype=cc.BF16, D1=8, D2=8, D3=8)
    need = cc.capscaps_conv_bwd_input_out16_workspace_bytes(*a)
    assert need > 0 and need % 256 == 0
    fn = cc.capscaps_conv_bwd_input_out16
    assert fn(0, FAKE, FAKE, *a, FAKE, need, None) == cc.EINVAL
    assert fn(FAKE, FAKE, FAKE + 4, *a, FAKE, need, None) == cc.EINVAL
    assert fn(FAKE, FAKE, FAKE, *a, FAKE, need - 1, None) == cc.EWORKSPACE
    assert fn(FAKE, FAKE, FAKE, *a, 0, 0, None) == cc.EWORKSPACE


def test_kernel_gradient_cuts_its_contraction_to_fill_the_chip():
    """The 16-bit kernel gradient reads these tensors in place, so its scratch is only the partial
    sums: (ranges a tap's pixel sequence is cut into) x (kernel tensor in fp32).  Tiles x ranges
    is to come close to a multiple of the 256 CUs."""
    def ranges(N, H, W, C, M, k, s, p, D, dtype):
        a = (N, H, W, C, M, k, k, s, p, 1, D, D, D, dtype)
        need = cc.capscaps_conv_bwd_kernel_workspace_bytes(*a)
        kernel_bytes = k * k * C * M * D * D * 4
        assert need % kernel_bytes == 0
        return need // kernel_bytes
    # config 5: 144 tiles (9 taps, 4 x 4 tiles of 256 x 256) x 16 = 9 full rounds
    assert ranges(64, 32, 32, 64, 64, 3, 1, 1, 16, cc.FP16) == 16
    # config 3: 9 tiles x 28 = 252 workgroups
    assert ranges(128, 28, 28, 32, 32, 3, 2, 1, 8, cc.BF16) == 28
    # 16 channels of 8x8 capsules are 128 rows: two taps per tile, 5 tiles x 51 = 255 workgroups
    assert ranges(64, 32, 32, 16, 32, 3, 1, 1, 8, cc.BF16) == 51
    # a layer too small to be worth cutting needs no scratch at all
    assert cc.capscaps_conv_bwd_kernel_workspace_bytes(2, 6, 6, 4, 4, 3, 3, 1, 1, 1, 8, 8, 8, cc.FP16) == 0


def test_scheme2_index_size_and_limits():
    a = _args()
    products = 2 * 6 * 6 * 4 * 3 * 3 * 3 * 1
    assert cc.capscaps_scheme2_index_bytes(*a) == products * 12
    # 2^31 or more input capsules: refused
    assert cc.capscaps_scheme2_index_bytes(*_args(N=1 << 20, H=64, W=64, C=8)) == 0


def test_yardstick_argument_checks():
    assert cc.capscaps_mfma_yardstick_flops(cc.FP16, 1024, 100) == 16 * 2 * 32 * 32 * 16 * 4 * 1024 * 100
    assert cc.capscaps_mfma_yardstick_flops(cc.FP32, 2, 3) == 16 * 4 * 2 * 32 * 32 * 2 * 4 * 2 * 3
    assert cc.capscaps_mfma_yardstick_flops(7, 1, 1) == 0
    assert cc.capscaps_mfma_yardstick(0, FAKE, cc.FP16, 1, 1, None) == cc.EINVAL
    assert cc.capscaps_mfma_yardstick(FAKE, FAKE, 5, 1, 1, None) == cc.EINVAL
    assert cc.capscaps_mfma_yardstick(FAKE, FAKE, cc.FP16, 0, 1, None) == cc.EINVAL
    assert cc.capscaps_mfma_yardstick(FAKE, FAKE, cc.FP16, 1, 0, None) == cc.EINVAL


def test_small_problem_kernel_is_left_for_larger_problems():
    for w in (wl.CONFIGS[1], wl.CONFIGS[2], wl.CONFIGS[4]):
        a = (w.N, w.H, w.W, w.C, w.M, w.kh, w.kw, w.stride, w.pad, w.D0, w.D1, w.D2, w.D3, w.dtype)
        assert cc.capscaps_select_path(*a) != cc.PATH_MFMA_SMALL
    # 16-bit problems leave earlier than fp32 ones (the kernel computes at the fp32 rate)
    mid = dict(N=4, H=16, W=16, C=16, M=16, D1=8, D2=8, D3=8)
    assert cc.capscaps_select_path(*_args(**mid)) == cc.PATH_MFMA_SMALL
    assert cc.capscaps_select_path(*_args(**mid, dtype=cc.BF16)) != cc.PATH_MFMA_SMALL


def test_huge_window_is_refused_not_wrapped():
    # a window over a whole large scalar image: kh*kw passes 2^31 and would wrap in 32 bits
    a = _args(N=1, H=46341, W=46341, C=1, M=1, kh=46341, kw=46341, pad=0, D1=1, D2=1, D3=1)
    assert cc.capscaps_select_path(*a) == cc.EUNSUPPORTED
    assert cc.capscaps_conv_fwd_ex(FAKE, FAKE, FAKE, *a, FAKE, 1 << 30, None) == cc.EUNSUPPORTED
    assert cc.capscaps_conv_fwd_workspace_bytes(*a) == 0
    assert cc.capscaps_conv_bwd_input(FAKE, FAKE, FAKE, *a, FAKE, 1 << 30, None) == cc.EUNSUPPORTED
    # 4096 x 4096 taps is the largest window taken
    b = _args(N=1, H=4096, W=4096, C=1, M=1, kh=4096, kw=4096, pad=0, D1=1, D2=1, D3=1)
    assert cc.capscaps_select_path(*b) > 0


def test_static_scratch_entry_point_checks_before_touching_the_gpu():
    a = _args()
    assert cc.capscaps_conv_fwd_static(None, FAKE, FAKE, *a, None) == cc.EINVAL
    assert cc.capscaps_conv_fwd_static(FAKE, FAKE + 4, FAKE, *a, None) == cc.EINVAL
    assert cc.capscaps_conv_fwd_static(FAKE, FAKE, FAKE, *_args(M=0), None) == cc.EINVAL
    # a repacked kernel larger than the fixed array
    big = _args(N=1, H=34, W=34, C=160, M=160, D1=16, D2=16, D3=16, dtype=cc.FP16)
    assert cc.capscaps_conv_fwd_static(FAKE, FAKE, FAKE, *big, None) == cc.ESCRATCH
    assert "scratch" in cc.capscaps_strerror(cc.ESCRATCH)
