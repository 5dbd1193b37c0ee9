"""GPU parity of the small-problem kernel (one launch, kernel tensor read in place, 16-column
tiles, the K loop shared by the four waves of a workgroup and, for long K loops on few tiles, cut
over workgroups with a fixed-order reduction) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import capsconv
from paper_2104_02621_amd import capscaps as cc
from paper_2104_02621_amd import workloads as wl
from tests.gpu_util import run_gpu, shape_args, to_device
from tests.test_gpu_parity import full_compare, small

pytestmark = pytest.mark.gpu

# shapes that exercise what the kernel decides by shape: one or two 16-row MFMA tiles per
# workgroup, 1..4 column tiles of 16 and several workgroups across the columns, K loops of one
# slab, of several with a ragged last one, and cut over workgroups (few tiles, long K), every
# combination of vector and element-wise loads (D2, D3 multiples of 4 or not), leading capsule
# dimension, strides, padding
SHAPES = [
    #         N  H   W   C   M  kh kw s  p D0  D1  D2  D3
    ("rows16", 1, 3, 3, 2, 2, 2, 2, 1, 0, 1, 4, 4, 4),     # 16 rows: one MFMA row tile
    ("cols48", 2, 6, 6, 3, 12, 3, 3, 1, 1, 1, 4, 4, 4),    # 48 columns
    ("cols80", 2, 5, 5, 2, 20, 3, 3, 1, 0, 1, 4, 4, 4),    # 80 columns: two column tiles
    ("cols200", 1, 4, 4, 2, 25, 2, 2, 1, 0, 1, 4, 4, 8),   # four column tiles, ragged
    ("fc_split", 24, 6, 6, 16, 10, 6, 6, 1, 0, 1, 4, 4, 4),  # 3 tiles, 36 slabs: K cut 9 ways
    ("fc_split3", 7, 5, 4, 9, 3, 5, 4, 1, 0, 2, 3, 5, 3),    # element-wise loads, D0 = 2, K cut
    ("kragged", 3, 8, 8, 5, 4, 3, 3, 2, 1, 1, 4, 4, 4),    # K = 180: three slabs, last ragged
    ("d2vec", 2, 7, 7, 3, 4, 3, 3, 1, 1, 1, 3, 8, 5),      # D2 in pieces of 4, D3 element-wise
    ("d3vec", 2, 7, 7, 3, 4, 3, 3, 1, 1, 1, 5, 3, 8),      # D2 element-wise, D3 in pieces of 4
    ("d0", 2, 6, 5, 4, 3, 2, 3, 1, 1, 3, 4, 4, 4),         # leading capsule index
    ("bigwin", 2, 9, 9, 2, 3, 9, 9, 1, 2, 1, 4, 4, 4),     # 81 taps, most of them in the padding
]


@pytest.mark.parametrize("dtype", [wl.FP32, wl.BF16, wl.FP16], ids=["fp32", "bf16", "fp16"])
@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_small_kernel_matches_oracle(shape, dtype):
    w = small(shape[0], dtype, *shape[1:], seed=len(shape[0]) + 120)
    full_compare(w, cc.PATH_MFMA_SMALL)
    wi = small(shape[0] + "_int", dtype, *shape[1:], dist="int", seed=121)
    i_st, k_st, i32, k32 = wl.generate(wi)
    ref = capsconv.conv_fwd(i32, k32, wi.stride, wi.pad)
    got = run_gpu(wi, to_device(i_st, dtype), to_device(k_st, dtype), cc.PATH_MFMA_SMALL)
    assert np.array_equal(got.cpu().numpy().astype(np.float64), ref), wi.name


@pytest.mark.parametrize("num", [1, 4])
def test_library_picks_it_for_the_launch_bound_configs(num):
    """Configurations 1 and 4: the library's own choice, full tensor against the oracle, integer
    data bit-exact, reruns bit-identical (configuration 4's K loop is cut over 8 workgroups per
    tile and reduced in a fixed order)."""
    import torch
    w = wl.config(num)
    assert cc.capscaps_select_path(*shape_args(w)) == cc.PATH_MFMA_SMALL
    full_compare(w, cc.PATH_AUTO)
    i_st, k_st, _, _ = wl.generate(w)
    I, K = to_device(i_st, w.dtype), to_device(k_st, w.dtype)
    a = run_gpu(w, I, K, cc.PATH_AUTO)
    b = run_gpu(w, I, K, cc.PATH_AUTO)
    assert torch.equal(a, b)
    wi = wl.integer_variant(w)
    i_st, k_st, i32, k32 = wl.generate(wi)
    ref = capsconv.conv_fwd(i32, k32, wi.stride, wi.pad)
    got = run_gpu(wi, to_device(i_st, wi.dtype), to_device(k_st, wi.dtype), cc.PATH_AUTO)
    assert np.array_equal(got.cpu().numpy().astype(np.float64), ref)
