"""Host-side checks of the seeded input generators (no arithmetic of the operator here)."""
import numpy as np
import pytest

from paper_2104_02621_amd import workloads as wl


def test_five_configs_and_their_sizes():
    shapes = [(w.Ho, w.Wo) for w in wl.CONFIGS]
    assert shapes == [(14, 14), (32, 32), (14, 14), (1, 1), (32, 32)]
    assert wl.config(1).flops_nominal() == 28_901_376
    assert wl.config(2).flops_nominal() == 97_844_723_712
    assert wl.config(3).flops_nominal() == 947_040_288_768
    assert wl.config(4).flops_nominal() == 377_487_360
    assert wl.config(5).flops_nominal() == 19_791_209_299_968
    assert wl.config(1).flops_tap_exact() == wl.config(1).flops_nominal()
    # stride 1, pad 1, 3x3 on 32: (94/96)^2 of the taps are in range
    assert wl.config(5).flops_tap_exact() * 96 * 96 == wl.config(5).flops_nominal() * 94 * 94
    assert wl.config(3).flops_tap_exact() * 42 * 42 == wl.config(3).flops_nominal() * 41 * 41
    assert wl.config(5).compulsory_bytes() == 2_147_483_648 + 18_874_368 + 4_294_967_296


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.14159, 1e-3],
                 np.float32)
    bits = wl.round_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(bits)
    # ties go to even mantissa: 1+2^-8 -> 1, 1+3*2^-8 -> 1+2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.0 + 2 ** -7
    assert back[3] == 1.0 + 2 ** -6
    import torch
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(back, ref)
    big = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    ref = torch.from_numpy(big).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(wl.bf16_bits_to_f32(wl.round_to_bf16_bits(big)), ref)


@pytest.mark.parametrize("num", [1, 4])
def test_generation_is_deterministic_and_in_distribution(num):
    w = wl.config(num)
    a = wl.generate(w)
    b = wl.generate(w)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    i32, k32 = a[2], a[3]
    assert i32.shape == w.input_shape and k32.shape == w.kernel_shape
    assert -1.0 <= i32.min() and i32.max() <= 1.0
    if w.kernel_dist == "normal":
        assert abs(k32.std() / w.kernel_sigma - 1) < 0.05


def test_storage_and_widened_values_agree():
    w = wl.config(3).with_batch(1)
    i_st, k_st, i32, k32 = wl.generate(w)
    assert i_st.dtype == np.uint16 and np.array_equal(wl.bf16_bits_to_f32(i_st), i32)
    w = wl.config(5).with_batch(1)
    i_st, k_st, i32, k32 = wl.generate(w)
    assert i_st.dtype == np.float16 and np.array_equal(i_st.astype(np.float32), i32)


def test_sampled_capsules_are_in_range_and_repeatable():
    w = wl.config(3)
    s = wl.sample_capsules(w, 1000, seed=7)
    assert s.shape == (1000, 4) and s.dtype == np.int32
    assert np.array_equal(s, wl.sample_capsules(w, 1000, seed=7))
    assert (s >= 0).all() and (s[:, 0] < w.N).all() and (s[:, 1] < w.Ho).all()
    assert (s[:, 2] < w.Wo).all() and (s[:, 3] < w.M).all()
    on_border = (s[:, 1] == 0) | (s[:, 1] == w.Ho - 1) | (s[:, 2] == 0) | (s[:, 2] == w.Wo - 1)
    assert on_border.sum() >= 250
