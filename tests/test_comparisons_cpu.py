"""The two framework-op comparison implementations are device-agnostic: on CPU tensors they must
reproduce the oracle too (the GPU tests repeat this on the device, together with scheme 2)."""
import numpy as np
import pytest
import torch

from oracle import capsconv
from paper_2104_02621_amd import comparisons as cmp

CASES = [
    # N  H  W  C  M kh kw s  p D0 D1 D2 D3
    (2, 5, 6, 2, 3, 2, 3, 1, 0, 2, 3, 4, 5),
    (2, 7, 6, 3, 2, 3, 3, 2, 1, 1, 4, 4, 4),
    (3, 4, 4, 2, 5, 4, 4, 1, 0, 1, 2, 3, 2),   # fully connected
    (1, 5, 5, 1, 1, 4, 4, 1, 0, 3, 3, 3, 3),   # Fig. 2's geometry
    (1, 3, 3, 2, 2, 3, 3, 2, 3, 1, 2, 4, 2),   # padding wider than the window's reach
]


@pytest.mark.parametrize("case", CASES)
def test_scheme1_and_framework_conv_match_oracle(case):
    N, H, W, C, M, kh, kw, s, p, D0, D1, D2, D3 = case
    rng = np.random.default_rng(sum(case))
    I = rng.standard_normal((N, H, W, C, D0, D1, D2)).astype(np.float32)
    K = rng.standard_normal((kh, kw, C, M, D0, D2, D3)).astype(np.float32)
    ref = capsconv.conv_fwd(I, K, s, p)
    scale = np.abs(ref).max()
    # a small element budget forces the image-group loop of scheme 1 through several rounds
    a = cmp.scheme1_fwd(torch.from_numpy(I), torch.from_numpy(K), s, p, max_batch_elems=3000)
    b = cmp.framework_conv_fwd(torch.from_numpy(I), torch.from_numpy(K), s, p)
    assert a.shape == b.shape == ref.shape
    assert np.abs(a.numpy() - ref).max() <= 1e-5 * scale
    assert np.abs(b.numpy() - ref).max() <= 1e-5 * scale


def test_fig2_all_ones_gives_48():
    """Fig. 2's worked example through both formulations."""
    I = torch.ones(1, 5, 5, 1, 3, 3, 3)
    K = torch.ones(4, 4, 1, 1, 3, 3, 3)
    assert torch.equal(cmp.scheme1_fwd(I, K), torch.full((1, 2, 2, 1, 3, 3, 3), 48.0))
    assert torch.equal(cmp.framework_conv_fwd(I, K), torch.full((1, 2, 2, 1, 3, 3, 3), 48.0))


def test_scheme1_refuses_oversized_batches():
    I = torch.zeros(1, 64, 64, 64, 1, 2, 2)
    K = torch.zeros(3, 3, 64, 64, 1, 2, 2)
    with pytest.raises(ValueError):
        cmp.scheme1_fwd(I, K, 1, 1)
