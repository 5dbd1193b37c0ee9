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


def test_scheme1_cuts_large_problems_into_bounded_multiplies(monkeypatch):
    """No batched multiply is handed more than MAX_BMM_BATCH products: the blocks run over
    images and, within an image, over output pixels."""
    rng = np.random.default_rng(77)
    I = rng.standard_normal((3, 6, 7, 3, 2, 3, 3)).astype(np.float32)
    K = rng.standard_normal((3, 3, 3, 4, 2, 3, 3)).astype(np.float32)
    ref = capsconv.conv_fwd(I, K, 1, 1)
    seen = []
    real_bmm = torch.bmm

    def spy(a, b):
        seen.append(a.shape[0])
        return real_bmm(a, b)

    monkeypatch.setattr(torch, "bmm", spy)
    for limit in (4 * 27 * 2 * 5, 4 * 27 * 2 * 42 * 2):       # 5 pixels; two whole images
        monkeypatch.setattr(cmp, "MAX_BMM_BATCH", limit)
        seen.clear()
        got = cmp.scheme1_fwd(torch.from_numpy(I), torch.from_numpy(K), 1, 1).numpy()
        assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()
        assert len(seen) > 1 and max(seen) <= limit
        assert sum(seen) == 3 * 42 * 4 * 27 * 2                # every small product, once


def test_scheme1_refuses_oversized_batches():
    # more small products for ONE output pixel than a batched multiply is handed
    I = torch.zeros(1, 32, 32, 64, 1, 1, 1)
    K = torch.zeros(32, 32, 64, 64, 1, 1, 1)
    with pytest.raises(ValueError):
        cmp.scheme1_fwd(I, K, 1, 0)
