"""Pins for the CPU oracle's backward pass (dL/dI and dL/dK of the capsule convolution): the
adjoint identities that tie them to the pinned forward oracle, automatic differentiation of a
library convolution, exact finite differences of the bilinear forward map, closed forms and
special cases.  CPU only."""
import numpy as np
import pytest

from oracle import capsconv
from tests.test_oracle_pins import rand_f32, rand_int

SHAPES = [
    # N  H  W  C  M kh kw s  p D0 D1 D2 D3
    (2, 6, 7, 3, 2, 3, 3, 1, 1, 1, 4, 4, 4),
    (2, 7, 5, 2, 3, 2, 3, 2, 1, 3, 3, 3, 3),
    (1, 8, 8, 2, 2, 3, 3, 2, 0, 2, 2, 5, 3),
    (3, 5, 9, 1, 4, 5, 1, 1, 2, 1, 3, 2, 6),
    (2, 6, 6, 4, 3, 3, 3, 3, 1, 2, 1, 4, 1),
    (2, 7, 7, 2, 2, 2, 2, 3, 2, 1, 2, 3, 2),
]


def make(shape, seed, integer):
    N, H, W, C, M, kh, kw, s, p, D0, D1, D2, D3 = shape
    rng = np.random.default_rng(seed)
    mk = rand_int if integer else rand_f32
    I = mk(rng, (N, H, W, C, D0, D1, D2))
    K = mk(rng, (kh, kw, C, M, D0, D2, D3))
    Ho, Wo = capsconv.out_shape(H, W, kh, kw, s, p)
    G = mk(rng, (N, Ho, Wo, M, D0, D1, D3))
    return I, K, G


@pytest.mark.parametrize("shape", SHAPES)
def test_adjoint_identities_exact_on_integers(shape):
    """<conv(I,K), G> = <I, dI(G,K)> = <K, dK(I,G)>: with small integers every sum is exact,
    so the three numbers must be equal.  A linear map has exactly one adjoint, and several random
    (I, K, G) triples leave no room for a wrong one."""
    s, p = shape[7], shape[8]
    for seed in range(4):
        I, K, G = make(shape, 100 + seed, integer=True)
        O = capsconv.conv_fwd(I, K, s, p)
        dI = capsconv.conv_bwd_input(G, K, I.shape[1:3], s, p)
        dK = capsconv.conv_bwd_kernel(I, G, K.shape[:2], s, p)
        lhs = float((O * G).sum())
        assert lhs == float((I * dI).sum())
        assert lhs == float((K * dK).sum())


@pytest.mark.parametrize("shape", SHAPES)
def test_unit_gradients_pick_single_entries_of_the_forward_map(shape):
    """dI[e] = d<O,G>/dI[e] = <conv(unit_e, K), G> for single entries e (and likewise for K):
    the backward results entry by entry from the forward oracle alone."""
    s, p = shape[7], shape[8]
    I, K, G = make(shape, 7, integer=True)
    dI = capsconv.conv_bwd_input(G, K, I.shape[1:3], s, p)
    dK = capsconv.conv_bwd_kernel(I, G, K.shape[:2], s, p)
    rng = np.random.default_rng(8)
    for _ in range(12):
        e = tuple(rng.integers(0, d) for d in I.shape)
        unit = np.zeros_like(I)
        unit[e] = 1
        assert dI[e] == float((capsconv.conv_fwd(unit, K, s, p) * G).sum())
        e = tuple(rng.integers(0, d) for d in K.shape)
        unit = np.zeros_like(K)
        unit[e] = 1
        assert dK[e] == float((capsconv.conv_fwd(I, unit, s, p) * G).sum())


@pytest.mark.parametrize("shape", SHAPES)
def test_equals_autograd_of_grouped_conv2d(shape):
    """The operator is a grouped conv2d (groups D0, batch (n,d1), channels (c,d2) -> (m,d3)):
    torch's CPU autograd through that library routine, in float64."""
    import torch
    import torch.nn.functional as F
    N, H, W, C, M, kh, kw, s, p, D0, D1, D2, D3 = shape
    I, K, G = make(shape, 21, integer=False)
    X = torch.from_numpy(I.astype(np.float64)).requires_grad_(True)
    Wt = torch.from_numpy(K.astype(np.float64)).requires_grad_(True)
    Xp = X.permute(0, 5, 4, 3, 6, 1, 2).reshape(N * D1, D0 * C * D2, H, W)
    Wp = Wt.permute(4, 3, 6, 2, 5, 0, 1).reshape(D0 * M * D3, C * D2, kh, kw)
    Y = F.conv2d(Xp, Wp, stride=s, padding=p, groups=D0)
    Ho, Wo = Y.shape[-2:]
    Y = Y.reshape(N, D1, D0, M, D3, Ho, Wo).permute(0, 5, 6, 3, 2, 1, 4)
    (Y * torch.from_numpy(G.astype(np.float64))).sum().backward()
    dI = capsconv.conv_bwd_input(G, K, (H, W), s, p)
    dK = capsconv.conv_bwd_kernel(I, G, (kh, kw), s, p)
    np.testing.assert_allclose(dI, X.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dK, Wt.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_worked_example_gradient_counts_the_windows():
    """Fig. 2's layer (all-ones 4x4 kernel of 3x3x3 capsules on 5x5, stride 1) with an all-ones
    output gradient: dI at pixel (h,w) = D3 * (#windows covering h) * (#windows covering w);
    dK = D1 * (number of output pixels) everywhere."""
    K = np.ones((4, 4, 1, 1, 3, 3, 3), np.float32)
    G = np.ones((1, 2, 2, 1, 3, 3, 3), np.float32)
    dI = capsconv.conv_bwd_input(G, K, (5, 5))
    cover = np.array([1, 2, 2, 2, 1])
    for h in range(5):
        for w in range(5):
            assert np.all(dI[0, h, w] == 3 * cover[h] * cover[w])
    I = np.ones((1, 5, 5, 1, 3, 3, 3), np.float32)
    dK = capsconv.conv_bwd_kernel(I, G, (4, 4))
    assert dK.shape == (4, 4, 1, 1, 3, 3, 3) and np.all(dK == 3 * 4)


def test_fully_connected_gradients_are_gemms():
    rng = np.random.default_rng(31)
    N, H, W, C, M, D0, D1, D2, D3 = 3, 3, 2, 2, 4, 2, 3, 4, 2
    I = rand_f32(rng, (N, H, W, C, D0, D1, D2))
    K = rand_f32(rng, (H, W, C, M, D0, D2, D3))
    G = rand_f32(rng, (N, 1, 1, M, D0, D1, D3))
    dI = capsconv.conv_bwd_input(G, K, (H, W))
    dK = capsconv.conv_bwd_kernel(I, G, (H, W))
    for d0 in range(D0):
        A = I[:, :, :, :, d0].astype(np.float64).transpose(0, 4, 1, 2, 3, 5).reshape(N * D1, -1)
        B = K[:, :, :, :, d0].astype(np.float64).transpose(0, 1, 2, 4, 3, 5).reshape(-1, M * D3)
        Gm = G[:, 0, 0, :, d0].astype(np.float64).transpose(0, 2, 1, 3).reshape(N * D1, M * D3)
        dA = (Gm @ B.T).reshape(N, D1, H, W, C, D2).transpose(0, 2, 3, 4, 1, 5)
        dB = (A.T @ Gm).reshape(H, W, C, D2, M, D3).transpose(0, 1, 2, 4, 3, 5)
        np.testing.assert_allclose(dI[:, :, :, :, d0], dA, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(dK[:, :, :, :, d0], dB, rtol=1e-12, atol=1e-12)


def test_rejects_shapes_that_do_not_fit():
    I, K, G = make(SHAPES[0], 1, integer=True)
    with pytest.raises(ValueError):
        capsconv.conv_bwd_input(G, K, (9, 9), 1, 1)
    with pytest.raises(ValueError):
        capsconv.conv_bwd_kernel(I, G[:, :-1], (3, 3), 1, 1)
