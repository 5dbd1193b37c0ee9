"""Pins for the CPU oracle: every check compares it with something that is not the oracle --
values the paper prints, closed forms, textbook/library special cases, other formulations of
the same sum, and invariants of the definition.  CPU only."""
import itertools
import os

import numpy as np
import pytest

from oracle import capsconv

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_fixture(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = (s.strip() for s in line.split("="))
            vals[k] = int(v)
    return vals


def rand_int(rng, shape, lo=-3, hi=3):
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)


def rand_f32(rng, shape):
    return rng.standard_normal(shape).astype(np.float32)


# ------------------------------------------------------------------------ P1: paper's numbers
def test_fig2_worked_example():
    """Fig. 2: all-ones 1x5x5x(3x3x3) input, all-ones 4x4x1x1x(3x3x3) kernel -> 2x2 of 48s.
    (Contracting over the leading capsule index too would give 144; dropping a tap row 36.)"""
    g = read_fixture("fig2_worked_example.txt")
    I = np.full((1, g["in_height"], g["in_width"], g["in_channels"], g["capsule_d0"],
                 g["capsule_d1"], g["capsule_d2"]), g["input_value"], np.float32)
    K = np.full((g["kernel_height"], g["kernel_width"], g["in_channels"], g["out_channels"],
                 g["capsule_d0"], g["capsule_d2"], g["capsule_d3"]), g["kernel_value"], np.float32)
    O = capsconv.conv_fwd(I, K, stride=g["stride"], pad=g["pad"])
    assert O.shape == (1, g["out_height"], g["out_width"], g["out_channels"], g["capsule_d0"],
                       g["capsule_d1"], g["capsule_d3"])
    assert np.all(O == g["output_value"])


def test_fig1_output_extent():
    g = read_fixture("fig1_shapes.txt")
    assert capsconv.out_shape(g["in_height"], g["in_width"], g["kernel_height"],
                              g["kernel_width"], g["stride"], g["pad"]) == (g["out_height"],
                                                                            g["out_width"])


@pytest.mark.parametrize("H,k,s,p,expect", [(28, 3, 2, 1, 14), (32, 3, 1, 1, 32), (6, 6, 1, 0, 1),
                                            (16, 3, 1, 0, 14), (7, 3, 3, 0, 2), (7, 2, 3, 2, 4)])
def test_output_extent_floor(H, k, s, p, expect):
    assert capsconv.out_shape(H, H, k, k, s, p) == (expect, expect)


# ------------------------------------------------------------------------ P2: closed form
@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 1), (2, 1), (2, 2), (3, 1)])
def test_constant_inputs_closed_form(stride, pad):
    """Input all a, kernel all b: O = a*b*C*D2*(number of in-range taps at that pixel)."""
    N, H, W, C, M, kh, kw, D0, D1, D2, D3 = 2, 7, 6, 3, 2, 3, 2, 2, 3, 5, 4
    a, b = 0.5, -2.0
    I = np.full((N, H, W, C, D0, D1, D2), a, np.float32)
    K = np.full((kh, kw, C, M, D0, D2, D3), b, np.float32)
    O = capsconv.conv_fwd(I, K, stride=stride, pad=pad)
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    assert O.shape == (N, Ho, Wo, M, D0, D1, D3)
    for x in range(Ho):
        rows = sum(0 <= x * stride - pad + p < H for p in range(kh))
        for y in range(Wo):
            cols = sum(0 <= y * stride - pad + q < W for q in range(kw))
            assert np.all(O[:, x, y] == a * b * C * D2 * rows * cols), (x, y)


# ------------------------------------------------------------------------ P3: scalar capsules
def test_scalar_capsules_are_ordinary_cross_correlation():
    """D0=D1=D2=D3=1 is Algorithm 1: multi-channel 2-D cross-correlation (no kernel flip)."""
    from scipy.signal import correlate2d
    rng = np.random.default_rng(3)
    N, H, W, C, M, kh, kw = 2, 9, 8, 3, 4, 3, 4
    I = rand_int(rng, (N, H, W, C, 1, 1, 1))
    K = rand_int(rng, (kh, kw, C, M, 1, 1, 1))
    O = capsconv.conv_fwd(I, K)
    for n, m in itertools.product(range(N), range(M)):
        ref = sum(correlate2d(I[n, :, :, c, 0, 0, 0].astype(np.float64),
                              K[:, :, c, m, 0, 0, 0].astype(np.float64), mode="valid")
                  for c in range(C))
        assert np.array_equal(O[n, :, :, m, 0, 0, 0], ref)


# ------------------------------------------------------------------------ P4: fully connected
def test_fully_connected_layer_is_one_gemm():
    """Kernel covering the whole input (Sec. 1.1: the FC capsule layer is a special case):
    per leading index d0, O[(n,d1),(m,d3)] = A[(n,d1),(h,w,c,d2)] @ B[(h,w,c,d2),(m,d3)]."""
    rng = np.random.default_rng(4)
    N, H, W, C, M, D0, D1, D2, D3 = 3, 4, 3, 2, 5, 2, 3, 4, 2
    I = rand_f32(rng, (N, H, W, C, D0, D1, D2))
    K = rand_f32(rng, (H, W, C, M, D0, D2, D3))
    O = capsconv.conv_fwd(I, K)
    assert O.shape == (N, 1, 1, M, D0, D1, D3)
    for d0 in range(D0):
        A = I[:, :, :, :, d0].astype(np.float64)               # n h w c d1 d2
        A = A.transpose(0, 4, 1, 2, 3, 5).reshape(N * D1, H * W * C * D2)
        B = K[:, :, :, :, d0].astype(np.float64)               # h w c m d2 d3
        B = B.transpose(0, 1, 2, 4, 3, 5).reshape(H * W * C * D2, M * D3)
        ref = (A @ B).reshape(N, D1, M, D3).transpose(0, 2, 1, 3)
        np.testing.assert_allclose(O[:, 0, 0, :, d0], ref, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------------ P5: grouped conv2d
def grouped_conv2d_reference(I, K, stride, pad):
    """The operator as a library grouped convolution: groups = D0, batch = (n, d1),
    in-channels per group = (c, d2), out-channels per group = (m, d3).  float64 on CPU."""
    import torch
    import torch.nn.functional as F
    N, H, W, C, D0, D1, D2 = I.shape
    kh, kw, _, M, _, _, D3 = K.shape
    X = torch.from_numpy(I.astype(np.float64)).permute(0, 5, 4, 3, 6, 1, 2)  # n d1 d0 c d2 h w
    X = X.reshape(N * D1, D0 * C * D2, H, W)
    Wt = torch.from_numpy(K.astype(np.float64)).permute(4, 3, 6, 2, 5, 0, 1)  # d0 m d3 c d2 p q
    Wt = Wt.reshape(D0 * M * D3, C * D2, kh, kw)
    Y = F.conv2d(X, Wt, stride=stride, padding=pad, groups=D0)                # (n d1) (d0 m d3)
    Ho, Wo = Y.shape[-2:]
    Y = Y.reshape(N, D1, D0, M, D3, Ho, Wo).permute(0, 5, 6, 3, 2, 1, 4)
    return Y.contiguous().numpy()


@pytest.mark.parametrize("shape", [
    # N  H  W  C  M kh kw s  p D0 D1 D2 D3
    (2, 6, 7, 3, 2, 3, 3, 1, 1, 1, 4, 4, 4),
    (2, 7, 5, 2, 3, 2, 3, 2, 1, 3, 3, 3, 3),
    (1, 8, 8, 2, 2, 3, 3, 2, 0, 2, 2, 5, 3),
    (3, 5, 9, 1, 4, 5, 1, 1, 2, 1, 3, 2, 6),
    (2, 6, 6, 4, 3, 3, 3, 3, 1, 2, 1, 4, 1),
])
def test_equals_grouped_conv2d(shape):
    N, H, W, C, M, kh, kw, s, p, D0, D1, D2, D3 = shape
    rng = np.random.default_rng(sum(shape))
    I = rand_f32(rng, (N, H, W, C, D0, D1, D2))
    K = rand_f32(rng, (kh, kw, C, M, D0, D2, D3))
    O = capsconv.conv_fwd(I, K, stride=s, pad=p)
    np.testing.assert_allclose(O, grouped_conv2d_reference(I, K, s, p), rtol=1e-11, atol=1e-11)


# ------------------------------------------------------------------------ P6: Algorithm 3 dataflow
def scheme1_reference(I, K, stride, pad):
    """Algorithm 3's dataflow in numpy: capsule im2col -> replicate input per output channel
    -> replicate kernel per output pixel -> one batched small-matrix multiply -> sum the
    kh*kw*C product matrices of each output capsule."""
    I = I.astype(np.float64)
    K = K.astype(np.float64)
    N, H, W, C, D0, D1, D2 = I.shape
    kh, kw, _, M, _, _, D3 = K.shape
    Ip = np.zeros((N, H + 2 * pad, W + 2 * pad, C, D0, D1, D2))
    Ip[:, pad:pad + H, pad:pad + W] = I
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    cols = np.empty((N, Ho, Wo, kh, kw, C, D0, D1, D2))            # capsule_im2col
    for x in range(Ho):
        for y in range(Wo):
            cols[:, x, y] = Ip[:, x * stride:x * stride + kh, y * stride:y * stride + kw]
    I_ext = np.broadcast_to(cols[:, :, :, None], (N, Ho, Wo, M, kh, kw, C, D0, D1, D2))
    K_ext = np.broadcast_to(K.transpose(3, 0, 1, 2, 4, 5, 6)[None, None, None],
                            (N, Ho, Wo, M, kh, kw, C, D0, D2, D3))
    O_ext = np.matmul(I_ext, K_ext)                                # batched small matmuls
    return O_ext.sum(axis=(4, 5, 6))                               # output_reduce


@pytest.mark.parametrize("stride,pad", [(1, 0), (2, 0), (1, 1), (2, 1)])
def test_equals_scheme1_dataflow(stride, pad):
    rng = np.random.default_rng(60 + stride * 2 + pad)
    N, H, W, C, M, kh, kw, D0, D1, D2, D3 = 2, 5, 6, 2, 3, 2, 3, 2, 3, 4, 5
    I = rand_f32(rng, (N, H, W, C, D0, D1, D2))
    K = rand_f32(rng, (kh, kw, C, M, D0, D2, D3))
    O = capsconv.conv_fwd(I, K, stride=stride, pad=pad)
    np.testing.assert_allclose(O, scheme1_reference(I, K, stride, pad), rtol=1e-11, atol=1e-11)


# ------------------------------------------------------------------------ P7: Algorithm 2 flat offsets
def flat_offset_reference(I, K, stride):
    """Algorithm 2 / Algorithm 5 dataflow in pure Python on flat buffers in the paper's own
    memory order (input [C][H][W][caps], kernel [C'][C][h][w][caps], output [C'][H'][W'][caps]),
    one image, no padding.  Per-location strides are D0*D1*D2, D0*D2*D3 and D0*D1*D3; the
    innermost loop index selects one matrix of the capsule's leading dimension."""
    H, W, C, D0, D1, D2 = I.shape
    kh, kw, _, M, _, _, D3 = K.shape
    Ho, Wo = (H - kh) // stride + 1, (W - kw) // stride + 1
    Iflat = I.astype(np.float64).transpose(2, 0, 1, 3, 4, 5).ravel()       # c h w d0 d1 d2
    Kflat = K.astype(np.float64).transpose(3, 2, 0, 1, 4, 5, 6).ravel()    # m c p q d0 d2 d3
    Oflat = np.zeros(M * Ho * Wo * D0 * D1 * D3)
    for oc in range(M):
        for i in range(Ho):
            for j in range(Wo):
                row_offset, col_offset = i * stride, j * stride
                for s in range(C):
                    for m in range(kh):
                        for n in range(kw):
                            for c in range(D0):
                                idx = (oc * C * kh * kw + s * kh * kw + m * kw + n) * D0 * D2 * D3 \
                                    + c * D2 * D3
                                i_idx = (s * H * W + (row_offset + m) * W + col_offset + n) \
                                    * D0 * D1 * D2 + c * D1 * D2
                                o_idx = (oc * Ho * Wo + i * Wo + j) * D0 * D1 * D3 + c * D1 * D3
                                A = Iflat[i_idx:i_idx + D1 * D2].reshape(D1, D2)
                                B = Kflat[idx:idx + D2 * D3].reshape(D2, D3)
                                Oflat[o_idx:o_idx + D1 * D3] += (A @ B).ravel()
    return Oflat.reshape(M, Ho, Wo, D0, D1, D3).transpose(1, 2, 0, 3, 4, 5)


@pytest.mark.parametrize("stride", [1, 2])
def test_equals_flat_offset_loop(stride):
    rng = np.random.default_rng(70 + stride)
    H, W, C, M, kh, kw, D0, D1, D2, D3 = 5, 6, 2, 3, 3, 2, 3, 2, 4, 3
    I = rand_f32(rng, (1, H, W, C, D0, D1, D2))
    K = rand_f32(rng, (kh, kw, C, M, D0, D2, D3))
    O = capsconv.conv_fwd(I, K, stride=stride)
    np.testing.assert_allclose(O[0], flat_offset_reference(I[0], K, stride), rtol=1e-11,
                               atol=1e-11)


# ------------------------------------------------------------------------ P8: invariants
def _case(seed, D=(2, 3, 4, 2), N=2, H=7, W=6, C=3, M=2, kh=3, kw=2, integer=True):
    rng = np.random.default_rng(seed)
    D0, D1, D2, D3 = D
    mk = rand_int if integer else rand_f32
    return mk(rng, (N, H, W, C, D0, D1, D2)), mk(rng, (kh, kw, C, M, D0, D2, D3))


def test_bilinear():
    I1, K1 = _case(80)
    I2, K2 = _case(81)
    f = capsconv.conv_fwd
    assert np.array_equal(f(2 * I1 - 3 * I2, K1, 2, 1), 2 * f(I1, K1, 2, 1) - 3 * f(I2, K1, 2, 1))
    assert np.array_equal(f(I1, K1 + 2 * K2, 1, 1), f(I1, K1, 1, 1) + 2 * f(I1, K2, 1, 1))


@pytest.mark.parametrize("pad", [1, 2])
def test_padding_equals_explicit_zero_border(pad):
    I, K = _case(82, integer=False)
    Ip = np.zeros((I.shape[0], I.shape[1] + 2 * pad, I.shape[2] + 2 * pad) + I.shape[3:],
                  np.float32)
    Ip[:, pad:-pad, pad:-pad] = I
    assert np.array_equal(capsconv.conv_fwd(I, K, 2, pad), capsconv.conv_fwd(Ip, K, 2, 0))


@pytest.mark.parametrize("stride", [2, 3])
def test_stride_subsamples_stride_one(stride):
    I, K = _case(83, H=9, W=8, integer=False)
    full = capsconv.conv_fwd(I, K, 1, 1)
    assert np.array_equal(capsconv.conv_fwd(I, K, stride, 1), full[:, ::stride, ::stride])


def test_translation_equivariance_in_the_interior():
    I, K = _case(84, H=8, W=8, integer=False)
    shifted = np.zeros_like(I)
    shifted[:, 1:, 2:] = I[:, :-1, :-2]
    a = capsconv.conv_fwd(I, K)
    b = capsconv.conv_fwd(shifted, K)
    assert np.array_equal(b[:, 1:, 2:], a[:, :-1, :-2])


def test_batch_and_channel_permutations():
    I, K = _case(85, N=3, M=4, integer=False)
    O = capsconv.conv_fwd(I, K, 1, 1)
    perm_n, perm_m, perm_c = [2, 0, 1], [3, 1, 0, 2], [1, 2, 0]
    assert np.array_equal(capsconv.conv_fwd(I[perm_n], K, 1, 1), O[perm_n])
    assert np.array_equal(capsconv.conv_fwd(I, K[:, :, :, perm_m], 1, 1), O[:, :, :, perm_m])
    # permuting input channels of both operands only reorders the sum
    np.testing.assert_allclose(capsconv.conv_fwd(I[:, :, :, perm_c], K[:, :, perm_c], 1, 1), O,
                               rtol=1e-12, atol=1e-12)


def test_identity_kernel_returns_input():
    rng = np.random.default_rng(86)
    N, H, W, C, D0, D1, D2 = 2, 4, 5, 3, 2, 3, 4
    I = rand_f32(rng, (N, H, W, C, D0, D1, D2))
    K = np.zeros((1, 1, C, C, D0, D2, D2), np.float32)
    for c in range(C):
        for d0 in range(D0):
            K[0, 0, c, c, d0] = np.eye(D2)
    assert np.array_equal(capsconv.conv_fwd(I, K), I.astype(np.float64))


def test_leading_index_is_a_batch_not_a_contraction():
    """Each d0 slice of the output depends only on the same d0 slice of input and kernel."""
    I, K = _case(87, D=(3, 2, 3, 2), integer=False)
    O = capsconv.conv_fwd(I, K, 1, 1)
    for d0 in range(3):
        Od = capsconv.conv_fwd(I[:, :, :, :, d0:d0 + 1], K[:, :, :, :, d0:d0 + 1], 1, 1)
        assert np.array_equal(O[:, :, :, :, d0:d0 + 1], Od)


# ------------------------------------------------------------------------ P9: orientation catcher
def test_single_capsule_lands_where_and_how_the_definition_says():
    """One non-zero, non-symmetric, non-square input capsule E at (h0, w0, c0): the output at
    (h0-p, w0-q) is exactly E @ K[p,q,c0,m] per leading index.  Catches a flipped kernel,
    K.I instead of I.K, transposed capsules, swapped spatial axes and d0/d1 mix-ups."""
    rng = np.random.default_rng(9)
    N, H, W, C, M, kh, kw, D0, D1, D2, D3 = 1, 6, 7, 3, 2, 3, 2, 2, 2, 3, 4
    K = rand_int(rng, (kh, kw, C, M, D0, D2, D3))
    E = rand_int(rng, (D0, D1, D2), 1, 5)
    h0, w0, c0 = 3, 4, 1
    I = np.zeros((N, H, W, C, D0, D1, D2), np.float32)
    I[0, h0, w0, c0] = E
    O = capsconv.conv_fwd(I, K)
    expect = np.zeros_like(O)
    for p in range(kh):
        for q in range(kw):
            x, y = h0 - p, w0 - q
            if 0 <= x < O.shape[1] and 0 <= y < O.shape[2]:
                for m in range(M):
                    for d0 in range(D0):
                        expect[0, x, y, m, d0] = E[d0].astype(np.float64) @ K[p, q, c0, m, d0]
    assert np.array_equal(O, expect)
    assert np.count_nonzero(O) > 0


# ------------------------------------------------------------------------ subset entry point, S, errors
def test_subset_matches_full_and_abs_sum():
    I, K = _case(90, integer=False)
    O, S = capsconv.conv_fwd(I, K, 2, 1, with_abs_sum=True)
    which = np.array([(n, x, y, m) for n in range(O.shape[0]) for x in range(O.shape[1])
                      for y in range(O.shape[2]) for m in range(O.shape[3])][::3], np.int32)
    Os, Ss = capsconv.conv_fwd_subset(I, K, which, 2, 1, with_abs_sum=True)
    for i, (n, x, y, m) in enumerate(which):
        assert np.array_equal(Os[i], O[n, x, y, m])
        assert np.array_equal(Ss[i], S[n, x, y, m])
    # S is the same operator applied to absolute values
    np.testing.assert_allclose(S, capsconv.conv_fwd(np.abs(I), np.abs(K), 2, 1), rtol=1e-12)
    assert np.all(S + 1e-12 >= np.abs(O))


@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 1), (2, 2)])
def test_abs_sum_closed_form(stride, pad):
    """The error scale S = sum |I*K| pinned without the oracle on both sides: input all a < 0,
    kernel all b > 0, with alternating signs laid over both so that O cancels but S cannot:
    S = |a*b| * C * D2 * (in-range taps at that pixel) everywhere, and O = 0 where the number of
    terms is even."""
    N, H, W, C, M, kh, kw, D0, D1, D2, D3 = 2, 6, 5, 3, 2, 3, 2, 2, 3, 4, 5
    a, b = -0.75, 1.5
    I = np.full((N, H, W, C, D0, D1, D2), a, np.float32)
    K = np.full((kh, kw, C, M, D0, D2, D3), b, np.float32)
    K[..., 1::2, :] *= -1                       # sign alternates along the contracted index d2
    O, S = capsconv.conv_fwd(I, K, stride=stride, pad=pad, with_abs_sum=True)
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    for x in range(Ho):
        rows = sum(0 <= x * stride - pad + p < H for p in range(kh))
        for y in range(Wo):
            cols = sum(0 <= y * stride - pad + q < W for q in range(kw))
            assert np.all(S[:, x, y] == abs(a * b) * C * D2 * rows * cols), (x, y)
    assert np.all(O == 0.0)                     # D2 is even: every capsule product cancels
    which = np.array([[1, Ho - 1, 0, 1], [0, 0, Wo - 1, 0]], np.int32)
    Os, Ss = capsconv.conv_fwd_subset(I, K, which, stride, pad, with_abs_sum=True)
    assert np.array_equal(Ss[0], S[1, Ho - 1, 0, 1]) and np.array_equal(Ss[1], S[0, 0, Wo - 1, 0])
    assert np.all(Os == 0.0)


def test_rejects_bad_requests():
    I, K = _case(91)
    with pytest.raises(ValueError):
        capsconv.conv_fwd(I, K[:, :, :2])                       # channel mismatch
    with pytest.raises(ValueError):
        capsconv.conv_fwd(I, K, stride=0)
    with pytest.raises(ValueError):
        capsconv.conv_fwd(I[:, :2], K)                          # kernel taller than input
    with pytest.raises(ValueError):
        capsconv.conv_fwd_subset(I, K, np.array([[0, 99, 0, 0]]))
    with pytest.raises(ValueError):
        capsconv.conv_fwd(I.astype(np.float64) + 1e-12, K)      # not representable in float32
