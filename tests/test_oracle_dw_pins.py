"""Pins for the oracle's depthwise 3x3 stage (Eq. 2 of the paper), its two gradients, and the DW + SCC block's
forward.

The oracle is checked against what Eq. 2 and the mathematics fix, never against itself and never
against the GPU path: a library grouped convolution, one-tap filters that must be pure shifts, the
number of taps that fall inside the map at corners, edges and interior, a dense matrix assembled tap
by tap with separate index code, and a hand-computed 3x3 example.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import scc_oracle as O

SHAPES = [(2, 3, 5, 7), (1, 4, 8, 8), (3, 2, 1, 1), (2, 5, 2, 9), (1, 1, 3, 3), (2, 2, 4, 6)]


def draw(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


@pytest.mark.parametrize("stride", [1, 2, 3])
@pytest.mark.parametrize("shape", SHAPES)
def test_equals_library_grouped_convolution(shape, stride):
    """Eq. 2 is a convolution with as many groups as channels (Section 2.2 calls DW the extreme case of GC):
    torch's conv2d with groups=C, padding 1 and no flip computes it in fp64."""
    N, C, H, W = shape
    x, k = draw(shape, 1), draw((C, 3, 3), 2)
    ref = F.conv2d(torch.from_numpy(x), torch.from_numpy(k).reshape(C, 1, 3, 3), stride=stride, padding=1, groups=C).numpy()
    got = O.depthwise3x3(x, k, stride)
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() <= 1e-13 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("i,j", list(itertools.product(range(3), range(3))))
def test_single_tap_is_a_shift(i, j):
    """A filter whose only non-zero tap is (i, j) copies pixel (m+i-1, n+j-1) to (m, n), zero past the border:
    fixes the orientation of the filter (no flip, rows before columns) and the centring."""
    x = draw((2, 3, 6, 5), 3)
    k = np.zeros((3, 3, 3))
    k[:, i, j] = [1.0, -2.0, 0.5]
    z = O.depthwise3x3(x, k, 1)
    want = np.zeros_like(x)
    for m in range(6):
        for n in range(5):
            r, c = m + i - 1, n + j - 1
            if 0 <= r < 6 and 0 <= c < 5:
                want[:, :, m, n] = x[:, :, r, c]
    want *= np.array([1.0, -2.0, 0.5]).reshape(1, 3, 1, 1)
    assert np.array_equal(z, want)


def test_centre_tap_with_stride_subsamples():
    """Only the centre tap set: output (m, n) is input (s*m, s*n), and there are floor((H-1)/s)+1 rows."""
    x = draw((1, 2, 7, 10), 4)
    k = np.zeros((2, 3, 3))
    k[:, 1, 1] = 1.0
    for s in (1, 2, 3, 4):
        z = O.depthwise3x3(x, k, s)
        assert z.shape == (1, 2, (7 - 1) // s + 1, (10 - 1) // s + 1)
        assert np.array_equal(z, x[:, :, ::s, ::s])


def test_tap_counts_at_the_border():
    """All-ones filter on an all-ones map counts the taps inside the map: 4 at corners, 6 on edges, 9 inside."""
    z = O.depthwise3x3(np.ones((1, 1, 5, 6)), np.ones((1, 3, 3)), 1)[0, 0]
    want = np.full((5, 6), 9.0)
    want[0, :] = want[-1, :] = want[:, 0] = want[:, -1] = 6.0
    want[0, 0] = want[0, -1] = want[-1, 0] = want[-1, -1] = 4.0
    assert np.array_equal(z, want)
    # stride 2 on an even map: the last output row is centred on row H-2, so only the first row/column lose taps
    z2 = O.depthwise3x3(np.ones((1, 1, 4, 4)), np.ones((1, 3, 3)), 2)[0, 0]
    assert np.array_equal(z2, np.array([[4.0, 6.0], [6.0, 9.0]]))


def test_hand_computed_example():
    """3x3 map 1..9, filter taps 1..9: the centre output is sum t*t = 285; the top-left one uses taps 5,6,8,9 on
    pixels 1,2,4,5 = 5+12+32+45 = 94; the bottom-right one taps 1,2,4,5 on pixels 5,6,8,9 = 5+12+32+45 = 94."""
    x = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    k = np.arange(1.0, 10.0).reshape(1, 3, 3)
    z = O.depthwise3x3(x, k, 1)[0, 0]
    assert z[1, 1] == 285.0 and z[0, 0] == 94.0 and z[2, 2] == 94.0
    # top-right: taps (1,0),(1,1),(2,0),(2,1) = 4,5,7,8 on pixels 2,3,5,6 = 8+15+35+48
    assert z[0, 2] == 106.0


@pytest.mark.parametrize("stride", [1, 2])
def test_dense_matrix_built_tap_by_tap(stride):
    """z = D x with D assembled from Eq. 2 one tap at a time (separate index code), channels never mixing."""
    N, C, H, W = 1, 3, 5, 4
    x, k = draw((N, C, H, W), 5), draw((C, 3, 3), 6)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    D = np.zeros((C * Ho * Wo, C * H * W))
    for a, m, n, i, j in itertools.product(range(C), range(Ho), range(Wo), range(3), range(3)):
        r, c = stride * m + i - 1, stride * n + j - 1
        if 0 <= r < H and 0 <= c < W:
            D[(a * Ho + m) * Wo + n, (a * H + r) * W + c] += k[a, i, j]
    want = (D @ x.reshape(-1)).reshape(1, C, Ho, Wo)
    assert np.abs(O.depthwise3x3(x, k, stride) - want).max() <= 1e-13
    # a channel's output depends on that channel only
    x2 = x.copy()
    x2[:, 1] += 1.0
    z1, z2 = O.depthwise3x3(x, k, stride), O.depthwise3x3(x2, k, stride)
    assert np.array_equal(z1[:, [0, 2]], z2[:, [0, 2]]) and not np.array_equal(z1[:, 1], z2[:, 1])


def test_linear_in_filter_and_in_input():
    x, y = draw((2, 3, 4, 5), 7), draw((2, 3, 4, 5), 8)
    k, h = draw((3, 3, 3), 9), draw((3, 3, 3), 10)
    a = O.depthwise3x3(2.0 * x - y, k, 2)
    b = 2.0 * O.depthwise3x3(x, k, 2) - O.depthwise3x3(y, k, 2)
    assert np.abs(a - b).max() <= 1e-13
    a = O.depthwise3x3(x, k + 3.0 * h, 1)
    b = O.depthwise3x3(x, k, 1) + 3.0 * O.depthwise3x3(x, h, 1)
    assert np.abs(a - b).max() <= 1e-13


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("cfg", [(8, 12, 2, 0.5), (12, 8, 3, 1.0 / 3.0), (16, 16, 4, 0.5), (6, 10, 1, 0.5)])
def test_block_forward_equals_library_composition(cfg, stride):
    """DW + SCC block (Section 3.1: SCC takes the place of PW after DW): a library depthwise convolution followed by
    the channel-stack composition of Section 4.1 (gather each filter's window, multiply, sum) in torch fp64."""
    Cin, Cout, cg, co = cfg
    L = Cin // cg
    x, k, w = draw((2, Cin, 6, 5), 11), draw((Cin, 3, 3), 12), draw((Cout, L), 13)
    z = F.conv2d(torch.from_numpy(x), torch.from_numpy(k).reshape(Cin, 1, 3, 3), stride=stride, padding=1, groups=Cin)
    step = L - int(co * L)
    idx = torch.tensor([[(f * step + j) % Cin for j in range(L)] for f in range(Cout)])
    ref = torch.einsum("nfjhw,fj->nfhw", z[:, idx], torch.from_numpy(w)).numpy()
    got = O.depthwise_scc_forward(x, k, w, cg, co, stride)
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        O.depthwise_out(0, 1)
    with pytest.raises(ValueError):
        O.depthwise_out(4, 0)
    with pytest.raises(AssertionError):
        O.depthwise3x3(np.zeros((1, 2, 3, 3)), np.zeros((3, 3, 3)))


# ----------------------------------------------------------------------------------------------------------
# the two gradients of the depthwise stage
@pytest.mark.parametrize("stride", [1, 2, 3])
@pytest.mark.parametrize("shape", SHAPES)
def test_gradients_equal_library_autograd(shape, stride):
    """torch differentiates its own grouped convolution (fp64): both gradients must agree with it."""
    N, C, H, W = shape
    x = torch.from_numpy(draw(shape, 21)).requires_grad_(True)
    k = torch.from_numpy(draw((C, 3, 3), 22)).requires_grad_(True)
    z = F.conv2d(x, k.reshape(C, 1, 3, 3), stride=stride, padding=1, groups=C)
    dz = draw(tuple(z.shape), 23)
    z.backward(torch.from_numpy(dz))
    dx, dk = O.depthwise3x3_backward(x.detach().numpy(), k.detach().numpy(), dz, stride)
    assert np.abs(dx - x.grad.numpy()).max() <= 1e-12 * max(1.0, np.abs(x.grad.numpy()).max())
    assert np.abs(dk - k.grad.numpy()).max() <= 1e-12 * max(1.0, np.abs(k.grad.numpy()).max())


@pytest.mark.parametrize("stride", [1, 2])
def test_grad_input_is_the_transposed_dense_matrix(stride):
    """With z = D x (D assembled tap by tap from Eq. 2, separate index code), dx = D^T dz."""
    N, C, H, W = 1, 2, 5, 4
    x, k = draw((N, C, H, W), 24), draw((C, 3, 3), 25)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    D = np.zeros((C * Ho * Wo, C * H * W))
    for a, m, n, i, j in itertools.product(range(C), range(Ho), range(Wo), range(3), range(3)):
        r, c = stride * m + i - 1, stride * n + j - 1
        if 0 <= r < H and 0 <= c < W:
            D[(a * Ho + m) * Wo + n, (a * H + r) * W + c] += k[a, i, j]
    dz = draw((N, C, Ho, Wo), 26)
    dx, _ = O.depthwise3x3_backward(x, k, dz, stride)
    assert np.abs(dx.reshape(-1) - D.T @ dz.reshape(-1)).max() <= 1e-13


@pytest.mark.parametrize("stride", [1, 2])
def test_adjoint_identities(stride):
    """<dz, DW(x; k)> = <dx, x> = <dk, k>: the stage is linear in x and in k, so both gradients pair back to it."""
    x, k = draw((3, 4, 6, 7), 27), draw((4, 3, 3), 28)
    z = O.depthwise3x3(x, k, stride)
    dz = draw(z.shape, 29)
    dx, dk = O.depthwise3x3_backward(x, k, dz, stride)
    lhs = float((dz * z).sum())
    assert abs(lhs - float((dx * x).sum())) <= 1e-10 * abs(lhs)
    assert abs(lhs - float((dk * k).sum())) <= 1e-10 * abs(lhs)


def test_gradients_by_central_differences():
    x, k = draw((2, 2, 4, 5), 30), draw((2, 3, 3), 31)
    dz = draw(O.depthwise3x3(x, k, 2).shape, 32)
    dx, dk = O.depthwise3x3_backward(x, k, dz, 2)
    loss = lambda xx, kk: float((O.depthwise3x3(xx, kk, 2) * dz).sum())
    h = 1e-5
    for idx in [(0, 0, 0, 0), (1, 1, 3, 4), (0, 1, 2, 2)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        assert abs((loss(xp, k) - loss(xm, k)) / (2 * h) - dx[idx]) <= 1e-8
    for idx in [(0, 0, 0), (1, 2, 2), (0, 1, 2)]:
        kp, km = k.copy(), k.copy()
        kp[idx] += h
        km[idx] -= h
        assert abs((loss(x, kp) - loss(x, km)) / (2 * h) - dk[idx]) <= 1e-8


def test_grad_of_single_tap_filter_is_the_opposite_shift():
    """Tap (i, j) alone moves pixel (m+i-1, n+j-1) to (m, n); its grad-input moves dz(m, n) back to (m+i-1, n+j-1)."""
    dz = draw((1, 1, 5, 6), 33)
    for i, j in itertools.product(range(3), range(3)):
        k = np.zeros((1, 3, 3))
        k[0, i, j] = 1.0
        dx, dk = O.depthwise3x3_backward(np.zeros((1, 1, 5, 6)), k, dz, 1)
        want = np.zeros((5, 6))
        for m in range(5):
            for n in range(6):
                r, c = m + i - 1, n + j - 1
                if 0 <= r < 5 and 0 <= c < 6:
                    want[r, c] = dz[0, 0, m, n]
        assert np.array_equal(dx[0, 0], want) and not dk.any()
