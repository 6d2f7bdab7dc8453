"""Pins for the CPU oracle: it is checked against what the paper and the mathematics fix,
never against itself and never against the GPU path.

Each test names the passage or identity it rests on.  The independent index code used
here (``paper_windows``, ``dense_matrix``) is written separately from the oracle's.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import scc_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------------------
# independent index generators
# ----------------------------------------------------------------------------------------
def paper_windows(Cin, Cout, cg, co):
    """Window starts as Algorithm 1 and Algorithm 2 define them, restated in a form of its own (and a
    different one from the oracle's): a window begins where the previous one ended, stepped back by the
    overlap in channels; positions are reduced modulo Cin; the list of distinct windows ends at the first
    start that has been seen before (its length is the cyclic distance), and filter k takes window
    k mod distance.  A window is identified by where it starts: for cg = 1 the pair (start, end) of
    Algorithm 1 would tell (0, Cin) and (0, 0) apart although they are the same window.
    Returns (starts, distance)."""
    width = Cin // cg
    back = int(co * width)
    cycle, pos = [], 0
    while len(cycle) < Cout and pos % Cin not in cycle:
        cycle.append(pos % Cin)
        pos = pos + width - back          # end of this window, minus the overlap
    return [cycle[k % len(cycle)] for k in range(Cout)], len(cycle)


def window_channels(Cin, Cout, cg, co):
    st, _ = paper_windows(Cin, Cout, cg, co)
    gw = Cin // cg
    return [[(s + j) % Cin for j in range(gw)] for s in st]


def dense_matrix(w, Cin, cg, co):
    """A[k, c] such that y = A @ x per pixel, filled entry by entry."""
    Cout, L = w.shape
    A = np.zeros((Cout, Cin))
    for k, chans in enumerate(window_channels(Cin, Cout, cg, co)):
        for j, c in enumerate(chans):
            A[k, c] += w[k, j]
    return A


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


SHAPES = [  # (N, Cin, Cout, H, W, cg, co)
    (2, 4, 4, 2, 3, 2, 0.5),
    (2, 6, 5, 1, 3, 2, 1.0 / 3.0),
    (1, 6, 7, 2, 2, 3, 0.5),
    (2, 8, 3, 3, 1, 2, 0.25),      # Cout smaller than the period
    (1, 12, 30, 2, 2, 3, 0.75),    # several cycles, partial last cycle
    (2, 16, 16, 3, 3, 4, 0.0),
    (1, 16, 24, 2, 2, 1, 0.3),     # one group, rotated full windows
    (1, 10, 9, 1, 5, 2, 1.0),      # 100% overlap: all filters share one window
    (1, 128, 20, 1, 2, 2, 0.33),   # stride 43 coprime to Cin, many wraps
    (2, 32, 32, 4, 4, 2, 0.5),
]


# ----------------------------------------------------------------------------------------
# O1: the worked example the paper prints
# ----------------------------------------------------------------------------------------
def _read_golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = [t.strip() for t in line.split("=")]
        out[k] = v
    return out


def test_worked_example_windows_and_gradient_sources():
    g = _read_golden("worked_example_cin4_cg2_co50.txt")
    Cin, cg, co = int(g["Cin"]), int(g["cg"]), float(g["co"])
    st = O.starts(Cin, 4, cg, co)
    L, _ = O.window(Cin, cg, co)
    for k in range(4):
        want = [int(t) for t in g["window[%d]" % k].split()]
        assert [(int(st[k]) + j) % Cin for j in range(L)] == want
    # cyclic distance: first filter index at which a window repeats
    st_long = O.starts(Cin, 12, cg, co)
    dist = next(k for k in range(1, 12) if st_long[k] == st_long[0])
    assert dist == int(g["cyclic_distance"])
    # grad-input on channel 3 draws on dy channels 2 and 3 only: probe with one-hot dy
    w = np.ones((4, L))
    srcs = []
    for k in range(4):
        dy = np.zeros((1, 4, 1, 1))
        dy[0, k] = 1.0
        if O.backward_input(dy, w, Cin, cg, co)[0, 3, 0, 0] != 0.0:
            srcs.append(k)
    assert srcs == [int(t) for t in g["grad_input_sources[3]"].split()]
    # and the forward really reads those channels: one-hot x
    for k in range(4):
        want = sorted(int(t) for t in g["window[%d]" % k].split())
        got = []
        for c in range(4):
            x = np.zeros((1, 4, 1, 1))
            x[0, c] = 1.0
            if O.forward(x, w, cg, co)[0, k, 0, 0] != 0.0:
                got.append(c)
        assert got == want


# ----------------------------------------------------------------------------------------
# O2: Algorithm 1 + Algorithm 2 as an independent generator of window starts
# ----------------------------------------------------------------------------------------
def test_starts_match_algorithm_1_and_2():
    rng = np.random.default_rng(7)
    cases = [(s[1], s[2], s[5], s[6]) for s in SHAPES]
    for _ in range(200):
        cg = int(rng.integers(1, 9))
        Cin = cg * int(rng.integers(1, 40))
        Cout = int(rng.integers(1, 100))
        co = float(rng.choice([0.0, 0.1, 0.25, 1 / 3, 0.33, 0.5, 0.66, 0.75, 0.9, 1.0, rng.random()]))
        cases.append((Cin, Cout, cg, co))
    for Cin, Cout, cg, co in cases:
        want, dist = paper_windows(Cin, Cout, cg, co)
        assert list(O.starts(Cin, Cout, cg, co)) == want, (Cin, Cout, cg, co)
        L, ov = O.window(Cin, cg, co)
        assert L == Cin // cg and ov == int(co * (Cin // cg))
        stride = (L - ov) % Cin
        period = Cin // math.gcd(stride, Cin) if stride else 1
        assert dist == min(Cout, period)


def test_cyclic_patterns_stated_in_the_paper():
    # Section 4.2: cg=2, co=50% -> every four filters share a window, whatever Cin (multiple of 4)
    for Cin in (4, 8, 32, 64, 256, 1024):
        st = O.starts(Cin, 16, 2, 0.5)
        assert all(st[k] == st[k + 4] for k in range(12)) and len(set(st[:4].tolist())) == 4
    # same passage: with one third overlap every three filters share a window
    # (holds when co*L is exactly L/3; 1/3 * 3 == 1.0 in binary floating point)
    st = O.starts(6, 9, 2, 1.0 / 3.0)
    assert all(st[k] == st[k + 3] for k in range(6)) and len(set(st[:3].tolist())) == 3
    # Section 3.2 example: Cin=64, Cout=128, cg=2 -> each filter multiplies 32 channels
    assert O.window(64, 2, 0.5)[0] == 32


def test_rejects_non_layers():
    for bad in [(6, 4, 0.5), (0, 1, 0.5), (8, 0, 0.5), (8, 2, -0.1), (8, 2, 1.5), (8, 2, float("nan"))]:
        with pytest.raises(ValueError):
            O.window(*bad)


# ----------------------------------------------------------------------------------------
# O3: one group -> pointwise convolution (Table 1, first footnote), rows rotated by s_k
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("co", [0.0, 1.0, 0.3, 0.5])
def test_one_group_is_pointwise_convolution(co):
    N, Cin, Cout, H, W = 2, 12, 7, 3, 2
    x, w, dy = rand((N, Cin, H, W), 1), rand((Cout, Cin), 2), rand((N, Cout, H, W), 3)
    st, _ = paper_windows(Cin, Cout, 1, co)
    wpw = np.zeros((Cout, Cin))
    for k in range(Cout):
        for j in range(Cin):
            wpw[k, (st[k] + j) % Cin] = w[k, j]
    if co in (0.0, 1.0):
        assert np.array_equal(wpw, w)          # identity rotation: plain PW with the same matrix
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(wpw.reshape(Cout, Cin, 1, 1), requires_grad=True)
    yt = F.conv2d(xt, wt)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(O.forward(x, w, 1, co), yt.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.backward_input(dy, w, Cin, 1, co), xt.grad.numpy(), rtol=0, atol=1e-12)
    dwpw = wt.grad.numpy().reshape(Cout, Cin)
    dw_want = np.array([[dwpw[k, (st[k] + j) % Cin] for j in range(Cin)] for k in range(Cout)])
    np.testing.assert_allclose(O.backward_weight(x, dy, 1, co), dw_want, rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------------------
# O4: zero overlap -> group pointwise convolution (Table 1, second footnote).
# Algorithm 1 hands filter k the group k mod cg; the library's grouped convolution hands
# output channel o the group o // (Cout/cg): equal after that permutation.
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("cg,Cin,Cout", [(2, 8, 6), (4, 16, 8), (3, 9, 12), (8, 64, 64)])
def test_zero_overlap_is_group_convolution(cg, Cin, Cout):
    N, H, W = 2, 2, 3
    L = Cin // cg
    x, w, dy = rand((N, Cin, H, W), 4), rand((Cout, L), 5), rand((N, Cout, H, W), 6)
    per = Cout // cg
    perm = [(k % cg) * per + k // cg for k in range(Cout)]      # SCC filter k -> library channel
    inv = np.argsort(perm)                                       # library channel -> SCC filter
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w[inv].reshape(Cout, L, 1, 1), requires_grad=True)
    yt = F.conv2d(xt, wt, groups=cg)
    yt.backward(torch.tensor(dy[:, inv]))
    np.testing.assert_allclose(O.forward(x, w, cg, 0.0), yt.detach().numpy()[:, perm], rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.backward_input(dy, w, Cin, cg, 0.0), xt.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.backward_weight(x, dy, cg, 0.0),
                               wt.grad.numpy().reshape(Cout, L)[perm], rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------------------
# O5: the channel-stack composition (Section 4.1): slice each filter's window, concatenate
# along channels, grouped convolution with groups = Cout; autograd gives both gradients.
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", SHAPES)
def test_channel_stack_composition(shape):
    N, Cin, Cout, H, W, cg, co = shape
    L = Cin // cg
    x, w, dy = rand((N, Cin, H, W), 10), rand((Cout, L), 11), rand((N, Cout, H, W), 12)
    idx = torch.tensor(list(itertools.chain.from_iterable(window_channels(Cin, Cout, cg, co))))
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w.reshape(Cout, L, 1, 1), requires_grad=True)
    stacked = xt.index_select(1, idx)                     # [N, Cout*L, H, W]
    assert stacked.shape[1] == Cout * L                   # Section 3.1: Cout*Cin/cg weights, MACs per pixel
    yt = F.conv2d(stacked, wt, groups=Cout)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(O.forward(x, w, cg, co), yt.detach().numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(O.backward_input(dy, w, Cin, cg, co), xt.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(O.backward_weight(x, dy, cg, co), wt.grad.numpy().reshape(Cout, L),
                               rtol=0, atol=1e-11)


def test_channel_stack_composition_medium_shape():
    N, Cin, Cout, H, W, cg, co = 3, 64, 96, 7, 5, 4, 0.5
    L = Cin // cg
    x, w, dy = rand((N, Cin, H, W), 13), rand((Cout, L), 14), rand((N, Cout, H, W), 15)
    idx = torch.tensor(list(itertools.chain.from_iterable(window_channels(Cin, Cout, cg, co))))
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w.reshape(Cout, L, 1, 1), requires_grad=True)
    yt = F.conv2d(xt.index_select(1, idx), wt, groups=Cout)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(O.forward(x, w, cg, co), yt.detach().numpy(), rtol=0, atol=1e-10)
    np.testing.assert_allclose(O.backward_input(dy, w, Cin, cg, co), xt.grad.numpy(), rtol=0, atol=1e-10)
    np.testing.assert_allclose(O.backward_weight(x, dy, cg, co), wt.grad.numpy().reshape(Cout, L),
                               rtol=0, atol=1e-10)


# ----------------------------------------------------------------------------------------
# O6: dense brute force: y = A x, dx = A^T dy, dw = band of dy x^T
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", SHAPES)
def test_dense_matrix_brute_force(shape):
    N, Cin, Cout, H, W, cg, co = shape
    L = Cin // cg
    x, w, dy = rand((N, Cin, H, W), 20), rand((Cout, L), 21), rand((N, Cout, H, W), 22)
    A = dense_matrix(w, Cin, cg, co)
    assert np.count_nonzero(dense_matrix(np.ones_like(w), Cin, cg, co)) == Cout * L   # nnz = Cout*Cin/cg
    y = np.einsum("kc,nchw->nkhw", A, x)
    dx = np.einsum("kc,nkhw->nchw", A, dy)
    G = np.einsum("nkhw,nchw->kc", dy, x)
    dw = np.array([[G[k, c] for c in chans] for k, chans in enumerate(window_channels(Cin, Cout, cg, co))])
    np.testing.assert_allclose(O.forward(x, w, cg, co), y, rtol=0, atol=1e-11)
    np.testing.assert_allclose(O.backward_input(dy, w, Cin, cg, co), dx, rtol=0, atol=1e-11)
    np.testing.assert_allclose(O.backward_weight(x, dy, cg, co), dw, rtol=0, atol=1e-11)


# ----------------------------------------------------------------------------------------
# O7/O8: bilinearity and the adjoint identity <dy, fwd(x,w)> = <bwdI(dy,w), x> = <bwdW(x,dy), w>
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", SHAPES)
def test_linearity_and_adjoint_identity(shape):
    N, Cin, Cout, H, W, cg, co = shape
    L = Cin // cg
    x1, x2 = rand((N, Cin, H, W), 30), rand((N, Cin, H, W), 31)
    w1, w2 = rand((Cout, L), 32), rand((Cout, L), 33)
    d1, d2 = rand((N, Cout, H, W), 34), rand((N, Cout, H, W), 35)
    a, b = 0.7, -1.9
    np.testing.assert_allclose(O.forward(a * x1 + b * x2, w1, cg, co),
                               a * O.forward(x1, w1, cg, co) + b * O.forward(x2, w1, cg, co), atol=1e-11)
    np.testing.assert_allclose(O.forward(x1, a * w1 + b * w2, cg, co),
                               a * O.forward(x1, w1, cg, co) + b * O.forward(x1, w2, cg, co), atol=1e-11)
    np.testing.assert_allclose(O.backward_input(a * d1 + b * d2, w1, Cin, cg, co),
                               a * O.backward_input(d1, w1, Cin, cg, co) + b * O.backward_input(d2, w1, Cin, cg, co),
                               atol=1e-11)
    np.testing.assert_allclose(O.backward_weight(a * x1 + b * x2, d1, cg, co),
                               a * O.backward_weight(x1, d1, cg, co) + b * O.backward_weight(x2, d1, cg, co),
                               atol=1e-11)
    np.testing.assert_allclose(O.backward_weight(x1, a * d1 + b * d2, cg, co),
                               a * O.backward_weight(x1, d1, cg, co) + b * O.backward_weight(x1, d2, cg, co),
                               atol=1e-11)
    s_fwd = float(np.sum(d1 * O.forward(x1, w1, cg, co)))
    s_dx = float(np.sum(O.backward_input(d1, w1, Cin, cg, co) * x1))
    s_dw = float(np.sum(O.backward_weight(x1, d1, cg, co) * w1))
    scale = abs(s_fwd) + 1.0
    assert abs(s_fwd - s_dx) <= 1e-11 * scale and abs(s_fwd - s_dw) <= 1e-11 * scale


# ----------------------------------------------------------------------------------------
# O9: cyclic channel-shift invariance.  Rotating the input channels by t window steps and
# moving every filter's weights t filters up moves the outputs t filters up.
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("t", [1, 3])
def test_cyclic_channel_shift_invariance(shape, t):
    N, Cin, Cout, H, W, cg, co = shape
    L, ov = Cin // cg, int(co * (Cin // cg))
    stride = L - ov
    if t >= Cout:
        pytest.skip("shift larger than the filter count")
    x, w = rand((N, Cin, H, W), 40), rand((Cout, L), 41)
    xs = np.empty_like(x)
    for c in range(Cin):
        xs[:, c] = x[:, (c - t * stride) % Cin]
    y = O.forward(x, w, cg, co)
    wraps_evenly = (Cout * stride) % Cin == 0
    ws = np.zeros_like(w)
    for k in range(Cout):
        if k + t < Cout:
            ws[k + t] = w[k]
        elif wraps_evenly:
            ws[(k + t) % Cout] = w[k]
    ys = O.forward(xs, ws, cg, co)
    for k in range(Cout):
        if k + t < Cout:
            np.testing.assert_allclose(ys[:, k + t], y[:, k], atol=1e-12)
        elif wraps_evenly:
            np.testing.assert_allclose(ys[:, (k + t) % Cout], y[:, k], atol=1e-12)


# ----------------------------------------------------------------------------------------
# O10: periodicity: equal weights one cyclic distance apart give equal outputs
# ----------------------------------------------------------------------------------------
def test_periodicity_of_outputs():
    for (N, Cin, Cout, H, W, cg, co) in SHAPES:
        _, dist = paper_windows(Cin, 10 * Cin + Cout, cg, co)   # true period (not clipped by Cout)
        if Cout <= dist:
            continue
        L = Cin // cg
        x, w = rand((N, Cin, H, W), 50), rand((Cout, L), 51)
        for k in range(dist, Cout):
            w[k] = w[k - dist]
        y = O.forward(x, w, cg, co)
        for k in range(dist, Cout):
            assert np.array_equal(y[:, k], y[:, k - dist])


# ----------------------------------------------------------------------------------------
# O11: coverage count: with w = 1 and dy = 1, dx counts the filters covering each channel
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", SHAPES)
def test_coverage_count(shape):
    N, Cin, Cout, H, W, cg, co = shape
    L, ov = Cin // cg, int(co * (Cin // cg))
    dx = O.backward_input(np.ones((N, Cout, H, W)), np.ones((Cout, L)), Cin, cg, co)
    count = np.zeros(Cin)
    for chans in window_channels(Cin, Cout, cg, co):
        for c in chans:
            count[c] += 1
    assert np.array_equal(dx, np.broadcast_to(count[None, :, None, None], dx.shape))
    assert count.sum() == Cout * L
    if (Cout * (L - ov)) % Cin == 0 and (L - ov) != 0 and Cout * L % Cin == 0:
        # filters spread evenly over the channel circle: every channel is covered Cout/cg times
        assert np.all(count == Cout * L // Cin)


# ----------------------------------------------------------------------------------------
# O12: central finite differences (the map is bilinear, so they are exact up to rounding)
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("cg,co", [(1, 0.4), (2, 0.5), (2, 0.0), (3, 0.5), (3, 1.0), (6, 0.0)])
def test_finite_differences(cg, co):
    N, Cin, Cout, H, W = 2, 6, 5, 1, 3
    L = Cin // cg
    x, w, r = rand((N, Cin, H, W), 60), rand((Cout, L), 61), rand((N, Cout, H, W), 62)
    f = lambda xx, ww: float(np.sum(r * O.forward(xx, ww, cg, co)))
    dx, dw = O.backward_input(r, w, Cin, cg, co), O.backward_weight(x, r, cg, co)
    h = 1e-3
    for i in np.ndindex(x.shape):
        e = np.zeros_like(x)
        e[i] = h
        assert abs((f(x + e, w) - f(x - e, w)) / (2 * h) - dx[i]) < 1e-9
    for i in np.ndindex(w.shape):
        e = np.zeros_like(w)
        e[i] = h
        assert abs((f(x, w + e) - f(x, w - e)) / (2 * h) - dw[i]) < 1e-9
