"""GPU parity on layers where many 32-filter tiles read the same channels, and many 32-channel blocks pull from the
same filters (one or two long windows with a hundred filters each; windows that start on every channel with a
handful of filters each, as in a channel-expanding layer) against the fp64 CPU oracle, element by element.
The shapes are sized so that the library's forward and grad-input take the kernels that stage the activation
operand once per workgroup of four tiles (at least 512 workgroups of 128 columns; four consecutive tiles reading at
least three times the channels of their common walk, resp. four channel blocks pulling from three to four times
the filters of their common walk): ragged last column tile, filter counts that leave tile rows and whole tiles of
the last workgroup empty, channel counts that leave the last block and the last workgroup partly empty, walks that
wrap past the last channel or run once around all windows, weight rows that are and are not 16-byte aligned
inside the walk.
Bar: max|gpu - ref| / max|ref| <= 2e-5 (the benchmark spec).
"""
import numpy as np
import pytest
import torch

import scc_workloads as Wk
from oracle import scc_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def S():
    import paper_2101_00745_amd as lib
    assert torch.cuda.is_available(), "these tests need the MI355X"
    lib.load()  # raises if libscc_hip.so is not built: no fallback
    return lib


def rel_err(got, ref):
    denom = float(np.max(np.abs(ref)))
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref))) / (denom if denom else 1.0)


# (N, Cin, Cout, H, W, cg, co)
SHAPES = [
    (37, 96, 200, 30, 30, 1, 0.5),      # 2 windows x 100 filters: 4 tiles per window, last one 4 rows; 20 columns in the last tile
    (17, 120, 500, 32, 32, 2, 0.33),    # 120 windows (every channel) x 5 filters: 30 banded tiles, last workgroup holds 2
    (9, 128, 520, 50, 40, 2, 0.34),     # 128 windows x 5 filters, 80 columns in the last tile
    (40, 80, 330, 22, 22, 1, 0.3),      # 10 windows, 8 channels apart, x 33 filters: second tile of a window has one row
]


# grad-input, (N, Cin, Cout, H, W, cg, co)
SHAPES_GRAD_INPUT = [
    (34, 120, 250, 44, 44, 1, 0.5),     # 2 windows x 125 filters; the last channel block has 24 channels; 32 columns in the last tile
    (33, 104, 400, 46, 44, 1, 0.3),     # 104 windows (every channel) x 4 filters, 16 of them missing: the walk is once around the circle
    (18, 224, 448, 44, 44, 1, 0.52),    # 56 windows, 4 channels apart; 7 channel blocks: the second workgroup of a column tile holds 3
]


def make(cfg):
    N, Cin, Cout, H, W, cg, co = cfg
    layer = Wk.Layer("shared_n%d_c%dto%d_%dx%d_cg%d" % (N, Cin, Cout, H, W, cg), 9, N=N, Cin=Cin, Cout=Cout, H=H, W=W, cg=cg,
                     co=co, layer=(SHAPES + SHAPES_GRAD_INPUT).index(cfg))
    return Wk.make_inputs(layer)


@pytest.mark.parametrize("cfg", SHAPES)
def test_forward_every_element(S, cfg):
    N, Cin, Cout, H, W, cg, co = cfg
    x, w, _ = make(cfg)
    y = S.scc_forward(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), cg, co)
    torch.cuda.synchronize()
    assert rel_err(y.cpu().numpy(), O.forward(x, w, cg, co)) <= 2e-5


def test_forward_writes_every_element_and_nothing_else(S):
    cfg = SHAPES[0]
    N, Cin, Cout, H, W, cg, co = cfg
    x, w, _ = make(cfg)
    n = N * Cout * H * W
    buf = torch.full((n + 256,), float("nan"), device="cuda")
    out = buf[:n].view(N, Cout, H, W)
    S.scc_forward(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), cg, co, out=out)
    torch.cuda.synchronize()
    assert not torch.isnan(out).any() and torch.isnan(buf[n:]).all()


def test_forward_twice_is_bitwise_equal(S):
    cfg = SHAPES[1]
    N, Cin, Cout, H, W, cg, co = cfg
    x, w, _ = make(cfg)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    a = S.scc_forward(xd, wd, cg, co)
    b = S.scc_forward(xd, wd, cg, co)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_zero_weight_windows_give_exact_zeros(S):
    """Filters whose weights are all zero give exactly zero whatever finite values their neighbours in the tile
    and in the workgroup's walk read."""
    cfg = SHAPES[2]
    N, Cin, Cout, H, W, cg, co = cfg
    x, w, _ = make(cfg)
    w = w.copy()
    w[1::3] = 0.0
    y = S.scc_forward(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), cg, co)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    assert np.all(got[:, 1::3] == 0.0)
    assert rel_err(got, O.forward(x, w, cg, co)) <= 2e-5


@pytest.mark.parametrize("cfg", SHAPES_GRAD_INPUT)
def test_grad_input_every_element(S, cfg):
    N, Cin, Cout, H, W, cg, co = cfg
    _, w, dy = make(cfg)
    n = N * Cin * H * W
    buf = torch.full((n + 256,), float("nan"), device="cuda")
    out = buf[:n].view(N, Cin, H, W)
    S.scc_backward_input(torch.from_numpy(dy).cuda(), torch.from_numpy(w).cuda(), Cin, cg, co, out=out)
    torch.cuda.synchronize()
    assert not torch.isnan(out).any() and torch.isnan(buf[n:]).all()      # every element written, nothing past the end
    assert rel_err(out.cpu().numpy(), O.backward_input(dy, w, Cin, cg, co)) <= 2e-5


def test_grad_input_twice_is_bitwise_equal(S):
    cfg = SHAPES_GRAD_INPUT[1]
    N, Cin, Cout, H, W, cg, co = cfg
    _, w, dy = make(cfg)
    dyd, wd = torch.from_numpy(dy).cuda(), torch.from_numpy(w).cuda()
    a = S.scc_backward_input(dyd, wd, Cin, cg, co)
    b = S.scc_backward_input(dyd, wd, Cin, cg, co)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_grad_input_of_zero_weight_filters_is_exact(S):
    """With every weight zero except one filter's, dx is exactly zero outside that filter's window whatever finite
    values dy holds, and matches the oracle inside."""
    cfg = SHAPES_GRAD_INPUT[2]
    N, Cin, Cout, H, W, cg, co = cfg
    _, w, dy = make(cfg)
    keep = 37
    w2 = np.zeros_like(w)
    w2[keep] = w[keep]
    dx = S.scc_backward_input(torch.from_numpy(dy).cuda(), torch.from_numpy(w2).cuda(), Cin, cg, co)
    torch.cuda.synchronize()
    got = dx.cpu().numpy()
    ref = O.backward_input(dy, w2, Cin, cg, co)
    assert np.all(got[ref == 0.0] == 0.0)
    assert rel_err(got, ref) <= 2e-5
