"""GPU parity on layers with few columns and long windows (the deep layers of a CNN: 2x2 to 8x8 maps, 64 to 512
channels per window, 32 to 300 filters per window) against the fp64 CPU oracle, element by element: every pass and the
combined backward.  These are the shapes where a tile's contraction is shared by several wavefronts and where a
column tile spans several samples.  Bar: max|gpu - ref| / max|ref| <= 2e-5 (the benchmark spec).
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


# (N, Cin, Cout, H, W, cg, co): ragged last column tile,
# Cout that is not a multiple of the tile or of the number of windows, windows that wrap, one and many windows,
# 32 to 300 filters per window, maps of 2x2 to 8x8 and a 1x4 strip
SHAPES = [
    (128, 512, 512, 4, 4, 2, 0.5), (37, 256, 256, 2, 2, 2, 0.5), (9, 128, 256, 4, 4, 2, 0.5), (5, 64, 200, 2, 6, 2, 0.5),
    (33, 128, 130, 2, 2, 4, 0.5), (3, 96, 96, 8, 8, 3, 0.0), (2, 256, 300, 4, 4, 1, 0.5), (7, 64, 64, 2, 2, 2, 1.0),
    (11, 192, 384, 1, 4, 2, 1.0 / 3.0), (64, 128, 128, 8, 8, 2, 0.5), (2, 1024, 1024, 2, 2, 2, 0.5), (130, 64, 97, 2, 2, 1, 0.25),
    (1, 128, 64, 4, 8, 4, 0.75), (16, 512, 1024, 2, 2, 2, 0.5), (20, 160, 320, 4, 4, 5, 0.5),
]


@pytest.mark.parametrize("cfg", SHAPES)
def test_dense_layers_every_element(S, cfg):
    N, Cin, Cout, H, W, cg, co = cfg
    layer = Wk.Layer("dense_n%d_c%dto%d_%dx%d_cg%d" % (N, Cin, Cout, H, W, cg), 9, N=N, Cin=Cin, Cout=Cout, H=H, W=W, cg=cg,
                     co=co, layer=SHAPES.index(cfg) % 10)
    x, w, dy = Wk.make_inputs(layer)
    xd, wd, dyd = (torch.from_numpy(a).cuda() for a in (x, w, dy))
    y = S.scc_forward(xd, wd, cg, co)
    dx = S.scc_backward_input(dyd, wd, Cin, cg, co)
    dw = S.scc_backward_weight(xd, dyd, cg, co)
    dx2, dw2 = S.scc_backward(xd, dyd, wd, cg, co)
    torch.cuda.synchronize()
    assert rel_err(y.cpu().numpy(), O.forward(x, w, cg, co)) <= 2e-5
    ref_dx, ref_dw = O.backward_input(dy, w, Cin, cg, co), O.backward_weight(x, dy, cg, co)
    assert rel_err(dx.cpu().numpy(), ref_dx) <= 2e-5 and rel_err(dx2.cpu().numpy(), ref_dx) <= 2e-5
    assert rel_err(dw.cpu().numpy(), ref_dw) <= 2e-5 and rel_err(dw2.cpu().numpy(), ref_dw) <= 2e-5


def test_forward_writes_every_element_and_nothing_else(S):
    N, Cin, Cout, H, W, cg, co = 5, 128, 130, 2, 2, 2, 0.5
    layer = Wk.Layer("dense_guard", 9, N=N, Cin=Cin, Cout=Cout, H=H, W=W, cg=cg, co=co)
    x, w, _ = Wk.make_inputs(layer)
    n = N * Cout * H * W
    buf = torch.full((n + 64,), float("nan"), device="cuda")
    out = buf[:n].view(N, Cout, H, W)
    S.scc_forward(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), cg, co, out=out)
    torch.cuda.synchronize()
    assert not torch.isnan(out).any() and torch.isnan(buf[n:]).all()
    assert rel_err(out.cpu().numpy(), O.forward(x, w, cg, co)) <= 2e-5
