"""GPU parity of scc_backward (both gradients in one call) against the fp64 CPU oracle.

Layers the fused kernel takes (fp32, windows of 64 channels starting on multiples of 32, at most 32 filters per
window, H*W a multiple of 4) and layers it declines, which run the two passes one after the other: the results
are held to the same bar either way, max|gpu - ref| / max|ref| <= 2e-5 (fp32) and 1e-2 (bf16 dx; dw is fp32 sums
of exact products of the same bf16 values in both dtypes and meets 2e-5).
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
    lib.load()
    return lib


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    denom = float(np.max(np.abs(ref)))
    return float(np.max(np.abs(got - ref))) / denom if denom else float(np.max(np.abs(got)))


def small(name, N, Cin, Cout, H, W, cg, co, **kw):
    return Wk.Layer(name, 11, N=N, Cin=Cin, Cout=Cout, H=H, W=W, cg=cg, co=co, **kw)


def check(S, layer, dtype=torch.float32, seed_offset=0):
    x, w, dy = Wk.make_inputs(layer, seed_offset)
    xd, wd, dyd = (torch.from_numpy(a).to(dtype).cuda() for a in (x, w, dy))
    xr, wr, dyr = (t.float().cpu().numpy() for t in (xd, wd, dyd))     # exactly the values the GPU sees
    dx, dw = S.scc_backward(xd, dyd, wd, layer.cg, layer.co)
    torch.cuda.synchronize()
    assert dx.shape == xd.shape and dx.dtype == dtype and dw.shape == (layer.Cout, layer.L) and dw.dtype == torch.float32
    e_dx = rel_err(dx.float().cpu().numpy(), O.backward_input(dyr, wr, layer.Cin, layer.cg, layer.co))
    e_dw = rel_err(dw.cpu().numpy(), O.backward_weight(xr, dyr, layer.cg, layer.co))
    assert e_dx <= (2e-5 if dtype == torch.float32 else 1e-2), (layer.name, "dx", e_dx)
    assert e_dw <= 2e-5, (layer.name, "dw", e_dw)
    return e_dx, e_dw


# the fused kernel's family: L = 64, stride 32 (cg = Cin/64, co = 0.5), Cout <= Cin
FUSED = [
    small("f_256_16x16", 4, 256, 256, 16, 16, 4, 0.5),
    small("f_two_windows", 9, 64, 64, 8, 8, 1, 0.5),                  # P = 2: windows b-1 and b are the only two
    small("f_ragged_cols", 5, 128, 128, 6, 6, 2, 0.5),                # 180 columns: last chunks partly empty
    small("f_14x14", 3, 512, 512, 14, 14, 8, 0.5, x_law="halfnormal"),
    small("f_missing_filters", 6, 128, 100, 10, 10, 2, 0.5),          # 25 filters per window: tile rows without a filter
    small("f_few_filters", 7, 192, 30, 8, 8, 3, 0.5),                 # 5 filters per window
    small("f_one_sample_big_plane", 1, 128, 128, 32, 32, 2, 0.5),
    small("f_many_samples_2x2", 200, 128, 128, 2, 2, 2, 0.5),         # planes of 4 columns: a chunk spans 8 samples
]
# declined by the fused kernel: overlap 0 / 0.25, long or short windows, odd planes, more than 32 filters per window
OTHER = [
    small("o_co0", 4, 256, 256, 8, 8, 4, 0.0),
    small("o_co25", 4, 256, 256, 8, 8, 4, 0.25),
    small("o_l128", 4, 256, 128, 8, 8, 2, 0.5),
    small("o_odd_plane", 4, 128, 128, 7, 7, 2, 0.5),
    small("o_64_filters_per_window", 4, 128, 256, 8, 8, 2, 0.5),
    small("o_tiny", 1, 4, 4, 1, 1, 2, 0.5),
]


@pytest.mark.parametrize("layer", FUSED + OTHER, ids=lambda l: l.name)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_backward_small_shapes(S, layer, dtype):
    check(S, layer, dtype)


@pytest.mark.parametrize("layer", [Wk.METRIC, Wk.LATE, Wk.STACK[2], Wk.BATCH_SWEEP[0], Wk.BATCH_SWEEP[4]],
                         ids=lambda l: l.name)
def test_backward_full_size_layers(S, layer):
    # full sizes, in the launch configuration the benchmark times; the error stays at fp32 rounding level
    e_dx, e_dw = check(S, layer)
    assert max(e_dx, e_dw) <= 2e-6


@pytest.mark.parametrize("layer", [Wk.METRIC_SWEEP[0], Wk.METRIC_SWEEP[3], Wk.STACK[0], Wk.STACK[6]], ids=lambda l: l.name)
def test_backward_full_size_layers_two_passes(S, layer):
    check(S, layer)


def test_backward_matches_the_separate_passes_and_repeats_bitwise(S):
    for layer in (Wk.METRIC, small("f_ragged_cols", 5, 128, 128, 6, 6, 2, 0.5)):
        x, w, dy = Wk.make_inputs(layer)
        xd, wd, dyd = (torch.from_numpy(a).cuda() for a in (x, w, dy))
        dx1, dw1 = S.scc_backward(xd, dyd, wd, layer.cg, layer.co)
        dx2, dw2 = S.scc_backward(xd, dyd, wd, layer.cg, layer.co)
        assert torch.equal(dx1, dx2) and torch.equal(dw1, dw2)
        dxs = S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co)
        dws = S.scc_backward_weight(xd, dyd, layer.cg, layer.co)
        scale_x, scale_w = float(dxs.abs().max()), float(dws.abs().max())
        assert float((dx1 - dxs).abs().max()) <= 2e-5 * scale_x
        assert float((dw1 - dws).abs().max()) <= 2e-5 * scale_w


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("layer", OTHER[:5] + [Wk.STACK[6], Wk.STACK[11], Wk.METRIC_SWEEP[1]], ids=lambda l: l.name)
def test_one_launch_for_both_passes_is_bitwise_the_separate_passes(S, layer, dtype):
    """Layers the fused kernel declines run the grad-weight and grad-input kernels as two ranges of one grid: same
    tiles, same arithmetic, same summation order, so dx equals that of the separate entry point bit for bit, and so
    does dw, except on layers whose columns the separate pass splits two ways: there the merged launch does not
    split them (one summation chain instead of two), and dw agrees to rounding."""
    x, w, dy = Wk.make_inputs(layer)
    xd, wd, dyd = (torch.from_numpy(a).to(dtype).cuda() for a in (x, w, dy))
    dx1, dw1 = S.scc_backward(xd, dyd, wd, layer.cg, layer.co)
    dx2, dw2 = S.scc_backward(xd, dyd, wd, layer.cg, layer.co)
    dxs = S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co)
    dws = S.scc_backward_weight(xd, dyd, layer.cg, layer.co)
    torch.cuda.synchronize()
    assert torch.equal(dx1, dxs) and torch.equal(dx1, dx2) and torch.equal(dw1, dw2)
    assert torch.equal(dw1, dws) or float((dw1 - dws).abs().max()) <= 2e-6 * float(dws.abs().max())


def test_backward_outputs_overwritten_and_workspace_contents_do_not_matter(S):
    layer = small("f_256_16x16", 4, 256, 256, 16, 16, 4, 0.5)
    x, w, dy = Wk.make_inputs(layer)
    xd, wd, dyd = (torch.from_numpy(a).cuda() for a in (x, w, dy))
    dx0, dw0 = S.scc_backward(xd, dyd, wd, layer.cg, layer.co)
    need = S.scc_backward_workspace_bytes(layer.N, layer.Cin, layer.Cout, layer.H, layer.W, layer.cg, layer.co)
    ws = torch.full((max(need, 4) // 4,), float("nan"), dtype=torch.float32, device="cuda").view(torch.uint8)
    dx1 = torch.full_like(dx0, float("nan"))
    dw1 = torch.full_like(dw0, 1e30)
    S.scc_backward(xd, dyd, wd, layer.cg, layer.co, out_dx=dx1, out_dw=dw1, workspace=ws)
    assert torch.equal(dx0, dx1) and torch.equal(dw0, dw1)
