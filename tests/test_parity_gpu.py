"""GPU parity: the HIP library (through its C ABI binding) against the fp64 CPU oracle,
element by element on identical seeded inputs.

Bar (written here, from the benchmark spec): max|gpu - ref| / max|ref| <= 2e-5 for
fp32 tensors and <= 1e-2 for bf16 tensors.  bf16 inputs are rounded to bf16 once, on the
host, and both sides consume those rounded values.  dw is binary32 in both dtypes: sums of
exact products of the values both sides see, so it is held to 2e-5 for bf16 inputs too.
"""
import dataclasses

import numpy as np
import pytest
import torch

import scc_workloads as Wk
from oracle import scc_oracle as O

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 2e-5, torch.bfloat16: 1e-2}


@pytest.fixture(scope="module")
def S():
    import paper_2101_00745_amd as lib
    assert torch.cuda.is_available(), "these tests need the MI355X"
    lib.load()  # raises if libscc_hip.so is not built: no fallback
    return lib


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    denom = float(np.max(np.abs(ref)))
    if denom == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref))) / denom


def to_dev(a, dtype):
    return torch.from_numpy(a).to(dtype).cuda()


def host(t):
    return t.float().cpu().numpy()


def host64(t):
    return t.double().cpu().numpy()


def check_layer(S, layer, dtype=torch.float32, seed_offset=0, passes=("fwd", "bwi", "bww")):
    x, w, dy = Wk.make_inputs(layer, seed_offset)
    xd, wd, dyd = to_dev(x, dtype), to_dev(w, dtype), to_dev(dy, dtype)
    xr, wr, dyr = host(xd), host(wd), host(dyd)          # exactly the values the GPU sees
    tol = TOL[dtype]
    errs = {}
    if "fwd" in passes:
        y = S.scc_forward(xd, wd, layer.cg, layer.co)
        assert y.shape == (layer.N, layer.Cout, layer.H, layer.W) and y.dtype == dtype
        errs["fwd"] = rel_err(host(y), O.forward(xr, wr, layer.cg, layer.co))
    if "bwi" in passes:
        dx = S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co)
        assert dx.shape == x.shape and dx.dtype == dtype
        errs["bwi"] = rel_err(host(dx), O.backward_input(dyr, wr, layer.Cin, layer.cg, layer.co))
    if "bww" in passes:
        dw = S.scc_backward_weight(xd, dyd, layer.cg, layer.co)
        assert dw.shape == (layer.Cout, layer.L) and dw.dtype == torch.float32
        # dw is float32 in both dtypes: exact products of the (bf16-rounded) inputs, fp32 sums
        errs["bww"] = rel_err(host(dw), O.backward_weight(xr, dyr, layer.cg, layer.co))
    torch.cuda.synchronize()
    for k, e in errs.items():
        bar = TOL[torch.float32] if k == "bww" else tol
        assert e <= bar, "%s %s %s: rel err %.3e > %.1e" % (layer.name, dtype, k, e, bar)
    return errs


def small(name, N, Cin, Cout, H, W, cg, co, **kw):
    return Wk.Layer(name, 9, N=N, Cin=Cin, Cout=Cout, H=H, W=W, cg=cg, co=co, **kw)


# Shapes the oracle finishes at once, spanning several tiles with ragged tails: odd H*W,
# H*W below one wavefront, Cout not a multiple of the period, Cout below the period, wraps.
SMALL_SHAPES = [
    Wk.SMALL,
    small("tiny_paper_example", 1, 4, 4, 1, 1, 2, 0.5),
    small("one_pixel", 3, 8, 8, 1, 1, 2, 0.5),
    small("odd_hw", 2, 24, 40, 7, 5, 3, 0.5),
    small("hw_3x3_many_n", 37, 16, 20, 3, 3, 2, 0.25),
    small("cout_below_period", 2, 64, 5, 6, 6, 4, 0.75),
    small("cout_not_multiple_of_period", 2, 64, 77, 9, 9, 4, 0.5),
    small("one_group_rotated", 2, 48, 40, 5, 5, 1, 0.3),
    small("one_group_no_overlap", 2, 32, 16, 4, 4, 1, 0.0),
    small("full_overlap", 2, 32, 48, 4, 4, 2, 1.0),
    small("zero_overlap_groups", 3, 96, 96, 10, 10, 4, 0.0),
    small("coprime_stride_wraps", 2, 128, 200, 8, 8, 2, 0.33),
    small("ragged_columns", 5, 64, 64, 13, 11, 2, 0.5),
    small("expand", 2, 32, 256, 12, 12, 2, 0.5),
    small("shrink", 2, 256, 32, 12, 12, 4, 0.5),
    small("l_is_one", 2, 16, 16, 5, 5, 16, 0.5),
    small("wide_window_1024", 1, 1024, 96, 2, 2, 2, 0.5),
    small("mid_256_16x16", 4, 256, 256, 16, 16, 4, 0.5),
    small("mid_512_14x14", 3, 512, 512, 14, 14, 8, 0.5, x_law="halfnormal"),
]


@pytest.mark.parametrize("layer", SMALL_SHAPES, ids=lambda l: l.name)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_small_shapes(S, layer, dtype):
    check_layer(S, layer, dtype)


def test_random_small_sweep(S):
    rng = np.random.default_rng(20210100745)
    for i in range(40):
        cg = int(rng.choice([1, 2, 3, 4, 8]))
        Cin = cg * int(rng.integers(1, 24))
        Cout = int(rng.integers(1, 80))
        H, W = int(rng.integers(1, 12)), int(rng.integers(1, 12))
        N = int(rng.integers(1, 6))
        co = float(rng.choice([0.0, 0.1, 0.25, 1 / 3, 0.33, 0.5, 0.66, 0.75, 1.0, rng.random()]))
        layer = small("rand%d" % i, N, Cin, Cout, H, W, cg, co)
        check_layer(S, layer, torch.float32, seed_offset=i)


# Full-size configurations, in the launch configuration the benchmark times.
@pytest.mark.parametrize("layer", Wk.METRIC_SWEEP, ids=lambda l: l.name)
def test_metric_layer_overlap_sweep(S, layer):
    check_layer(S, layer, torch.float32)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_late_stage_layer(S, dtype):
    check_layer(S, Wk.LATE, dtype)


def test_metric_layer_bf16(S):
    check_layer(S, Wk.METRIC, torch.bfloat16)


def test_channel_expanding_layer(S):
    check_layer(S, Wk.EXPAND, torch.float32)


@pytest.mark.parametrize("layer", Wk.STACK, ids=lambda l: l.name)
def test_mobilenet_shaped_stack(S, layer):
    check_layer(S, layer, torch.float32)


@pytest.mark.parametrize("layer", Wk.CG_SWEEP, ids=lambda l: l.name)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_group_count_sweep(S, layer, dtype):
    # cg = 1 is a (rotated) pointwise convolution with 256-channel windows; cg = 8 has 32-channel windows
    check_layer(S, layer, dtype)


@pytest.mark.parametrize("layer", Wk.BATCH_SWEEP[:3] + Wk.BATCH_SWEEP[4:5], ids=lambda l: l.name)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_batch_sweep(S, layer, dtype):
    # inference-sized batches (16, 32, 64) and one above the metric layer's (256), every element compared
    check_layer(S, layer, dtype)


def test_batch_512_every_element(S):
    # N = 512 (134 MB per tensor): every element of all three passes
    check_layer(S, Wk.BATCH_SWEEP[5], torch.float32)


def test_chip_filling_grid_with_ragged_tail(S):
    # 258 column tiles x 8 filter tiles = 2064 wavefronts: the forward and grad-input launch workgroups of 8
    # wavefronts here (the forward with its second half delayed), with 14x14 planes and a last column tile
    # that is only a quarter full
    check_layer(S, small("fills_chip", 168, 256, 256, 14, 14, 4, 0.5))
    check_layer(S, small("fills_chip_co0", 168, 256, 256, 14, 14, 4, 0.0))


def test_largest_batch_every_sample(S):
    # N = 1024 (268 MB per tensor, the top of the paper's batch sweep).  Forward and grad-input are
    # independent per sample, so the oracle takes them in slices of 128 samples, all 1024 of them;
    # grad-weight sums over every sample and is compared whole.
    layer = Wk.BATCH_SWEEP[-1]
    x, w, dy = Wk.make_inputs(layer)
    xd, wd, dyd = to_dev(x, torch.float32), to_dev(w, torch.float32), to_dev(dy, torch.float32)
    y = S.scc_forward(xd, wd, layer.cg, layer.co)
    dx = S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co)
    dw = S.scc_backward_weight(xd, dyd, layer.cg, layer.co)
    torch.cuda.synchronize()
    yh, dxh, w64 = host(y), host(dx), w.astype(np.float64)
    del y, dx
    for lo in range(0, layer.N, 128):
        sl = slice(lo, lo + 128)
        assert rel_err(yh[sl], O.forward(x[sl].astype(np.float64), w64, layer.cg, layer.co)) <= TOL[torch.float32], lo
        assert rel_err(dxh[sl], O.backward_input(dy[sl].astype(np.float64), w64, layer.Cin, layer.cg, layer.co)) \
            <= TOL[torch.float32], lo
    ref = O.backward_weight(x.astype(np.float64), dy.astype(np.float64), layer.cg, layer.co)
    assert rel_err(host(dw), ref) <= TOL[torch.float32]


@pytest.mark.parametrize("xs,ws", [(2.0 ** -90, 2.0 ** 40), (2.0 ** 90, 2.0 ** -40), (2.0 ** -40, 2.0 ** -40), (1e-3, 1e3)],
                         ids=["tiny_x", "huge_x", "tiny_both", "mixed"])
def test_fp32_dynamic_range(S, xs, ws):
    # fp32 operands are split into bf16 pieces on the way to the matrix cores; bf16 keeps the binary32 exponent
    # range, so scaling the inputs by large powers of two must not change the relative error
    layer = small("range", 8, 64, 64, 8, 8, 2, 0.5)       # 512 columns: the matrix-core kernels take it
    x, w, dy = Wk.make_inputs(layer)
    x, w = (x * np.float32(xs)), (w * np.float32(ws))    # dy stays O(1) so that no gradient leaves the fp32 range
    xd, wd, dyd = to_dev(x, torch.float32), to_dev(w, torch.float32), to_dev(dy, torch.float32)
    x64, w64, dy64 = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
    assert rel_err(host64(S.scc_forward(xd, wd, layer.cg, layer.co)), O.forward(x64, w64, layer.cg, layer.co)) <= 2e-6
    assert rel_err(host64(S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co)),
                   O.backward_input(dy64, w64, layer.Cin, layer.cg, layer.co)) <= 2e-6
    assert rel_err(host64(S.scc_backward_weight(xd, dyd, layer.cg, layer.co)),
                   O.backward_weight(x64, dy64, layer.cg, layer.co)) <= 2e-6


def test_fp32_per_channel_scales(S):
    # every channel plane has its own scale (2^-30 .. 2^30) and the weights undo it, so all products of a sum
    # are of similar size although the operands differ by 18 orders of magnitude: an error in the low-order
    # pieces of the bf16 split of either operand would show at full size
    layer = small("scales", 8, 96, 80, 8, 8, 3, 0.4)
    x, w, dy = Wk.make_inputs(layer)
    rng = np.random.default_rng(4242)
    sc = (2.0 ** rng.integers(-30, 31, size=layer.Cin)).astype(np.float32)
    x = x * sc[None, :, None, None]
    starts = O.starts(layer.Cin, layer.Cout, layer.cg, layer.co)
    for k in range(layer.Cout):
        idx = (starts[k] + np.arange(layer.L)) % layer.Cin
        w[k] = w[k] / sc[idx]
    xd, wd = to_dev(x, torch.float32), to_dev(w, torch.float32)
    ref = O.forward(x.astype(np.float64), w.astype(np.float64), layer.cg, layer.co)
    assert rel_err(host64(S.scc_forward(xd, wd, layer.cg, layer.co)), ref) <= 2e-6


def test_fp32_error_is_at_rounding_level(S):
    # on the metric layer the error against the fp64 oracle is that of fp32 accumulation (a few 1e-7), far
    # below the 2e-5 bar: the split loses nothing that fp32 arithmetic would keep
    errs = check_layer(S, Wk.METRIC)
    assert max(errs.values()) <= 1e-6, errs


def test_adjoint_identity_on_gpu_outputs(S):
    layer = Wk.METRIC
    x, w, dy = Wk.make_inputs(layer)
    xd, wd, dyd = to_dev(x, torch.float32), to_dev(w, torch.float32), to_dev(dy, torch.float32)
    y = host(S.scc_forward(xd, wd, layer.cg, layer.co)).astype(np.float64)
    dx = host(S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co)).astype(np.float64)
    dw = host(S.scc_backward_weight(xd, dyd, layer.cg, layer.co)).astype(np.float64)
    a, b, c = float(np.sum(dy * y)), float(np.sum(dx * x)), float(np.sum(dw * w))
    scale = float(np.sqrt(np.sum((dy * y) ** 2)))      # size of the terms being summed
    assert abs(a - b) <= 1e-3 * scale and abs(a - c) <= 1e-3 * scale


def test_two_runs_are_bitwise_equal(S):
    for layer in (Wk.METRIC, small("ragged_columns", 5, 64, 64, 13, 11, 2, 0.5)):
        x, w, dy = Wk.make_inputs(layer)
        xd, wd, dyd = to_dev(x, torch.float32), to_dev(w, torch.float32), to_dev(dy, torch.float32)
        runs = []
        for _ in range(2):
            runs.append((S.scc_forward(xd, wd, layer.cg, layer.co).clone(),
                         S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co).clone(),
                         S.scc_backward_weight(xd, dyd, layer.cg, layer.co).clone()))
        for a, b in zip(*runs):
            assert torch.equal(a, b)


def test_outputs_are_overwritten_not_accumulated(S):
    layer = Wk.SMALL
    x, w, dy = Wk.make_inputs(layer)
    xd, wd, dyd = to_dev(x, torch.float32), to_dev(w, torch.float32), to_dev(dy, torch.float32)
    y0 = S.scc_forward(xd, wd, layer.cg, layer.co)
    junk = torch.full_like(y0, 1e30)
    assert torch.equal(S.scc_forward(xd, wd, layer.cg, layer.co, out=junk), y0)
    dx0 = S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co)
    junk = torch.full_like(dx0, float("nan"))
    assert torch.equal(S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co, out=junk), dx0)
    dw0 = S.scc_backward_weight(xd, dyd, layer.cg, layer.co)
    junk = torch.full_like(dw0, float("nan"))
    assert torch.equal(S.scc_backward_weight(xd, dyd, layer.cg, layer.co, out=junk), dw0)


def test_uncovered_channels_get_zero_gradient(S):
    # Cout below the period: some input channels lie in no window
    layer = small("uncovered", 2, 64, 2, 4, 4, 4, 0.0)
    x, w, dy = Wk.make_inputs(layer)
    dx = host(S.scc_backward_input(to_dev(dy, torch.float32), to_dev(w, torch.float32), 64, 4, 0.0))
    assert np.all(dx[:, 32:] == 0.0) and np.any(dx[:, :32] != 0.0)


def test_non_default_stream(S):
    layer = dataclasses.replace(Wk.SMALL, N=4)
    x, w, dy = Wk.make_inputs(layer)
    xd, wd = to_dev(x, torch.float32), to_dev(w, torch.float32)
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        y = S.scc_forward(xd, wd, layer.cg, layer.co)
    st.synchronize()
    assert rel_err(host(y), O.forward(x, w, layer.cg, layer.co)) <= 2e-5


def test_random_sweep_matrix_core_shapes(S):
    """Shapes the tiled matrix-core kernels accept (window of 8+ channels, hundreds of columns), with
    ragged column tiles, partial filter tiles, banded and dense windows, wraps; fp32 and bf16."""
    rng = np.random.default_rng(7452101)
    for i in range(36):
        cg = int(rng.choice([1, 2, 3, 4, 8]))
        L = int(rng.choice([8, 12, 16, 20, 24, 32, 40, 48, 64, 96]))
        Cin = cg * L
        Cout = int(rng.integers(8, 200))
        H, W = int(rng.integers(2, 15)), int(rng.integers(2, 15))
        if i % 3 == 0:
            W = 4 * max(1, W // 4)            # H*W a multiple of 4: vector plane accesses
        N = int(rng.integers(2, 9))
        co = float(rng.choice([0.0, 0.125, 0.25, 1 / 3, 0.33, 0.5, 0.625, 0.75, 0.9, 1.0]))
        layer = small("mc%d" % i, N, Cin, Cout, H, W, cg, co)
        check_layer(S, layer, torch.bfloat16 if i % 4 == 3 else torch.float32, seed_offset=100 + i)


def test_random_sweep_wide_tiles_long_windows(S):
    """Thousands of columns (128- and 64-column tiles, one wavefront per tile) and windows of 64-320 channels
    (several staged weight blocks per contraction, contractions shared by 2 or 4 wavefronts), fp32 and bf16."""
    rng = np.random.default_rng(7452102)
    for i in range(12):
        cg = int(rng.choice([1, 2, 4]))
        L = int(rng.choice([64, 80, 128, 192, 256, 320]))
        Cin = cg * L
        Cout = int(rng.integers(24, 260))
        H = W = int(rng.choice([4, 7, 8, 14, 16]))
        N = int(rng.integers(8, 48))
        co = float(rng.choice([0.0, 0.25, 1 / 3, 0.5, 0.75, 0.9]))
        layer = small("wide%d" % i, N, Cin, Cout, H, W, cg, co)
        check_layer(S, layer, torch.bfloat16 if i % 3 == 2 else torch.float32, seed_offset=200 + i)


def test_unaligned_tensor_views(S):
    """Tensors that start 4 bytes into an allocation: the 16-byte plane accesses must not be used."""
    layer = small("unaligned", 3, 64, 96, 8, 8, 2, 0.5)
    x, w, dy = Wk.make_inputs(layer)

    def shifted(a):
        buf = torch.empty(a.size + 1, dtype=torch.float32, device="cuda")
        v = buf[1:].view(a.shape)
        v.copy_(torch.from_numpy(a))
        assert v.data_ptr() % 16 == 4 and v.is_contiguous()
        return v

    xd, wd, dyd = shifted(x), shifted(w), shifted(dy)
    y = torch.empty(layer.N * layer.Cout * layer.HW + 1, dtype=torch.float32, device="cuda")[1:].view(
        layer.N, layer.Cout, layer.H, layer.W)
    dx = torch.empty(x.size + 1, dtype=torch.float32, device="cuda")[1:].view(x.shape)
    S.scc_forward(xd, wd, layer.cg, layer.co, out=y)
    S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co, out=dx)
    dw = S.scc_backward_weight(xd, dyd, layer.cg, layer.co)
    assert rel_err(host(y), O.forward(x, w, layer.cg, layer.co)) <= 2e-5
    assert rel_err(host(dx), O.backward_input(dy, w, layer.Cin, layer.cg, layer.co)) <= 2e-5
    assert rel_err(host(dw), O.backward_weight(x, dy, layer.cg, layer.co)) <= 2e-5


def test_workspace_contract(S):
    import ctypes
    layer = Wk.METRIC
    need = S.scc_backward_weight_workspace_bytes(layer.N, layer.Cin, layer.Cout, layer.H, layer.W, layer.cg, layer.co)
    assert need > 0 and need % 4 == 0
    x, w, dy = Wk.make_inputs(layer)
    xd, dyd = to_dev(x, torch.float32), to_dev(dy, torch.float32)
    dw = torch.empty(layer.Cout, layer.L, device="cuda")
    lib = S.load()
    shape = (layer.N, layer.Cin, layer.Cout, layer.H, layer.W, layer.cg, layer.co, 0)
    small_ws = torch.empty(need - 4, dtype=torch.uint8, device="cuda")
    # too small, missing, misaligned: rejected on the host, dw untouched
    dw.fill_(7.0)
    assert lib.scc_backward_weight(xd.data_ptr(), dyd.data_ptr(), dw.data_ptr(), *shape, small_ws.data_ptr(),
                                   need - 4, None) == -5
    assert lib.scc_backward_weight(xd.data_ptr(), dyd.data_ptr(), dw.data_ptr(), *shape, None, 0, None) == -5
    big = torch.empty(need + 512, dtype=torch.uint8, device="cuda")
    assert lib.scc_backward_weight(xd.data_ptr(), dyd.data_ptr(), dw.data_ptr(), *shape, big.data_ptr() + 4,
                                   need, None) == -5
    torch.cuda.synchronize()
    assert bool((dw == 7.0).all())
    # workspace full of NaN beforehand: contents before the call must not matter
    ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device="cuda")
    got = S.scc_backward_weight(xd, dyd, layer.cg, layer.co, workspace=ws.view(torch.uint8))
    assert rel_err(host(got), O.backward_weight(x, dy, layer.cg, layer.co)) <= 2e-5


@pytest.mark.parametrize("layer", Wk.STACK + [Wk.METRIC_SWEEP[0], Wk.METRIC_SWEEP[1], Wk.METRIC_SWEEP[3], Wk.EXPAND],
                         ids=lambda l: l.name)
def test_bf16_more_layers(S, layer):
    # bf16 on every layer of the 13-layer stack, the rest of the overlap sweep and the channel-expanding layer
    check_layer(S, layer, torch.bfloat16)


def test_zero_weight_windows_give_exact_zeros(S):
    """Banded tiles put filters of neighbouring windows side by side and multiply each with zero weights outside
    its own window.  With finite inputs that masking is exact: filters whose weights are all zero give exactly
    zero, whatever their neighbours' windows hold, and channels covered only by such filters get exactly zero
    gradient; everything else still matches the oracle."""
    for layer in (small("banded", 3, 256, 256, 8, 8, 4, 0.25), small("banded_odd", 2, 96, 120, 5, 5, 2, 1 / 3),
                  small("dense", 3, 128, 128, 8, 8, 2, 0.5)):
        x, w, dy = Wk.make_inputs(layer)
        x *= np.float32(1e20)                                  # large but finite
        starts = O.starts(layer.Cin, layer.Cout, layer.cg, layer.co)
        dead = [k for k in range(layer.Cout) if starts[k] == starts[1]]      # every filter of one window
        w[dead] = 0.0
        xd, wd, dyd = to_dev(x, torch.float32), to_dev(w, torch.float32), to_dev(dy, torch.float32)
        y = host(S.scc_forward(xd, wd, layer.cg, layer.co))
        assert np.all(y[:, dead] == 0.0), layer.name
        assert rel_err(y, O.forward(x.astype(np.float64), w.astype(np.float64), layer.cg, layer.co)) <= 2e-5
        # grad-input with every weight zero except one window's: channels outside that window get exact zeros
        w2 = np.zeros_like(w)
        w2[dead] = 1.0
        dx = host(S.scc_backward_input(dyd, to_dev(w2, torch.float32), layer.Cin, layer.cg, layer.co))
        inside = sorted({(starts[1] + j) % layer.Cin for j in range(layer.L)})
        outside = [c for c in range(layer.Cin) if c not in inside]
        assert np.all(dx[:, outside] == 0.0), layer.name
        assert rel_err(dx, O.backward_input(dy.astype(np.float64), w2.astype(np.float64), layer.Cin, layer.cg,
                                            layer.co)) <= 2e-5


def test_non_finite_input_stays_in_its_own_column(S):
    """An Inf in one element of x may turn outputs of other filters at the SAME sample and pixel into NaN (zero
    weights multiply it inside a tile), as the header says; it never reaches another sample or pixel, and every
    output that stays finite still matches the oracle."""
    for layer in (small("banded", 3, 256, 256, 8, 8, 4, 0.25), small("dense", 3, 128, 128, 8, 8, 2, 0.5)):
        x, w, _ = Wk.make_inputs(layer)
        x[1, 5, 0, 3] = np.inf
        y = host(S.scc_forward(to_dev(x, torch.float32), to_dev(w, torch.float32), layer.cg, layer.co))
        bad = ~np.isfinite(y)
        n, _, h, ww = np.nonzero(bad)
        assert bad.any() and set(n.tolist()) == {1} and set(zip(h.tolist(), ww.tolist())) == {(0, 3)}
        x0 = x.copy()
        x0[1, 5, 0, 3] = 0.0
        ref = O.forward(x0.astype(np.float64), w.astype(np.float64), layer.cg, layer.co)
        ok = np.isfinite(y)
        assert float(np.max(np.abs(y[ok] - ref[ok]))) <= 2e-5 * float(np.max(np.abs(ref)))


def test_subnormal_operands(S):
    """Operands far below the normal range.  fp32 tensors that go through the bf16 split keep all three pieces
    down to about 2^-110; below that the low pieces underflow and the error is bounded in absolute terms (a
    fraction of the smallest normal number) instead of relative ones.  grad-weight as a separate pass multiplies
    in binary32 and keeps full accuracy."""
    layer = small("subnormal", 8, 128, 128, 8, 8, 2, 0.5)
    x, w, dy = Wk.make_inputs(layer)
    w64, dy64 = w.astype(np.float64), dy.astype(np.float64)
    wd, dyd = to_dev(w, torch.float32), to_dev(dy, torch.float32)
    for scale, rel_bar, abs_bar in ((2.0 ** -100, 2e-6, 0.0), (2.0 ** -130, 0.0, 2.0 ** -129)):
        xs = (x * np.float32(scale)).astype(np.float32)          # 2^-130: every element is subnormal
        dys = (dy * np.float32(scale)).astype(np.float32)
        xd = to_dev(xs, torch.float32)
        y = host64(S.scc_forward(xd, wd, layer.cg, layer.co))
        dx = host64(S.scc_backward_input(to_dev(dys, torch.float32), wd, layer.Cin, layer.cg, layer.co))
        dw = host64(S.scc_backward_weight(xd, dyd, layer.cg, layer.co))
        ry = O.forward(xs.astype(np.float64), w64, layer.cg, layer.co)
        rdx = O.backward_input(dys.astype(np.float64), w64, layer.Cin, layer.cg, layer.co)
        rdw = O.backward_weight(xs.astype(np.float64), dy64, layer.cg, layer.co)
        for got, ref in ((y, ry), (dx, rdx)):
            assert float(np.max(np.abs(got - ref))) <= rel_bar * float(np.max(np.abs(ref))) + abs_bar, scale
        assert rel_err(dw, rdw) <= 2e-6, scale
