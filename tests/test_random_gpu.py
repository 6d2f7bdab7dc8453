"""Randomised GPU parity over every entry point: seeded random layer shapes (channel counts, group counts, overlaps,
map sizes, batches, both dtypes, depthwise strides), each checked element by element against the fp64 CPU oracle.
The draws are fixed by the seed, so a failure names a reproducible case.  Bar: the benchmark spec, 2e-5 (fp32) and
1e-2 (bf16) of the largest reference magnitude; dw and the depthwise filters' gradient are binary32 in both dtypes
and held to 2e-5."""
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
    lib.load()
    return lib


def rel_err(got, ref):
    denom = float(np.max(np.abs(ref)))
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref))) / (denom if denom else 1.0)


def host(t):
    return t.float().cpu().numpy()


def draw_case(rng):
    cg = int(rng.choice([1, 2, 2, 3, 4, 4, 5, 8]))
    L = int(rng.choice([4, 8, 12, 16, 24, 32, 48, 64, 96, 128]))
    Cin = cg * L
    Cout = int(rng.choice([1, 3, 8, 17, 32, 40, 64, 96, 130, 256]))
    co = float(rng.choice([0.0, 0.25, 1.0 / 3.0, 0.5, 0.5, 0.75, 1.0]))
    H, W = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16])), int(rng.choice([1, 2, 4, 6, 8, 9, 16, 20]))
    N = int(rng.choice([1, 2, 3, 5, 16, 33, 64]))
    # keep the oracle's work per case bounded
    while N > 1 and N * H * W * Cout * L > 6e7:
        N //= 2
    return N, Cin, Cout, H, W, cg, co


@pytest.mark.parametrize("seed", range(24))
def test_random_layers(S, seed):
    rng = np.random.default_rng(7459000 + seed)
    for _ in range(4):
        N, Cin, Cout, H, W, cg, co = draw_case(rng)
        dtype = torch.float32 if rng.random() < 0.7 else torch.bfloat16
        s = int(rng.choice([1, 1, 2, 3]))
        tag = "seed %d: N=%d %d->%d %dx%d cg=%d co=%.3f stride=%d %s" % (seed, N, Cin, Cout, H, W, cg, co, s, dtype)
        L = Cin // cg
        x = rng.standard_normal((N, Cin, H, W)).astype(np.float32)
        w = (rng.standard_normal((Cout, L)) * np.sqrt(2.0 / L)).astype(np.float32)
        dy = rng.standard_normal((N, Cout, H, W)).astype(np.float32)
        xin = rng.standard_normal((N, Cin, H * s, W * s)).astype(np.float32)
        kdw = (rng.standard_normal((Cin, 3, 3)) / 3.0).astype(np.float32)
        xd, wd, dyd, xind, kd = (torch.from_numpy(a).to(dtype).cuda() for a in (x, w, dy, xin, kdw))
        xr, wr, dyr, xinr, kr = (host(t) for t in (xd, wd, dyd, xind, kd))        # the values the GPU sees
        tol = TOL[dtype]
        y = S.scc_forward(xd, wd, cg, co)
        dx = S.scc_backward_input(dyd, wd, Cin, cg, co)
        dw = S.scc_backward_weight(xd, dyd, cg, co)
        dx2, dw2 = S.scc_backward(xd, dyd, wd, cg, co)
        yb = S.scc_dw_forward(xind, kd, wd, cg, co, s)
        ybf = S.scc_dw_forward(xind, kd, wd, cg, co, s, fused=True) if S.scc_dw_forward_fusable(N, Cin, Cout, H * s, W * s, s, cg, co, dtype) else None
        z = S.scc_depthwise3x3_forward(xind, kd, s)
        gx, gk = S.scc_depthwise3x3_backward(xind, kd, xd, s)                      # x doubles as dz: it has z's shape
        torch.cuda.synchronize()
        assert rel_err(host(y), O.forward(xr, wr, cg, co)) <= tol, tag
        ref_dx, ref_dw = O.backward_input(dyr, wr, Cin, cg, co), O.backward_weight(xr, dyr, cg, co)
        assert rel_err(host(dx), ref_dx) <= tol and rel_err(host(dx2), ref_dx) <= tol, tag
        assert rel_err(host(dw), ref_dw) <= 2e-5 and rel_err(host(dw2), ref_dw) <= 2e-5, tag
        ref_blk = O.depthwise_scc_forward(xinr, kr, wr, cg, co, s)
        assert rel_err(host(yb), ref_blk) <= tol, tag
        if ybf is not None:
            assert rel_err(host(ybf), ref_blk) <= tol, tag
        assert rel_err(host(z), O.depthwise3x3(xinr, kr, s)) <= tol, tag
        ref_gx, ref_gk = O.depthwise3x3_backward(xinr, kr, xr, s)
        assert rel_err(host(gx), ref_gx) <= tol and rel_err(host(gk), ref_gk) <= 2e-5, tag
