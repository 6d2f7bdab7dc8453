"""The allocation-free grad-weight entry point against the ordinary one, through the C ABI.

scc_backward_weight_static keeps its K-split partials in a buffer the library holds itself.  Two calls in a
row, the second on a smaller problem, must each reproduce scc_backward_weight (same kernels and summation
order: bitwise equal, and within the fp32 bar of the parity tests), whatever the buffer held before.
"""
import ctypes

import numpy as np
import pytest
import torch

import scc_workloads as Wk

pytestmark = pytest.mark.gpu

TOL = 2e-5


def _args(layer, dtype_code):
    return (layer.N, layer.Cin, layer.Cout, layer.H, layer.W, layer.cg, float(layer.co), dtype_code)


def _rel(a, b):
    a, b = a.double().cpu().numpy(), b.double().cpu().numpy()
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_static_scratch_matches_workspace_entry_point_twice(dtype):
    import paper_2101_00745_amd as S
    assert torch.cuda.is_available(), "this test needs the MI355X"
    lib = S.load()
    code = 0 if dtype == torch.float32 else 1
    big = Wk.METRIC                                                     # 2 MiB of partials
    little = Wk.Layer("little", 9, N=24, Cin=128, Cout=96, H=12, W=12, cg=2, co=0.5)   # 144 KiB of partials
    for layer in (big, little):                                         # the second call is the smaller one
        need = lib.scc_backward_weight_workspace_bytes(*_args(layer, code))
        assert 0 < need <= S.scc.STATIC_SCRATCH_BYTES, (layer.name, need)
        x, _, dy = Wk.make_inputs(layer)
        xd, dyd = torch.from_numpy(x).to(dtype).cuda(), torch.from_numpy(dy).to(dtype).cuda()
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        ref = torch.empty(layer.Cout, layer.L, dtype=torch.float32, device="cuda")
        got = torch.full_like(ref, float("nan"))
        st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        assert lib.scc_backward_weight(xd.data_ptr(), dyd.data_ptr(), ref.data_ptr(), *_args(layer, code),
                                       ws.data_ptr(), need, st) == 0
        assert lib.scc_backward_weight_static(xd.data_ptr(), dyd.data_ptr(), got.data_ptr(), *_args(layer, code),
                                              st) == 0
        torch.cuda.synchronize()
        assert _rel(got, ref) <= TOL, layer.name
        assert torch.equal(got, ref), layer.name
        # and once more on the same inputs: what the previous call left in the buffer does not matter
        again = torch.full_like(ref, float("nan"))
        assert lib.scc_backward_weight_static(xd.data_ptr(), dyd.data_ptr(), again.data_ptr(), *_args(layer, code),
                                              st) == 0
        torch.cuda.synchronize()
        assert torch.equal(again, ref), layer.name


def test_static_scratch_binding_and_problem_without_scratch():
    import paper_2101_00745_amd as S
    layer = Wk.SMALL                                                    # takes the generic kernel: no scratch at all
    x, _, dy = Wk.make_inputs(layer)
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    out = torch.empty(layer.Cout, layer.L, dtype=torch.float32, device="cuda")
    S.scc_backward_weight_static(xd, dyd, layer.cg, layer.co, out)
    torch.cuda.synchronize()
    assert torch.equal(out, S.scc_backward_weight(xd, dyd, layer.cg, layer.co))
