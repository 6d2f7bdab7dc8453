"""The PyTorch layer over the C ABI: autograd results against the fp64 oracle, and a depthwise + SCC block
that trains end to end on the GPU."""
import numpy as np
import pytest
import torch

import scc_workloads as Wk
from oracle import scc_oracle as O

pytestmark = pytest.mark.gpu


def rel(got, ref):
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)) / np.max(np.abs(ref)))


@pytest.mark.parametrize("bias", [False, True])
def test_autograd_matches_oracle(bias):
    from paper_2101_00745_amd.nn import SCC
    layer = Wk.Layer("nn_case", 9, N=3, Cin=64, Cout=96, H=9, W=8, cg=4, co=0.5)
    x, w, dy = Wk.make_inputs(layer)
    m = SCC(layer.Cin, layer.Cout, cg=layer.cg, co=layer.co, bias=bias)
    b = np.linspace(-1, 1, layer.Cout).astype(np.float32)
    with torch.no_grad():
        m.weight.copy_(torch.from_numpy(w))
        if bias:
            m.bias.copy_(torch.from_numpy(b))
    xd = torch.from_numpy(x).cuda().requires_grad_(True)
    y = m(xd)
    y.backward(torch.from_numpy(dy).cuda())
    y_ref = O.forward(x, w, layer.cg, layer.co) + (b.astype(np.float64)[None, :, None, None] if bias else 0.0)
    assert rel(y.detach().cpu().numpy(), y_ref) <= 2e-5
    assert rel(xd.grad.cpu().numpy(), O.backward_input(dy, w, layer.Cin, layer.cg, layer.co)) <= 2e-5
    assert rel(m.weight.grad.cpu().numpy(), O.backward_weight(x, dy, layer.cg, layer.co)) <= 2e-5
    if bias:
        assert rel(m.bias.grad.cpu().numpy(), dy.astype(np.float64).sum(axis=(0, 2, 3))) <= 2e-5


def test_depthwise_scc_block_trains():
    """A student DW3x3 + SCC block fitted to a teacher block of the same shape: the loss must fall."""
    from paper_2101_00745_amd.nn import SCC
    torch.manual_seed(0)

    def block():
        return torch.nn.Conv2d(32, 32, 3, padding=1, groups=32, bias=False).cuda(), SCC(32, 64, cg=2, co=0.5, bias=True)

    def run(b, x):
        return b[1](torch.relu(b[0](x)))

    teacher, student = block(), block()
    x = torch.randn(16, 32, 8, 8, device="cuda")
    with torch.no_grad():
        target = run(teacher, x)
    opt = torch.optim.Adam(list(student[0].parameters()) + list(student[1].parameters()), lr=0.02)
    losses = []
    for _ in range(60):
        opt.zero_grad()
        loss = torch.nn.functional.mse_loss(run(student, x), target)
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert losses[-1] < 0.5 * losses[0], losses[::10]


def test_module_rejects_bad_configuration():
    from paper_2101_00745_amd.nn import SCC
    from paper_2101_00745_amd.scc import SccError
    with pytest.raises(SccError):
        SCC(30, 16, cg=4, co=0.5)      # 30 % 4 != 0
    with pytest.raises(SccError):
        SCC(32, 16, cg=4, co=1.5)
