"""Thin Python binding of the SCC C ABI (include/scc.h): argument marshalling only.

Every step of the computation runs in the HIP kernels of libscc_hip.so.  PyTorch supplies
device memory (``torch.empty``), raw pointers (``data_ptr``) and the current HIP stream,
nothing else.  There is no CPU path: if the library is missing or a tensor is not on the
GPU the call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libscc_hip.so")

SCC_F32, SCC_BF16 = 0, 1
SYMBOLS = ("scc_window_params", "scc_forward", "scc_backward_input",
           "scc_backward_weight_workspace_bytes", "scc_backward_weight", "scc_backward_weight_static",
           "scc_backward_workspace_bytes", "scc_backward",
           "scc_depthwise3x3_out", "scc_depthwise3x3_forward", "scc_depthwise3x3_backward_workspace_bytes",
           "scc_depthwise3x3_backward", "scc_dw_forward_workspace_bytes", "scc_dw_forward_fusable", "scc_dw_forward",
           "scc_status_string")
STATIC_SCRATCH_BYTES = 8 << 20    # SCC_STATIC_SCRATCH_BYTES of include/scc.h

_lib = None


class SccError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(message)
        self.status = status


def load():
    """Load libscc_hip.so (built in-tree by ``paper_2101_00745_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libscc_hip.so is not built: run `python -m paper_2101_00745_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_dbl, c_vp, c_sz = ctypes.c_int, ctypes.c_double, ctypes.c_void_p, ctypes.c_size_t
    ip = ctypes.POINTER(c_int)
    shape = [c_int, c_int, c_int, c_int, c_int, c_int, c_dbl, c_int]  # N Cin Cout H W cg co dtype
    lib.scc_window_params.argtypes = [c_int, c_int, c_int, c_dbl, ip, ip, ip]
    lib.scc_window_params.restype = c_int
    lib.scc_forward.argtypes = [c_vp, c_vp, c_vp] + shape + [c_vp]
    lib.scc_forward.restype = c_int
    lib.scc_backward_input.argtypes = [c_vp, c_vp, c_vp] + shape + [c_vp]
    lib.scc_backward_input.restype = c_int
    lib.scc_backward_weight_workspace_bytes.argtypes = shape
    lib.scc_backward_weight_workspace_bytes.restype = c_sz
    lib.scc_backward_weight.argtypes = [c_vp, c_vp, c_vp] + shape + [c_vp, c_sz, c_vp]
    lib.scc_backward_weight.restype = c_int
    lib.scc_backward_workspace_bytes.argtypes = shape
    lib.scc_backward_workspace_bytes.restype = c_sz
    lib.scc_backward.argtypes = [c_vp] * 5 + shape + [c_vp, c_sz, c_vp]
    lib.scc_backward.restype = c_int
    lib.scc_backward_weight_static.argtypes = [c_vp, c_vp, c_vp] + shape + [c_vp]
    lib.scc_backward_weight_static.restype = c_int
    lib.scc_depthwise3x3_out.argtypes = [c_int, c_int]
    lib.scc_depthwise3x3_out.restype = c_int
    lib.scc_depthwise3x3_forward.argtypes = [c_vp, c_vp, c_vp] + [c_int] * 6 + [c_vp]
    lib.scc_depthwise3x3_forward.restype = c_int
    lib.scc_depthwise3x3_backward_workspace_bytes.argtypes = [c_int] * 6
    lib.scc_depthwise3x3_backward_workspace_bytes.restype = c_sz
    lib.scc_depthwise3x3_backward.argtypes = [c_vp] * 5 + [c_int] * 6 + [c_vp, c_sz, c_vp]
    lib.scc_depthwise3x3_backward.restype = c_int
    dw_shape = [c_int] * 7 + [c_dbl, c_int]     # N, Cin, Cout, H, W, dw_stride, cg, co, dtype
    lib.scc_dw_forward_workspace_bytes.argtypes = dw_shape
    lib.scc_dw_forward_workspace_bytes.restype = c_sz
    lib.scc_dw_forward_fusable.argtypes = dw_shape
    lib.scc_dw_forward_fusable.restype = c_int
    lib.scc_dw_forward.argtypes = [c_vp] * 4 + dw_shape + [c_vp, c_sz, c_vp]
    lib.scc_dw_forward.restype = c_int
    lib.scc_status_string.argtypes = [c_int]
    lib.scc_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def scc_status_string(status):
    return load().scc_status_string(int(status)).decode()


def _check(status):
    if status != 0:
        raise SccError(status, scc_status_string(status))


def scc_window_params(Cin, Cout, cg, co):
    """(L, stride, period) of Algorithm 1 for this layer; host only."""
    L, s, p = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(load().scc_window_params(Cin, Cout, cg, float(co), ctypes.byref(L), ctypes.byref(s), ctypes.byref(p)))
    return L.value, s.value, p.value


def _dtype_code(t):
    if t.dtype == torch.float32:
        return SCC_F32
    if t.dtype == torch.bfloat16:
        return SCC_BF16
    raise TypeError("SCC tensors must be float32 or bfloat16, got %s" % t.dtype)


def _dev(*tensors):
    for t in tensors:
        if not t.is_cuda:
            raise ValueError("SCC tensors must live on the GPU (there is no CPU path)")
        if not t.is_contiguous():
            raise ValueError("SCC tensors must be dense and contiguous (NCHW)")
    dev = tensors[0].device
    if any(t.device != dev for t in tensors):
        raise ValueError("SCC tensors must share one device")
    return dev


def _stream(dev):
    return ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)


def scc_forward(x, w, cg, co, out=None):
    """y = SCC(x; w): x [N,Cin,H,W], w [Cout,Cin//cg] -> y [N,Cout,H,W] (same dtype)."""
    dev = _dev(x, w)
    N, Cin, H, W = x.shape
    Cout = w.shape[0]
    if w.dtype != x.dtype or w.dim() != 2 or (cg >= 1 and Cin % cg == 0 and w.shape[1] != Cin // cg):
        raise ValueError("w must be [Cout, Cin//cg] with the dtype of x")
    y = torch.empty((N, Cout, H, W), dtype=x.dtype, device=dev) if out is None else out
    if out is not None:
        _dev(out)
        assert out.shape == (N, Cout, H, W) and out.dtype == x.dtype
    with torch.cuda.device(dev):
        _check(load().scc_forward(x.data_ptr(), w.data_ptr(), y.data_ptr(), N, Cin, Cout, H, W, cg, float(co),
                                  _dtype_code(x), _stream(dev)))
    return y


def scc_backward_input(dy, w, Cin, cg, co, out=None):
    """dx from dy [N,Cout,H,W] and w [Cout,Cin//cg] -> dx [N,Cin,H,W]."""
    dev = _dev(dy, w)
    N, Cout, H, W = dy.shape
    if w.dtype != dy.dtype or w.dim() != 2 or w.shape[0] != Cout or \
            (cg >= 1 and Cin % cg == 0 and w.shape[1] != Cin // cg):
        raise ValueError("w must be [Cout, Cin//cg] with the dtype of dy")
    dx = torch.empty((N, Cin, H, W), dtype=dy.dtype, device=dev) if out is None else out
    if out is not None:
        _dev(out)
        assert out.shape == (N, Cin, H, W) and out.dtype == dy.dtype
    with torch.cuda.device(dev):
        _check(load().scc_backward_input(dy.data_ptr(), w.data_ptr(), dx.data_ptr(), N, Cin, Cout, H, W, cg,
                                         float(co), _dtype_code(dy), _stream(dev)))
    return dx


def scc_backward_weight_workspace_bytes(N, Cin, Cout, H, W, cg, co, dtype=torch.float32):
    code = SCC_F32 if dtype == torch.float32 else SCC_BF16
    return int(load().scc_backward_weight_workspace_bytes(N, Cin, Cout, H, W, cg, float(co), code))


def scc_backward_weight(x, dy, cg, co, out=None, workspace=None):
    """dw (float32 [Cout, Cin//cg]) from x [N,Cin,H,W] and dy [N,Cout,H,W]."""
    dev = _dev(x, dy)
    N, Cin, H, W = x.shape
    Cout = dy.shape[1]
    if dy.dtype != x.dtype or dy.shape != (N, Cout, H, W):
        raise ValueError("dy must be [N,Cout,H,W] with the dtype of x")
    code = _dtype_code(x)
    need = int(load().scc_backward_weight_workspace_bytes(N, Cin, Cout, H, W, cg, float(co), code))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    L = Cin // cg if cg >= 1 and Cin % cg == 0 else 1
    dw = torch.empty((Cout, L), dtype=torch.float32, device=dev) if out is None else out
    if out is not None:
        _dev(out)
        assert out.shape == (Cout, L) and out.dtype == torch.float32
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        _check(load().scc_backward_weight(x.data_ptr(), dy.data_ptr(), dw.data_ptr(), N, Cin, Cout, H, W, cg,
                                          float(co), code, ws_ptr, ws_len, _stream(dev)))
    return dw


def scc_backward_weight_static(x, dy, cg, co, out):
    """scc_backward_weight on the library's own static scratch: the call itself allocates nothing, so the
    caller passes the output tensor ``out`` (float32 [Cout, Cin//cg])."""
    dev = _dev(x, dy, out)
    N, Cin, H, W = x.shape
    Cout = dy.shape[1]
    if dy.dtype != x.dtype or dy.shape != (N, Cout, H, W):
        raise ValueError("dy must be [N,Cout,H,W] with the dtype of x")
    L = Cin // cg if cg >= 1 and Cin % cg == 0 else 1
    if out.shape != (Cout, L) or out.dtype != torch.float32:
        raise ValueError("out must be float32 [Cout, Cin//cg]")
    with torch.cuda.device(dev):
        _check(load().scc_backward_weight_static(x.data_ptr(), dy.data_ptr(), out.data_ptr(), N, Cin, Cout, H, W, cg,
                                                 float(co), _dtype_code(x), _stream(dev)))
    return out


def scc_backward_workspace_bytes(N, Cin, Cout, H, W, cg, co, dtype=torch.float32):
    code = SCC_F32 if dtype == torch.float32 else SCC_BF16
    return int(load().scc_backward_workspace_bytes(N, Cin, Cout, H, W, cg, float(co), code))


def scc_backward(x, dy, w, cg, co, out_dx=None, out_dw=None, workspace=None):
    """(dx, dw) of one layer in one call: x [N,Cin,H,W], dy [N,Cout,H,W], w [Cout,Cin//cg]."""
    dev = _dev(x, dy, w)
    N, Cin, H, W = x.shape
    Cout = dy.shape[1]
    if dy.dtype != x.dtype or dy.shape != (N, Cout, H, W):
        raise ValueError("dy must be [N,Cout,H,W] with the dtype of x")
    if w.dtype != x.dtype or w.dim() != 2 or w.shape[0] != Cout or \
            (cg >= 1 and Cin % cg == 0 and w.shape[1] != Cin // cg):
        raise ValueError("w must be [Cout, Cin//cg] with the dtype of x")
    code = _dtype_code(x)
    need = int(load().scc_backward_workspace_bytes(N, Cin, Cout, H, W, cg, float(co), code))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    L = Cin // cg if cg >= 1 and Cin % cg == 0 else 1
    dx = torch.empty_like(x) if out_dx is None else out_dx
    dw = torch.empty((Cout, L), dtype=torch.float32, device=dev) if out_dw is None else out_dw
    for o, shp, dt in ((out_dx, x.shape, x.dtype), (out_dw, (Cout, L), torch.float32)):
        if o is not None:
            _dev(o)
            assert o.shape == shp and o.dtype == dt
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        _check(load().scc_backward(x.data_ptr(), dy.data_ptr(), w.data_ptr(), dx.data_ptr(), dw.data_ptr(), N, Cin, Cout,
                                   H, W, cg, float(co), code, ws_ptr, ws_len, _stream(dev)))
    return dx, dw


def scc_depthwise3x3_out(size, dw_stride):
    """Rows (columns) the depthwise 3x3 stage produces from `size` rows at spatial stride `dw_stride`."""
    r = int(load().scc_depthwise3x3_out(int(size), int(dw_stride)))
    _check(min(r, 0))
    return r


def scc_depthwise3x3_forward(x, kdw, dw_stride=1, out=None):
    """z = DW3x3(x; kdw): x [N,C,H,W], kdw [C,3,3] -> z [N,C,Ho,Wo] (Eq. 2: centred taps, zero outside the map)."""
    dev = _dev(x, kdw)
    N, C, H, W = x.shape
    if kdw.dtype != x.dtype or tuple(kdw.shape) != (C, 3, 3):
        raise ValueError("kdw must be [C, 3, 3] with the dtype of x")
    Ho, Wo = scc_depthwise3x3_out(H, dw_stride), scc_depthwise3x3_out(W, dw_stride)
    z = torch.empty((N, C, Ho, Wo), dtype=x.dtype, device=dev) if out is None else out
    if out is not None:
        _dev(out)
        assert out.shape == (N, C, Ho, Wo) and out.dtype == x.dtype
    with torch.cuda.device(dev):
        _check(load().scc_depthwise3x3_forward(x.data_ptr(), kdw.data_ptr(), z.data_ptr(), N, C, H, W, int(dw_stride),
                                               _dtype_code(x), _stream(dev)))
    return z


def scc_depthwise3x3_backward(x, kdw, dz, dw_stride=1, need_dx=True, need_dk=True, out_dx=None, out_dk=None,
                              workspace=None):
    """(dx, dkdw) of the depthwise 3x3 stage: x [N,C,H,W], kdw [C,3,3], dz [N,C,Ho,Wo] -> dx like x, dkdw [C,3,3] float32.
    A gradient that is not needed comes back as None."""
    dev = _dev(x, kdw, dz)
    N, C, H, W = x.shape
    Ho, Wo = scc_depthwise3x3_out(H, dw_stride), scc_depthwise3x3_out(W, dw_stride)
    if kdw.dtype != x.dtype or tuple(kdw.shape) != (C, 3, 3):
        raise ValueError("kdw must be [C, 3, 3] with the dtype of x")
    if dz.dtype != x.dtype or tuple(dz.shape) != (N, C, Ho, Wo):
        raise ValueError("dz must be [N, C, Ho, Wo] with the dtype of x")
    if not (need_dx or need_dk):
        return None, None
    code = _dtype_code(x)
    need = int(load().scc_depthwise3x3_backward_workspace_bytes(N, C, H, W, int(dw_stride), code)) if need_dk else 0
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    dx = (torch.empty_like(x) if out_dx is None else out_dx) if need_dx else None
    dk = (torch.empty((C, 3, 3), dtype=torch.float32, device=dev) if out_dk is None else out_dk) if need_dk else None
    for o, shp, dt in ((out_dx, x.shape, x.dtype), (out_dk, (C, 3, 3), torch.float32)):
        if o is not None:
            _dev(o)
            assert o.shape == shp and o.dtype == dt
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        _check(load().scc_depthwise3x3_backward(x.data_ptr(), kdw.data_ptr(), dz.data_ptr(),
                                                dx.data_ptr() if dx is not None else None,
                                                dk.data_ptr() if dk is not None else None, N, C, H, W, int(dw_stride),
                                                code, ws_ptr, ws_len, _stream(dev)))
    return dx, dk


def scc_dw_forward_workspace_bytes(N, Cin, Cout, H, W, dw_stride, cg, co, dtype=torch.float32):
    code = SCC_F32 if dtype == torch.float32 else SCC_BF16
    return int(load().scc_dw_forward_workspace_bytes(N, Cin, Cout, H, W, int(dw_stride), cg, float(co), code))


def scc_dw_forward_fusable(N, Cin, Cout, H, W, dw_stride, cg, co, dtype=torch.float32):
    """True when the fused kernel can run the layer (it then also runs without a workspace)."""
    code = SCC_F32 if dtype == torch.float32 else SCC_BF16
    r = int(load().scc_dw_forward_fusable(N, Cin, Cout, H, W, int(dw_stride), cg, float(co), code))
    _check(min(r, 0))
    return r == 1


def scc_dw_forward(x, kdw, w, cg, co, dw_stride=1, out=None, workspace=None, fused=None):
    """y = SCC(DW3x3(x; kdw); w), the forward of a DW + SCC block: x [N,Cin,H,W], kdw [Cin,3,3], w [Cout,Cin//cg]
    -> y [N,Cout,Ho,Wo].  fused=None: the path the library prefers (a workspace is allocated when it asks for
    one); fused=True: no workspace is passed, so the fused kernel runs or the call is refused; fused=False: the
    two stages through a workspace, also where the library would fuse."""
    dev = _dev(x, kdw, w)
    N, Cin, H, W = x.shape
    Cout = w.shape[0]
    if kdw.dtype != x.dtype or tuple(kdw.shape) != (Cin, 3, 3):
        raise ValueError("kdw must be [Cin, 3, 3] with the dtype of x")
    if w.dtype != x.dtype or w.dim() != 2 or (cg >= 1 and Cin % cg == 0 and w.shape[1] != Cin // cg):
        raise ValueError("w must be [Cout, Cin//cg] with the dtype of x")
    Ho, Wo = scc_depthwise3x3_out(H, dw_stride), scc_depthwise3x3_out(W, dw_stride)
    if fused is False:
        z = scc_depthwise3x3_forward(x, kdw, dw_stride)
        return scc_forward(z, w, cg, co, out=out)
    code = _dtype_code(x)
    need = int(load().scc_dw_forward_workspace_bytes(N, Cin, Cout, H, W, int(dw_stride), cg, float(co), code))
    if fused:
        workspace = None
    elif workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    y = torch.empty((N, Cout, Ho, Wo), dtype=x.dtype, device=dev) if out is None else out
    if out is not None:
        _dev(out)
        assert out.shape == (N, Cout, Ho, Wo) and out.dtype == x.dtype
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        _check(load().scc_dw_forward(x.data_ptr(), kdw.data_ptr(), w.data_ptr(), y.data_ptr(), N, Cin, Cout, H, W,
                                     int(dw_stride), cg, float(co), code, ws_ptr, ws_len, _stream(dev)))
    return y
