"""MI355X-native sliding-channel convolution (DSXplore, Section 3.1 / 4.2): forward,
grad-input and grad-weight of one SCC layer as gfx950 HIP kernels behind a C ABI."""
from .scc import (SCC_BF16, SCC_F32, SccError, load, scc_backward, scc_backward_input, scc_backward_workspace_bytes, scc_backward_weight, scc_backward_weight_static,
                  scc_backward_weight_workspace_bytes, scc_depthwise3x3_backward, scc_depthwise3x3_forward, scc_depthwise3x3_out, scc_dw_forward, scc_dw_forward_fusable, scc_dw_forward_workspace_bytes,
                  scc_forward, scc_status_string, scc_window_params)

__all__ = ["SCC_F32", "SCC_BF16", "SccError", "load", "scc_forward", "scc_backward", "scc_backward_workspace_bytes", "scc_backward_input", "scc_backward_weight", "scc_backward_weight_static",
           "scc_backward_weight_workspace_bytes", "scc_status_string", "scc_window_params", "scc_depthwise3x3_forward", "scc_depthwise3x3_backward",
           "scc_depthwise3x3_out", "scc_dw_forward", "scc_dw_forward_fusable", "scc_dw_forward_workspace_bytes"]
