"""MI355X (gfx950) depthwise 1-D convolution: forward, input gradient and weight gradient
of the S4ConvD operator (Sec. IV-A of the paper), as hand-written HIP kernels behind a C ABI.

``binding`` marshals torch GPU tensors into the C ABI; ``workloads`` draws the seeded synthetic
inputs; ``roofline`` holds the byte/flop bookkeeping and the parity metric.
"""
from .binding import (  # noqa: F401
    BF16, F32, DwconvError, dwconv_bwd_input, dwconv_bwd_weight, dwconv_bwd_weight_finalize,
    dwconv_bwd_weight_partial, dwconv_bwd_weight_slices, dwconv_bwd_weight_workspace_bytes, dwconv_fwd,
    new_workspace, status_string,
)
