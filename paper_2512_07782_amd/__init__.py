"""GatedFWA (memory-gated sliding-window softmax attention) for AMD MI355X.

Thin Python binding over the C ABI of `libgfwa.so` (see `include/gfwa.h`).  The binding only
marshals arguments: every step of the path runs in the HIP kernels.  PyTorch is used for device
memory and streams.
"""
from .binding import (  # noqa: F401
    GfwaError,
    gfwa_backward,
    gfwa_backward_gqa,
    gfwa_backward_fast_workspace_bytes,
    gfwa_backward_workspace_bytes,
    gfwa_decode,
    gfwa_decode_static,
    gfwa_decode_workspace_bytes,
    gfwa_forward,
    gfwa_forward_gqa,
    gfwa_gate_activation_backward,
    gfwa_gate_activation_prefix,
    gfwa_gate_prefix,
    gfwa_gate_prefix_stp,
    gfwa_gate_scan_workspace_bytes,
    gfwa_probe_copy,
    gfwa_probe_mfma,
    gfwa_profile_enable,
    gfwa_profile_kernel_name,
    gfwa_profile_read,
    gfwa_strerror,
    gfwa_version,
    lib_path,
    load_library,
)
