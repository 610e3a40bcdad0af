"""CPU oracle (test infrastructure only).

Plain C definition of what the sub-bit 3x3 convolution path computes, with a ctypes
wrapper.  Imported by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline
leg only.  It shares nothing with the HIP library and is never a fallback for it.
"""
from .oracle import (  # noqa: F401
    build,
    threads,
    decode,
    out_size,
    sign,
    pack_rows,
    pack_channels,
    expand,
    conv_bin,
    conv_sign,
    project_backward,
    subset_update,
    pack_indices,
    decode8,
    conv1x1_bin,
    project8,
    conv_f32,
    two_stage_bin,
    two_stage_f32,
    project,
)
