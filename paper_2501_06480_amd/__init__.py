"""Flash Window Attention hot path for MI355X (gfx950).

``binding`` is the thin ctypes layer over the C-ABI library built from
``csrc/`` (hand-written HIP); ``autograd`` wraps its calls as differentiable torch
functions (imported on demand: ``from paper_2501_06480_amd import autograd``);
``synth`` draws seeded synthetic workloads.
Nothing here computes attention on the CPU: if the HIP library is missing,
calls fail loudly.
"""
from . import synth  # noqa: F401
from .binding import (  # noqa: F401
    FwaError, fwa_forward, fwa_backward, fwa_backward_noalloc, fwa_backward_workspace_bytes, fwa_bias_gather,
    fwa_bias_scatter, fwa_status_string, library_path, load_library,
)
