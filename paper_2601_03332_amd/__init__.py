"""MI355X-native LUT-KAN layer forward (arxiv 2601.03332): thin Python binding over liblutkan.so.

Every step of the hot path runs in the HIP kernels of the C-ABI library; this package only marshals
arguments (torch tensors -> raw device pointers, the current HIP stream) and keeps buffers alive.
There is no CPU fallback: importing works anywhere, calling a forward without a GPU raises.
"""
from .binding import (  # noqa: F401
    ALGO_AUTO, ALGO_GATHER, ALGO_TILED, ALGO_TILED_WIDE, PARAM_FP32, PARAM_FP16, SPAN_DOMAIN, SPAN_EXTENDED, PROBE_VALU_FMA,
    PROBE_LDS_READ, PROBE_L2_READ, PROBE_HBM_READ, PROBE_VALU_MIX, PROBE_VALU_FMAC, ASYM_UINT8, CLIP_X, CLOSED, HALF_OPEN, REPR_PHI,
    REPR_SPLINE_COMPONENT, SYM_INT8, ZERO_SPLINE, Artifact, BsplineLayer, LutKanError, LutLayer,
    bspline_forward_workspace_bytes, bspline_kan_forward, library_path, lutkan_error_stats,
    lutkan_artifact_from_arrays, lutkan_artifact_load, lutkan_compile, lutkan_forward, lutkan_forward_edges,
    lutkan_forward_locate, lutkan_forward_trace, bspline_forward_edges, bspline_forward_locate,
    lutkan_forward_workspace_bytes, lutkan_last_error, lutkan_last_plan, lutkan_chain_forward, lutkan_model_forward,
    lutkan_model_workspace_bytes, lutkan_probe_launch, lutkan_version, load_library, lutkan_forward_static_scratch,
    STATIC_SCRATCH_BYTES,
)
