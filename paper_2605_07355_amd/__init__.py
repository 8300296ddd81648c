"""Temporal Token Fusion (TTF) for AMD Instinct MI355X.

Thin Python binding over the C-ABI library ``libttf.so`` (hand-written HIP kernels for
gfx950).  PyTorch is used for device memory and streams only; every step of the pass runs in
the library's kernels.  There is no CPU or PyTorch fallback: if the library is missing the
import of :mod:`paper_2605_07355_amd.binding` functions raises.
"""
from .binding import (  # noqa: F401
    TTFError,
    TTFOutput,
    TTFBuffers,
    STAGE_NAMES,
    library_path,
    load_library,
    ttf_compress,
    ttf_compress_static,
    TTF_STATIC_WORKSPACE_BYTES,
    ttf_workspace_size,
    ttf_status_string,
    ttf_last_hip_error,
    ttf_compress_segment,
    TTFTiedBuffers,
    ttf_compress_tied,
    ttf_tied_workspace_size,
    ttf_restore_map,
    ttf_restore,
    ttf_decode_alignment,
    ttf_select_threshold,
    ttf_regate,
    ttf_set_speculation,
    ttf_search_route,
    ttf_profile_enable,
    ttf_profile_read,
)
