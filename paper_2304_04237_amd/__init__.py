"""MI355X-native Slide Attention operator (arxiv 2304.04237, Sec. 4).

A thin binding over libslide_attn.so (hand-written gfx950 HIP kernels behind a
C ABI, see include/slide_attn.h).  PyTorch is used for device memory and streams
only; every step of the operator runs in the library's kernels.  There is no
CPU fallback: importing works anywhere, calling needs the built library and a GPU.
"""
from .binding import (  # noqa: F401
    SlideAttnError,
    lib_path,
    load_library,
    slide_attn_bwd,
    slide_attn_bwd_nhwc,
    slide_attn_bwd_two_branch,
    slide_attn_fwd,
    slide_attn_fwd_nhwc,
    slide_attn_fwd_noalloc,
    slide_attn_fwd_two_branch,
    slide_attn_fwd_path,
    slide_attn_fwd_shift,
    slide_attn_fwd_traffic_probe,
    slide_attn_fwd_variant,
    slide_attn_bwd_variant,
    slide_attn_workspace_bytes,
    slide_reparam,
    slide_status_string,
)
