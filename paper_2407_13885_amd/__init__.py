"""attnw: attention weights P = softmax(scale * Q K^T) on MI355X (gfx950).

The compute lives in ``libattnw.so`` (hand-written HIP, C ABI declared in
``include/attnw.h``); ``binding`` marshals arguments for it and nothing else.
Importing the package does not load the library; the first call does, and it
raises if the library has not been built - there is no CPU fallback.
"""
from .binding import (  # noqa: F401
    ATTNW_BF16,
    ATTNW_F32,
    AttnwError,
    attnw_attention,
    attnw_fused,
    attnw_gemm_scores,
    attnw_scale,
    attnw_softmax,
    attnw_softmax_cast,
    attnw_status_string,
    attnw_version,
    build,
    library_path,
    load_library,
)
