"""MI355X (gfx950) implementation of the SVG-EAR attention hot path.

Thin ctypes binding over libsvgear.so (hand-written HIP kernels behind a C ABI, declared in
include/svgear.h). PyTorch is used only to own device memory and streams; every step of
the path runs inside the library. There is no CPU fallback: importing works anywhere,
calling any stage without the built library or without a GPU raises.
"""
from .binding import (  # noqa: F401
    SvgearError,
    lib_path,
    load_library,
    kmeans,
    permute,
    permute_rows,
    probe_route,
    sparse_attn_comp,
    unpermute,
    attention_layer,
    run_pair,
    EXPORTED_SYMBOLS,
    PROBE_PLAIN,
    ROUTE_PER_ROW,
    USE_GIVEN_SCORES,
)
