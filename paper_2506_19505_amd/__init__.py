"""AnTKV online path for AMD MI355X: thin Python binding over libantkv.so (hand-written HIP, gfx950).

Every step runs inside the HIP library; this package only marshals torch tensors (used for device
memory and streams) into the C ABI declared in include/antkv.h.  There is no CPU fallback: importing the
binding without a built library, or calling it without a GPU, raises.
"""
from .binding import (
    AntkvError,
    DecodeWorkspace,
    Geometry,
    anchor_select,
    append_token,
    prefill_attn,
    kmeans_step,
    decode_attn,
    decode_attn_prerope,
    decode_attn_prerope_workspace,
    decode_attn_static,
    DECODE_FIXED_ORDER,
    DECODE_WIDE_TABLE,
    set_decode_options,
    encode,
    gather_rows,
    lib_path,
    load_library,
    topk,
    version,
)

__all__ = [
    "AntkvError",
    "DecodeWorkspace",
    "Geometry",
    "anchor_select",
    "append_token",
    "prefill_attn",
    "kmeans_step",
    "decode_attn",
    "decode_attn_prerope",
    "decode_attn_prerope_workspace",
    "decode_attn_static",
    "DECODE_FIXED_ORDER",
    "DECODE_WIDE_TABLE",
    "set_decode_options",
    "encode",
    "gather_rows",
    "lib_path",
    "load_library",
    "topk",
    "version",
]
