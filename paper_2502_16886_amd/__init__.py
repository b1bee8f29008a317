"""rfkv: ReFreeKV's threshold-free KV-cache compression pass for AMD MI355X (gfx950).

`binding` exposes the C ABI of librfkv.so (include/rfkv.h); `workloads` makes the
seeded synthetic inputs; `device` moves a layer to the GPU and calls the library;
`build` compiles the library with hipcc.
"""
from . import binding, workloads  # noqa: F401
from .binding import (RfkvError, RfkvParams, make_params, rfkv_compact, rfkv_compress_layer,  # noqa: F401
                      rfkv_decode_attention, rfkv_decode_workspace_bytes, rfkv_masked_attention, rfkv_score,
                      rfkv_select, rfkv_version, rfkv_workspace_bytes)
