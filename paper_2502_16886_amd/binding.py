"""ctypes binding of librfkv.so -- argument marshalling only.

The functions have the names and meanings of the C entry points in include/rfkv.h.
torch is used for device memory (`torch.empty`, `data_ptr`) and the current HIP
stream; every step of the computation runs inside the library's kernels.  There
is no fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

RFKV_OK = 0
RFKV_INVALID_ARG = 1
RFKV_UNSUPPORTED = 2
RFKV_WORKSPACE_TOO_SMALL = 3
RFKV_OUTPUT_TOO_SMALL = 4
RFKV_DEVICE_ERROR = 5
STATIC_SCRATCH_BYTES = 16 * 1024 * 1024

RANK_POSITION = 0
RANK_SCORE = 1
DTYPE_FP32 = 0
DTYPE_BF16 = 1
PER_HEAD = 0
PER_LAYER = 1

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "librfkv.so")


class RfkvParams(ctypes.Structure):
    """Mirror of `rfkv_params`."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("window", ctypes.c_int32), ("n_sink", ctypes.c_int32),
        ("threshold", ctypes.c_float), ("rank_mode", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("min_keep", ctypes.c_int32), ("granularity", ctypes.c_int32),
        ("k_stride_tok", ctypes.c_int64), ("k_stride_head", ctypes.c_int64),
        ("v_stride_tok", ctypes.c_int64), ("v_stride_head", ctypes.c_int64),
        ("q_stride_row", ctypes.c_int64), ("q_stride_head", ctypes.c_int64),
        ("out_pad_rows", ctypes.c_int64),
    ]


class RfkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def load_library() -> ctypes.CDLL:
    """dlopen librfkv.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2502_16886_amd.build` "
            "(there is no CPU fallback for the compression pass)")
    # torch ships its own HIP runtime; it has to be in the process before librfkv.so is mapped, or
    # the library binds to a second copy of the runtime and its launches fail on torch's streams
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(RfkvParams)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    lib.rfkv_version.restype = i32
    lib.rfkv_version.argtypes = []
    lib.rfkv_status_string.restype = ctypes.c_char_p
    lib.rfkv_status_string.argtypes = [ctypes.c_int]
    lib.rfkv_last_device_error.restype = i32
    lib.rfkv_last_device_error.argtypes = []
    lib.rfkv_workspace_bytes.restype = sz
    lib.rfkv_workspace_bytes.argtypes = [P, i64, i32]
    lib.rfkv_score.restype = ctypes.c_int
    lib.rfkv_score.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.rfkv_select.restype = ctypes.c_int
    lib.rfkv_select.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.rfkv_compact.restype = ctypes.c_int
    lib.rfkv_compact.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp]
    lib.rfkv_compress_layer.restype = ctypes.c_int
    lib.rfkv_compress_layer.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, sz, vp]
    lib.rfkv_layers_workspace_bytes.restype = sz
    lib.rfkv_layers_workspace_bytes.argtypes = [P, i32, i64, i32]
    lib.rfkv_compress_layers.restype = ctypes.c_int
    lib.rfkv_compress_layers.argtypes = [P, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, sz, vp]
    lib.rfkv_compress_layer_static.restype = ctypes.c_int
    lib.rfkv_compress_layer_static.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp]
    lib.rfkv_compress_layer_timed.restype = ctypes.c_int
    lib.rfkv_compress_layer_timed.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, sz, vp, vp]
    lib.rfkv_score_lse.restype = ctypes.c_int
    lib.rfkv_score_lse.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.rfkv_compress_layer_lse.restype = ctypes.c_int
    lib.rfkv_compress_layer_lse.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, sz, vp]
    lib.rfkv_decode_workspace_bytes.restype = sz
    lib.rfkv_decode_workspace_bytes.argtypes = [P, i32, i32]
    lib.rfkv_decode_attention.restype = ctypes.c_int
    lib.rfkv_decode_attention.argtypes = [P, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.rfkv_masked_attention.restype = ctypes.c_int
    lib.rfkv_masked_attention.argtypes = [P, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    _lib = lib
    return lib


EXPORTED_SYMBOLS = ("rfkv_version", "rfkv_status_string", "rfkv_last_device_error", "rfkv_workspace_bytes",
                    "rfkv_score", "rfkv_select", "rfkv_compact", "rfkv_compress_layer",
                    "rfkv_compress_layer_static", "rfkv_layers_workspace_bytes", "rfkv_compress_layers",
                    "rfkv_compress_layer_timed", "rfkv_score_lse", "rfkv_compress_layer_lse",
                    "rfkv_decode_workspace_bytes", "rfkv_decode_attention", "rfkv_masked_attention")
KERNEL_NAMES = ("score_stats", "score_merge", "score_reduce", "select", "compact")


def status_string(status: int) -> str:
    return load_library().rfkv_status_string(int(status)).decode()


def rfkv_version() -> int:
    return int(load_library().rfkv_version())


def rfkv_last_device_error() -> int:
    return int(load_library().rfkv_last_device_error())


def rfkv_workspace_bytes(params: RfkvParams, total_tokens: int, max_seqlen: int) -> int:
    return int(load_library().rfkv_workspace_bytes(ctypes.byref(params), int(total_tokens), int(max_seqlen)))


def _ptr(x) -> int | None:
    """Address of a torch tensor / numpy array / raw int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return x.ctypes.data           # numpy (host)


def _stream(stream) -> int | None:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(status: int, where: str, check: bool) -> int:
    if check and status != RFKV_OK:
        raise RfkvError(status, where)
    return status


def rfkv_score(params, q_win, k, cu_host, cu_dev, scores, ws, ws_bytes, stream=None, check=True) -> int:
    st = load_library().rfkv_score(ctypes.byref(params), _ptr(q_win), _ptr(k), _ptr(cu_host), _ptr(cu_dev),
                                   _ptr(scores), _ptr(ws), int(ws_bytes), _stream(stream))
    return _check(st, "rfkv_score", check)


def rfkv_score_lse(params, q_win, lse_win, k, cu_host, cu_dev, scores, ws, ws_bytes, stream=None, check=True) -> int:
    st = load_library().rfkv_score_lse(ctypes.byref(params), _ptr(q_win), _ptr(lse_win), _ptr(k), _ptr(cu_host),
                                       _ptr(cu_dev), _ptr(scores), _ptr(ws), int(ws_bytes), _stream(stream))
    return _check(st, "rfkv_score_lse", check)


def rfkv_select(params, scores, cu_host, cu_dev, kept, out_offsets, idx, ws, ws_bytes, stream=None,
                check=True) -> int:
    st = load_library().rfkv_select(ctypes.byref(params), _ptr(scores), _ptr(cu_host), _ptr(cu_dev), _ptr(kept),
                                    _ptr(out_offsets), _ptr(idx), _ptr(ws), int(ws_bytes), _stream(stream))
    return _check(st, "rfkv_select", check)


def rfkv_compact(params, k, v, cu_host, cu_dev, kept, out_offsets, idx, k_out, v_out, out_capacity_rows,
                 stream=None, check=True) -> int:
    st = load_library().rfkv_compact(ctypes.byref(params), _ptr(k), _ptr(v), _ptr(cu_host), _ptr(cu_dev),
                                     _ptr(kept), _ptr(out_offsets), _ptr(idx), _ptr(k_out), _ptr(v_out),
                                     int(out_capacity_rows), _stream(stream))
    return _check(st, "rfkv_compact", check)


def rfkv_compress_layer(params, q_win, k, v, cu_host, cu_dev, scores_opt, kept, out_offsets, idx_opt, k_out,
                        v_out, out_capacity_rows, ws, ws_bytes, stream=None, check=True) -> int:
    st = load_library().rfkv_compress_layer(ctypes.byref(params), _ptr(q_win), _ptr(k), _ptr(v), _ptr(cu_host),
                                            _ptr(cu_dev), _ptr(scores_opt), _ptr(kept), _ptr(out_offsets),
                                            _ptr(idx_opt), _ptr(k_out), _ptr(v_out), int(out_capacity_rows),
                                            _ptr(ws), int(ws_bytes), _stream(stream))
    return _check(st, "rfkv_compress_layer", check)


def _ptr_array(items, n):
    """Host array of n addresses (None for a NULL array)."""
    if items is None:
        return None
    assert len(items) == n
    arr = (ctypes.c_void_p * n)(*[_ptr(x) for x in items])
    return arr


def rfkv_layers_workspace_bytes(params, n_layers: int, total_tokens: int, max_seqlen: int) -> int:
    return int(load_library().rfkv_layers_workspace_bytes(ctypes.byref(params), int(n_layers), int(total_tokens),
                                                          int(max_seqlen)))


def rfkv_compress_layers(params, q_win, k, v, cu_host, cu_dev, scores_opt, kept, out_offsets, idx_opt, k_out, v_out,
                         out_capacity_rows, ws, ws_bytes, stream=None, check=True) -> int:
    """q_win, k, ... are sequences of per-layer tensors (scores_opt / idx_opt may be None)."""
    n = len(k)
    arrays = [_ptr_array(x, n) for x in (q_win, k, v)]
    outs = [_ptr_array(x, n) for x in (scores_opt, kept, out_offsets, idx_opt, k_out, v_out)]
    st = load_library().rfkv_compress_layers(ctypes.byref(params), n, arrays[0], arrays[1], arrays[2], _ptr(cu_host),
                                             _ptr(cu_dev), outs[0], outs[1], outs[2], outs[3], outs[4], outs[5],
                                             int(out_capacity_rows), _ptr(ws), int(ws_bytes), _stream(stream))
    return _check(st, "rfkv_compress_layers", check)


def rfkv_compress_layer_static(params, q_win, k, v, cu_host, cu_dev, scores_opt, kept, out_offsets, idx_opt, k_out,
                               v_out, out_capacity_rows, stream=None, check=True) -> int:
    st = load_library().rfkv_compress_layer_static(ctypes.byref(params), _ptr(q_win), _ptr(k), _ptr(v),
                                                   _ptr(cu_host), _ptr(cu_dev), _ptr(scores_opt), _ptr(kept),
                                                   _ptr(out_offsets), _ptr(idx_opt), _ptr(k_out), _ptr(v_out),
                                                   int(out_capacity_rows), _stream(stream))
    return _check(st, "rfkv_compress_layer_static", check)


def rfkv_compress_layer_lse(params, q_win, lse_win, k, v, cu_host, cu_dev, scores_opt, kept, out_offsets, idx_opt,
                            k_out, v_out, out_capacity_rows, ws, ws_bytes, stream=None, check=True) -> int:
    st = load_library().rfkv_compress_layer_lse(ctypes.byref(params), _ptr(q_win), _ptr(lse_win), _ptr(k), _ptr(v),
                                                _ptr(cu_host), _ptr(cu_dev), _ptr(scores_opt), _ptr(kept),
                                                _ptr(out_offsets), _ptr(idx_opt), _ptr(k_out), _ptr(v_out),
                                                int(out_capacity_rows), _ptr(ws), int(ws_bytes), _stream(stream))
    return _check(st, "rfkv_compress_layer_lse", check)


def rfkv_compress_layer_timed(params, q_win, k, v, cu_host, cu_dev, scores_opt, kept, out_offsets, idx_opt,
                              k_out, v_out, out_capacity_rows, ws, ws_bytes, stream=None, check=True):
    """Returns (status, [ms per kernel in KERNEL_NAMES order]); synchronises the stream."""
    ms = (ctypes.c_float * len(KERNEL_NAMES))()
    st = load_library().rfkv_compress_layer_timed(
        ctypes.byref(params), _ptr(q_win), _ptr(k), _ptr(v), _ptr(cu_host), _ptr(cu_dev), _ptr(scores_opt),
        _ptr(kept), _ptr(out_offsets), _ptr(idx_opt), _ptr(k_out), _ptr(v_out), int(out_capacity_rows), _ptr(ws),
        int(ws_bytes), _stream(stream), ctypes.cast(ms, ctypes.c_void_p))
    return _check(st, "rfkv_compress_layer_timed", check), list(ms)


def rfkv_decode_workspace_bytes(params, n_new: int, max_seqlen: int) -> int:
    return int(load_library().rfkv_decode_workspace_bytes(ctypes.byref(params), int(n_new), int(max_seqlen)))


def rfkv_decode_attention(params, q_new, n_new, k_c, v_c, cu_host, out_offsets, kept_opt, out, ws, ws_bytes,
                          stream=None, check=True) -> int:
    st = load_library().rfkv_decode_attention(ctypes.byref(params), _ptr(q_new), int(n_new), _ptr(k_c), _ptr(v_c),
                                              _ptr(cu_host), _ptr(out_offsets), _ptr(kept_opt), _ptr(out), _ptr(ws),
                                              int(ws_bytes), _stream(stream))
    return _check(st, "rfkv_decode_attention", check)


def rfkv_masked_attention(params, q_new, n_new, k, v, cu_host, cu_dev, keep_mask, out, ws, ws_bytes, stream=None,
                          check=True) -> int:
    st = load_library().rfkv_masked_attention(ctypes.byref(params), _ptr(q_new), int(n_new), _ptr(k), _ptr(v),
                                              _ptr(cu_host), _ptr(cu_dev), _ptr(keep_mask), _ptr(out), _ptr(ws),
                                              int(ws_bytes), _stream(stream))
    return _check(st, "rfkv_masked_attention", check)


# ----------------------------------------------------------------------------
# convenience: parameter struct for contiguous [N, Hkv, d] / [rows, Hq, d] tensors
# ----------------------------------------------------------------------------
def make_params(batch, n_q_heads, n_kv_heads, head_dim, window, dtype, n_sink=4, threshold=0.01,
                rank_mode=RANK_POSITION, softmax_scale=0.0, min_keep=0, granularity=PER_HEAD,
                out_pad_rows=0) -> RfkvParams:
    p = RfkvParams()
    p.batch, p.n_q_heads, p.n_kv_heads, p.head_dim = batch, n_q_heads, n_kv_heads, head_dim
    p.window, p.n_sink, p.threshold, p.rank_mode = window, n_sink, threshold, rank_mode
    p.dtype = DTYPE_BF16 if dtype in ("bf16", DTYPE_BF16) else DTYPE_FP32
    p.softmax_scale, p.min_keep = softmax_scale, min_keep
    p.granularity, p.out_pad_rows = granularity, out_pad_rows
    p.k_stride_tok = p.v_stride_tok = n_kv_heads * head_dim
    p.k_stride_head = p.v_stride_head = head_dim
    p.q_stride_row = n_q_heads * head_dim
    p.q_stride_head = head_dim
    return p


@dataclass
class LayerBuffers:
    """Device buffers for one rfkv_compress_layer call (all owned by the caller)."""
    scores: object
    kept: object
    out_offsets: object
    idx: object
    k_out: object
    v_out: object
    ws: object
    ws_bytes: int
    capacity_rows: int


def alloc_layer_buffers(params: RfkvParams, total_tokens: int, max_seqlen: int, device="cuda",
                        capacity_rows: int | None = None) -> LayerBuffers:
    import torch
    units = params.batch * params.n_kv_heads
    rows = total_tokens * params.n_kv_heads if capacity_rows is None else capacity_rows
    if params.out_pad_rows > 0 and capacity_rows is None:       # padded layout: a fixed slot per unit
        rows = units * params.out_pad_rows
    tdt = torch.bfloat16 if params.dtype == DTYPE_BF16 else torch.float32
    ws_bytes = rfkv_workspace_bytes(params, total_tokens, max_seqlen)
    if ws_bytes == 0 and total_tokens > 0:
        raise RfkvError(RFKV_UNSUPPORTED, "rfkv_workspace_bytes")
    return LayerBuffers(
        scores=torch.empty((params.n_kv_heads, total_tokens), dtype=torch.float32, device=device),
        kept=torch.empty(units, dtype=torch.int32, device=device),
        out_offsets=torch.empty(units + 1, dtype=torch.int64, device=device),
        idx=torch.empty(max(1, total_tokens * params.n_kv_heads, rows if params.out_pad_rows > 0 else 0),
                        dtype=torch.int32, device=device),
        k_out=torch.empty((max(1, rows), params.head_dim), dtype=tdt, device=device),
        v_out=torch.empty((max(1, rows), params.head_dim), dtype=tdt, device=device),
        ws=torch.empty(max(256, ws_bytes), dtype=torch.uint8, device=device),
        ws_bytes=ws_bytes, capacity_rows=rows)
