"""Device plumbing around librfkv: move a synthetic layer (workloads.Layer) to the GPU with torch,
allocate the caller-owned buffers and call rfkv_compress_layer through the ctypes binding.  Holds
none of the method's arithmetic; used by the benchmark, the smoke check and the GPU tests."""
from __future__ import annotations

import numpy as np

from . import binding as B
from . import workloads as W


def to_device(arr: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def to_host_bits(t, dtype: str) -> np.ndarray:
    import torch
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class DeviceLayer:
    """Inputs of one layer resident on the GPU plus the parameter struct."""

    def __init__(self, layer: W.Layer, rank_mode=B.RANK_POSITION, threshold=None, min_keep=0, n_sink=None,
                 kv_layout="token_major", granularity=B.PER_HEAD, out_pad_rows=0):
        import torch
        c = layer.cfg
        self.layer = layer
        self.dtype = c.dtype
        self.q = to_device(layer.q_win, c.dtype)
        self.k = to_device(layer.k, c.dtype)
        self.v = to_device(layer.v, c.dtype)
        self.cu_host = np.ascontiguousarray(layer.cu_seqlens, dtype=np.int32)
        self.cu_dev = torch.from_numpy(self.cu_host).cuda()
        self.batch = len(self.cu_host) - 1
        self.N = int(self.cu_host[-1])
        self.max_len = int(np.diff(self.cu_host).max()) if self.batch else 0
        self.params = B.make_params(self.batch, c.n_q_heads, c.n_kv_heads, c.head_dim, c.window, c.dtype,
                                    n_sink=c.n_sink if n_sink is None else n_sink,
                                    threshold=c.threshold if threshold is None else threshold,
                                    rank_mode=rank_mode, min_keep=min_keep, granularity=granularity,
                                    out_pad_rows=out_pad_rows)
        self.kv_layout = kv_layout
        if kv_layout == "head_major":
            # [Hkv, N, d]: each head's rows contiguous (for one sequence, the [B, H, n, d] cache layout)
            self.k = self.k.permute(1, 0, 2).contiguous()
            self.v = self.v.permute(1, 0, 2).contiguous()
            self.params.k_stride_tok = self.params.v_stride_tok = c.head_dim
            self.params.k_stride_head = self.params.v_stride_head = max(self.N, 1) * c.head_dim
        else:
            assert kv_layout == "token_major"          # [N, Hkv, d]
        self.buf = B.alloc_layer_buffers(self.params, self.N, self.max_len)

    def compress(self, stream=None, lse_win=None, keep_whole=False):
        """One fused pass; with `lse_win` (device float32 [window rows, Hq]) through rfkv_compress_layer_lse.
        `keep_whole`: the layer keeps its whole cache (threshold 0, no scores asked for, no queries
        handed over): the library scores nothing and only re-lays the cache out per unit."""
        b = self.buf
        if keep_whole:
            p = B.RfkvParams.from_buffer_copy(self.params)
            p.threshold = 0.0
            return B.rfkv_compress_layer(p, None, self.k, self.v, self.cu_host, self.cu_dev, None, b.kept,
                                         b.out_offsets, b.idx, b.k_out, b.v_out, b.capacity_rows, b.ws, b.ws_bytes,
                                         stream)
        if lse_win is not None:
            return B.rfkv_compress_layer_lse(self.params, self.q, lse_win, self.k, self.v, self.cu_host, self.cu_dev,
                                             b.scores, b.kept, b.out_offsets, b.idx, b.k_out, b.v_out,
                                             b.capacity_rows, b.ws, b.ws_bytes, stream)
        return B.rfkv_compress_layer(self.params, self.q, self.k, self.v, self.cu_host, self.cu_dev, b.scores,
                                     b.kept, b.out_offsets, b.idx, b.k_out, b.v_out, b.capacity_rows, b.ws,
                                     b.ws_bytes, stream)

    def results(self) -> dict:
        import torch
        torch.cuda.synchronize()
        b = self.buf
        offs = b.out_offsets.cpu().numpy()
        total = int(offs[-1])
        return dict(scores=b.scores.cpu().numpy(), kept=b.kept.cpu().numpy().astype(np.int64), out_offsets=offs,
                    idx=b.idx[:total].cpu().numpy().astype(np.int64),
                    k_out=to_host_bits(b.k_out[:total], self.dtype), v_out=to_host_bits(b.v_out[:total], self.dtype))


class LayerSet:
    """Several layers of one prefilled batch (same shapes, strides and sequence lengths, each with its own
    buffers) and the scratch of one rfkv_compress_layers call over all of them."""

    def __init__(self, dls):
        import torch
        self.dls = list(dls)
        d0 = self.dls[0]
        assert all(np.array_equal(d.cu_host, d0.cu_host) for d in self.dls)
        self.ws_bytes = B.rfkv_layers_workspace_bytes(d0.params, len(self.dls), d0.N, d0.max_len)
        self.ws = torch.empty(max(256, self.ws_bytes), dtype=torch.uint8, device="cuda")

    def compress(self, stream=None, with_scores=True, with_idx=True):
        d0 = self.dls[0]
        bufs = [d.buf for d in self.dls]
        return B.rfkv_compress_layers(d0.params, [d.q for d in self.dls], [d.k for d in self.dls],
                                      [d.v for d in self.dls], d0.cu_host, d0.cu_dev,
                                      [b.scores for b in bufs] if with_scores else None, [b.kept for b in bufs],
                                      [b.out_offsets for b in bufs], [b.idx for b in bufs] if with_idx else None,
                                      [b.k_out for b in bufs], [b.v_out for b in bufs], bufs[0].capacity_rows,
                                      self.ws, self.ws_bytes, stream)


def compress_model(layers, n_frozen: int = 2, stream=None) -> None:
    """Alg. 1's loop over the layers of a prefilled model with Sec. 3.3 "Retaining Bottom Layers":
    the first `n_frozen` layers keep their whole cache, every other layer is compressed.  `layers`:
    DeviceLayer objects in layer order; each one's buffers hold its result afterwards."""
    for i, dl in enumerate(layers):
        dl.compress(stream, keep_whole=i < n_frozen)


def threshold_as_float32(T: float) -> float:
    """The library takes T as a float; the oracle must be given the same number."""
    return float(np.float32(T))


def unit_slices(layer: W.Layer):
    """(unit, b, h, first packed token, end packed token) for every (sequence, KV head)."""
    Hkv = layer.cfg.n_kv_heads
    cu = layer.cu_seqlens
    for b in range(len(cu) - 1):
        for h in range(Hkv):
            yield b * Hkv + h, b, h, int(cu[b]), int(cu[b + 1])

