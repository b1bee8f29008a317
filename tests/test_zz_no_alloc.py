"""The entry point that allocates nothing (rfkv_compress_layer_static: its scratch is a fixed array in
the library's device image) against rfkv_compress_layer with a caller-owned workspace: same bits, on
two calls in a row, the second with a smaller input, so that whatever the first call left in the shared
array must not leak into the second."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import rfkv_harness as H                                   # noqa: E402
from paper_2502_16886_amd import binding as B              # noqa: E402
from paper_2502_16886_amd import workloads as W            # noqa: E402

pytestmark = pytest.mark.gpu
KEYS = ("scores", "kept", "out_offsets", "idx", "k_out", "v_out")


def _both(layer, mode, **kw):
    import torch
    dl = H.DeviceLayer(layer, rank_mode=mode, **kw)
    dl.compress()
    ref = dl.results()
    b = dl.buf
    for t in (b.scores, b.kept, b.out_offsets, b.idx, b.k_out, b.v_out):
        t.zero_()
    before = torch.cuda.memory_allocated()
    B.rfkv_compress_layer_static(dl.params, dl.q, dl.k, dl.v, dl.cu_host, dl.cu_dev, b.scores, b.kept, b.out_offsets,
                                 b.idx, b.k_out, b.v_out, b.capacity_rows)
    assert torch.cuda.memory_allocated() == before
    got = dl.results()
    for key in KEYS:
        assert np.array_equal(got[key], ref[key]), key
    return ref


@pytest.mark.parametrize("mode", [B.RANK_POSITION, B.RANK_SCORE])
def test_static_scratch_entry_point_matches_the_workspace_one(mode):
    big = W.Config("t", 1, 32, 8, 128, 32, "bf16", batch=2, context=6000)
    first = _both(W.make_layer(1, 3, cfg=big, lengths=[6000, 2500]), mode)
    small = W.Config("t", 1, 8, 2, 128, 32, "bf16", batch=3, context=900)
    second = _both(W.make_layer(1, 4, cfg=small, lengths=[900, 1, 411]), mode)
    assert first["kept"].sum() > second["kept"].sum() > 0
    # the paper's k = 1 (kept logits in the scratch) and the wide-window kernels (row-blocked statistics)
    _both(W.make_layer(1, 5, cfg=W.Config("t", 1, 32, 8, 128, 1, "bf16", batch=1, context=3000), lengths=[3000]), mode)
    _both(W.make_layer(1, 6, cfg=W.Config("t", 1, 28, 4, 128, 32, "bf16", batch=1, context=1500), lengths=[1500]), mode)


def test_static_scratch_rejects_what_does_not_fit():
    import torch
    p = B.make_params(1, 32, 8, 128, 32, "bf16")
    n = 400000                                             # 400000 x 8 positions: 25 MB of index lists and scores
    assert B.rfkv_workspace_bytes(p, n, n) > B.STATIC_SCRATCH_BYTES
    cu = np.array([0, n], np.int32)
    t = torch.empty(4096, dtype=torch.uint8, device="cuda")
    st = B.rfkv_compress_layer_static(p, t, t, t, cu, t, None, t, t, None, t, t, n * 8, check=False)
    assert st == B.RFKV_WORKSPACE_TOO_SMALL
