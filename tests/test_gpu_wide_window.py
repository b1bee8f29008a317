"""GPU parity of the wide-window scoring path (window * G beyond the streaming kernels' 512 rows: the
window sizes of the paper's ablation of k, 1 % .. 10 % of n) against the float64 oracle: scores,
selection in both rankings, compacted rows."""
import numpy as np
import pytest

import rfkv_harness as H
from oracle import refreekv_oracle as O
from paper_2502_16886_amd import binding as B
from paper_2502_16886_amd import workloads as W

pytestmark = pytest.mark.gpu


WIDE = [
    # (Hq, Hkv, d, dtype, window, lens)
    (8, 2, 128, "bf16", 300, [3000]),                 # 10 % of n, 1200 rows
    (28, 4, 128, "bf16", 200, [2000, 150, 700]),      # G = 7: 1400 rows; one sequence shorter than the window
    (4, 4, 64, "bf16", 600, [1300, 5, 601]),          # G = 1, d = 64
    (8, 2, 64, "fp32", 150, [900, 149]),              # fp32: 600 rows
    (4, 1, 128, "bf16", 1024, [700]),                 # window >= n: the whole causal attention matrix
    (32, 8, 128, "bf16", 129, [1111, 300]),           # 516 rows: just past the streaming kernels' limit
    (8, 2, 128, "bf16", 300, [0, 900, 0, 1]),         # empty sequences and a one-token sequence in a wide batch
    (8, 2, 128, "bf16", 40, [0, 333]),                # 160 rows (the smallest wide window) with an empty sequence
]


@pytest.mark.parametrize("case", WIDE, ids=lambda c: f"Hq{c[0]}_Hkv{c[1]}_d{c[2]}_{c[3]}_w{c[4]}")
@pytest.mark.parametrize("rank_mode", [B.RANK_POSITION, B.RANK_SCORE], ids=["position", "score"])
def test_wide_window_small_shapes(case, rank_mode):
    Hq, Hkv, d, dtype, w, lens = case
    cfg = W.Config("t", 1, Hq, Hkv, d, w, dtype, batch=len(lens), context=max(lens), threshold=0.02)
    layer = W.make_layer(3, 1, cfg=cfg, lengths=lens)
    dl = H.DeviceLayer(layer, rank_mode=rank_mode)
    dl.compress()
    rep = H.compare_layer(layer, dl.results(), rank_mode)
    print(rep)


def test_wide_window_rejections():
    import torch
    t = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")
    cu = np.array([0, 100], np.int32)
    p = B.make_params(1, 8, 2, 128, 300, "fp32")              # fp32 rows of 512 bytes
    st = B.rfkv_compress_layer(p, t, t, t, cu, t, None, t, t, None, t, t, 200, t, 1 << 16, check=False)
    assert st == B.RFKV_UNSUPPORTED
    p = B.make_params(1, 8, 2, 128, 20000, "bf16")            # 80000 rows
    st = B.rfkv_compress_layer(p, t, t, t, cu, t, None, t, t, None, t, t, 200, t, 1 << 16, check=False)
    assert st == B.RFKV_UNSUPPORTED


def test_wide_window_full_size_one_percent():
    """The headline shape (32 q / 8 kv heads, d = 128, n = 32768) with the ablation's k = 1 % of n
    (328 window positions, 1312 score rows per KV head): every score, the selection and the
    compacted rows against the oracle, in the launch configuration the benchmark times."""
    cfg = W.Config("llama3-8b-32k-w328", 32, 32, 8, 128, 328, "bf16", batch=1, context=32768)
    layer = W.make_layer("H", 1, cfg=cfg)
    dl = H.DeviceLayer(layer, kv_layout="head_major")
    dl.compress()
    gpu = dl.results()
    rep = H.compare_layer(layer, gpu, B.RANK_POSITION)
    print(rep)
    # mass conservation, a property of Eq. 2 that holds at any size: sum_i cnt_i A'[i] = w per head
    n, w = 32768, 328
    cnt = np.minimum(w, n - np.arange(n))
    mass = (gpu["scores"].astype(np.float64) * cnt).sum(axis=1)
    assert np.abs(mass - w).max() < 1e-3 * w


def test_wide_window_ten_percent():
    """k = 10 % of n at n = 16384 (1638 window positions, 6552 score rows per KV head, 52 blocks of 128
    rows): full parity and mass conservation per head."""
    n, w, Hq, Hkv, d = 16384, 1638, 32, 8, 128
    cfg = W.Config("t", 1, Hq, Hkv, d, w, "bf16", batch=1, context=n)
    layer = W.make_layer("H", 2, cfg=cfg)
    dl = H.DeviceLayer(layer, kv_layout="head_major")
    dl.compress()
    gpu = dl.results()
    rep = H.compare_layer(layer, gpu, B.RANK_POSITION)
    print(rep)
    cnt = np.minimum(w, n - np.arange(n))
    mass = (gpu["scores"].astype(np.float64) * cnt).sum(axis=1)
    assert np.abs(mass - w).max() < 1e-3 * w
