"""GPU parity of the entry points that take the window rows' log-sum-exp from the caller
(rfkv_score_lse, rfkv_compress_layer_lse): one pass over K, against the float64 oracle given the
same float32 lse values."""
import numpy as np
import pytest

import rfkv_harness as H
from oracle import refreekv_oracle as O
from paper_2502_16886_amd import binding as B
from paper_2502_16886_amd import workloads as W

pytestmark = pytest.mark.gpu


def _lse32(layer, perturb=None):
    c = layer.cfg
    lse = O.oracle_window_lse(layer.f64("q_win"), layer.f64("k"), layer.cu_seqlens, c.n_q_heads, c.n_kv_heads, c.window)
    if perturb is not None:
        lse = lse + perturb(lse.shape)
    return lse.astype(np.float32)


def _run(layer, lse32, rank_mode, kv_layout="token_major"):
    import torch
    c = layer.cfg
    dl = H.DeviceLayer(layer, rank_mode=rank_mode, kv_layout=kv_layout)
    dl.compress(lse_win=torch.from_numpy(lse32).cuda())
    gpu = dl.results()
    ref_scores = O.oracle_score_lse(layer.f64("q_win"), lse32.astype(np.float64), layer.f64("k"), layer.cu_seqlens,
                                    c.n_q_heads, c.n_kv_heads, c.window)
    ref = H.oracle_layer(layer, rank_mode, scores=ref_scores)
    return dl, gpu, H.compare_layer(layer, gpu, rank_mode, ref=ref)


CASES = [
    # (Hq, Hkv, d, dtype, window, lens): one per scoring kernel family
    (32, 8, 128, "bf16", 32, [2500, 300]),            # streaming kernel, 4 row tiles
    (8, 2, 64, "bf16", 16, [700, 5, 64]),             # 2 row tiles, d = 64, a sequence shorter than the window
    (32, 8, 128, "bf16", 1, [1800, 1]),               # the paper's k = 1 (no kept logits needed here)
    (28, 4, 128, "bf16", 32, [1500]),                 # G = 7: 224 rows, wide-window column sums
    (8, 2, 128, "bf16", 300, [2000]),                 # 1200 rows
    (8, 2, 128, "fp32", 32, [600]),                   # fp32 d = 128, 128 rows: the register-operand kernels
    (8, 2, 64, "fp32", 16, [512]),                    # config 0's shape
    (8, 2, 128, "bf16", 32, [0, 400, 0]),             # empty sequences
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: f"Hq{c[0]}_Hkv{c[1]}_d{c[2]}_{c[3]}_w{c[4]}")
@pytest.mark.parametrize("rank_mode", [B.RANK_POSITION, B.RANK_SCORE], ids=["position", "score"])
def test_compress_layer_from_lse(case, rank_mode):
    Hq, Hkv, d, dtype, w, lens = case
    cfg = W.Config("t", 1, Hq, Hkv, d, w, dtype, batch=len(lens), context=max(lens), threshold=0.02)
    layer = W.make_layer(5, 0, cfg=cfg, lengths=lens)
    _, gpu, rep = _run(layer, _lse32(layer), rank_mode)
    print(rep)
    # with the exact normalisers the result is the two-pass result up to rounding
    two = H.DeviceLayer(layer, rank_mode=rank_mode)
    two.compress()
    s2 = two.results()["scores"]
    assert np.abs(gpu["scores"] - s2).max() <= 1e-4 * np.abs(s2).max()


def test_scores_follow_the_given_lse_not_their_own():
    cfg = W.Config("t", 1, 8, 2, 128, 32, "bf16", batch=1, context=900)
    layer = W.make_layer(5, 1, cfg=cfg, lengths=[900])
    rng = np.random.default_rng(3)
    lse32 = _lse32(layer, perturb=lambda shape: rng.uniform(-0.5, 0.5, shape))
    _, gpu, rep = _run(layer, lse32, B.RANK_POSITION)
    exact = O.oracle_score(layer.f64("q_win"), layer.f64("k"), layer.cu_seqlens, 8, 2, 32)
    assert np.abs(gpu["scores"] - exact).max() > 1e-2 * np.abs(exact).max()      # visibly not the softmax scores


def test_score_lse_entry_point_and_rejections():
    import torch
    cfg = W.Config("t", 1, 8, 2, 128, 32, "bf16", batch=2, context=400)
    layer = W.make_layer(5, 2, cfg=cfg, lengths=[400, 77])
    lse32 = _lse32(layer)
    dl = H.DeviceLayer(layer)
    lse_dev = torch.from_numpy(lse32).cuda()
    b = dl.buf
    B.rfkv_score_lse(dl.params, dl.q, lse_dev, dl.k, dl.cu_host, dl.cu_dev, b.scores, b.ws, b.ws_bytes)
    torch.cuda.synchronize()
    ref = O.oracle_score_lse(layer.f64("q_win"), lse32.astype(np.float64), layer.f64("k"), layer.cu_seqlens, 8, 2, 32)
    rel, nbad = H.score_errors(b.scores.cpu().numpy(), ref)
    assert nbad == 0
    st = B.rfkv_score_lse(dl.params, dl.q, None, dl.k, dl.cu_host, dl.cu_dev, b.scores, b.ws, b.ws_bytes, check=False)
    assert st == B.RFKV_INVALID_ARG
    st = B.rfkv_compress_layer_lse(dl.params, dl.q, None, dl.k, dl.v, dl.cu_host, dl.cu_dev, b.scores, b.kept,
                                   b.out_offsets, b.idx, b.k_out, b.v_out, b.capacity_rows, b.ws, b.ws_bytes, check=False)
    assert st == B.RFKV_INVALID_ARG


def test_full_size_headline_from_lse():
    """The headline shape in the benchmark's launch configuration (head-major K/V), every unit."""
    layer = W.make_layer("H", 3)
    _, gpu, rep = _run(layer, _lse32(layer), B.RANK_POSITION, kv_layout="head_major")
    print(rep)
    assert rep["exact"] == rep["units"]
