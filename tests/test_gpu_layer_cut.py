"""GPU parity of the per-layer cut (one stopping position per layer and sequence, norm over all KV
heads; both rankings) and of the padded output layout, against the float64 oracle."""
import numpy as np
import pytest

import rfkv_harness as H
from oracle import refreekv_oracle as O
from paper_2502_16886_amd import binding as B
from paper_2502_16886_amd import workloads as W

pytestmark = pytest.mark.gpu


def _gather(layer, kept, offs, idx):
    return O.oracle_compact(layer.k, layer.v, layer.cu_seqlens, kept, offs, idx)


def _check_layer_cut(layer, threshold=None, min_keep=0, kv_layout="token_major", mode=B.RANK_POSITION):
    c = layer.cfg
    T = H.threshold_as_float32(c.threshold if threshold is None else threshold)
    dl = H.DeviceLayer(layer, rank_mode=mode, threshold=threshold, min_keep=min_keep, kv_layout=kv_layout,
                       granularity=B.PER_LAYER)
    dl.compress()
    gpu = dl.results()
    # scores do not depend on the granularity
    ref_scores = O.oracle_score(layer.f64("q_win"), layer.f64("k"), layer.cu_seqlens, c.n_q_heads, c.n_kv_heads, c.window)
    rel, nbad = H.score_errors(gpu["scores"], ref_scores)
    assert nbad == 0
    # stage-exact: the oracle's per-layer rule on the GPU's own scores gives the GPU's selection, bit for bit
    kept, offs, idx = O.oracle_select_layer(gpu["scores"].astype(np.float64), layer.cu_seqlens, mode,
                                            c.n_sink, T, min_keep, form="cumsum")
    assert np.array_equal(gpu["kept"], kept), f"{gpu['kept']} vs {kept}"
    assert np.array_equal(gpu["out_offsets"], offs)
    assert np.array_equal(gpu["idx"], idx)
    k_out, v_out = _gather(layer, kept, offs, idx)
    assert np.array_equal(gpu["k_out"], k_out) and np.array_equal(gpu["v_out"], v_out)
    # every head of a sequence keeps the same number of positions
    Hkv = c.n_kv_heads
    assert np.all(gpu["kept"].reshape(-1, Hkv) == gpu["kept"].reshape(-1, Hkv)[:, :1])
    # end to end: from the oracle's own scores the cut may move only when it sits on a rounding edge
    kept_ref, _, _ = O.oracle_select_layer(ref_scores, layer.cu_seqlens, mode, c.n_sink, T, min_keep,
                                           form="cumsum")
    # (the score ranking's cut is ill-conditioned: a step of the rule is ~1e-9 of the mass at these lengths)
    assert np.abs(gpu["kept"] - kept_ref).max() <= (2 if mode == B.RANK_POSITION else max(2, int(2e-3 * kept_ref.max())))
    return gpu, int(np.sum(gpu["kept"] == kept_ref)), len(kept)


@pytest.mark.parametrize("Hq,Hkv,d,w,lens,T", [
    (8, 2, 128, 32, [777], 0.01),
    (32, 8, 128, 32, [1500, 333, 0, 40], 0.02),
    (28, 4, 128, 32, [2100], 0.01),
    (8, 8, 64, 16, [300, 1, 45, 1029], 0.05),
    (4, 1, 128, 5, [3, 2, 4, 70], 0.01),           # n <= m
    (8, 2, 128, 16, [600, 90], 0.0),               # T = 0 keeps everything
    (8, 2, 128, 16, [600, 90], 1.0),               # T = 1 keeps one position
])
@pytest.mark.parametrize("mode", [B.RANK_POSITION, B.RANK_SCORE], ids=["position", "score"])
def test_layer_cut_small_shapes(Hq, Hkv, d, w, lens, T, mode):
    cfg = W.Config("t", 1, Hq, Hkv, d, w, "bf16", batch=len(lens), context=max(lens), threshold=T)
    layer = W.make_layer(0, 5, cfg=cfg, lengths=lens)
    gpu, same, units = _check_layer_cut(layer, mode=mode)
    if T == 0.0:
        assert np.array_equal(gpu["kept"], np.repeat(lens, Hkv))
    if T == 1.0:
        assert np.all(gpu["kept"] == 1)


def test_layer_cut_score_ranking_ties_and_long_rows():
    """The score ranking's per-layer cut where its sort has to work: a row longer than one LDS chunk (16385 and
    40000 positions: strides in global memory, a padded power of two), and equal scores (fed straight to
    rfkv_select: every head keeps its lowest positions)."""
    import torch
    cfg = W.Config("t", 1, 8, 2, 128, 16, "bf16", batch=2, context=40000, threshold=0.02)
    layer = W.make_layer(0, 8, cfg=cfg, lengths=[16385, 40000])
    _check_layer_cut(layer, mode=B.RANK_SCORE)
    n, Hkv = 9001, 3
    p = B.make_params(1, 3, Hkv, 128, 1, "bf16", threshold=0.1, rank_mode=B.RANK_SCORE, granularity=B.PER_LAYER)
    cu = np.array([0, n], dtype=np.int32)
    cu_d = torch.from_numpy(cu).cuda()
    host = np.full((Hkv, n), 0.25, np.float32)
    host[1, 8900:9000] = 0.5                                 # one head has a hundred larger scores, near its end
    scores = torch.from_numpy(host).cuda()
    buf = B.alloc_layer_buffers(p, n, n)
    B.rfkv_select(p, scores, cu, cu_d, buf.kept, buf.out_offsets, buf.idx, buf.ws, buf.ws_bytes)
    torch.cuda.synchronize()
    kept, offs, idx = O.oracle_select_layer(host.astype(np.float64), cu, O.RANK_SCORE, 4, H.threshold_as_float32(0.1), 0,
                                            form="cumsum")
    assert np.array_equal(buf.kept.cpu().numpy(), kept) and kept[0] == kept[1] == kept[2]
    assert np.array_equal(buf.idx[:int(offs[-1])].cpu().numpy(), idx)
    c = int(kept[0])
    assert 100 < c < 8900
    assert np.array_equal(idx[:c], np.arange(c))             # ties: the lowest positions
    assert np.array_equal(idx[c:2 * c], np.concatenate([np.arange(c - 100), np.arange(8900, 9000)]))


@pytest.mark.parametrize("mode", [B.RANK_POSITION, B.RANK_SCORE], ids=["position", "score"])
def test_layer_cut_fp32_config0_and_min_keep(mode):
    layer = W.make_layer(0, 0)
    _check_layer_cut(layer, mode=mode)
    gpu, _, _ = _check_layer_cut(layer, threshold=0.5, min_keep=300, mode=mode)
    assert np.all(gpu["kept"] == 300)


def test_layer_cut_full_size_headline_score_ranking():
    layer = W.make_layer("H", 2)
    gpu, same, units = _check_layer_cut(layer, kv_layout="head_major", mode=B.RANK_SCORE)
    print(f"headline layer 2, score ranking: shared cut keeps {gpu['kept'][0]} per head; "
          f"{same}/{units} units equal to the float64 oracle's own cut")


def test_layer_cut_full_size_headline():
    layer = W.make_layer("H", 2)
    gpu, same, units = _check_layer_cut(layer, kv_layout="head_major")
    per_head = H.DeviceLayer(layer, kv_layout="head_major")
    per_head.compress()
    ph = per_head.results()
    print(f"headline layer 2: shared cut keeps {gpu['kept'][0]} per head; per-head cuts keep {ph['kept'].tolist()}; "
          f"{same}/{units} units equal to the float64 oracle's own cut")
    assert same == units


def test_padded_layout_matches_ragged():
    cfg = W.Config("t", 1, 8, 2, 128, 32, "bf16", batch=3, context=900)
    lens = [900, 130, 411]
    layer = W.make_layer(0, 6, cfg=cfg, lengths=lens)
    for gran in (B.PER_HEAD, B.PER_LAYER):
        ragged = H.DeviceLayer(layer, granularity=gran)
        ragged.compress()
        r = ragged.results()
        pad = 1024
        padded = H.DeviceLayer(layer, granularity=gran, out_pad_rows=pad)
        padded.buf.k_out.view(dtype=__import__("torch").int16).fill_(-1)
        padded.compress()
        p = padded.results()
        units = len(r["kept"])
        assert np.array_equal(p["kept"], r["kept"])
        # against the oracle: its rule on the GPU's scores, its gather, laid out slot by slot; the mask is t < kept[u]
        sel = O.oracle_select_layer if gran == B.PER_LAYER else O.oracle_select
        okept, ooffs, oidx = sel(p["scores"].astype(np.float64), layer.cu_seqlens, O.RANK_POSITION, cfg.n_sink,
                                 H.threshold_as_float32(cfg.threshold), 0, form="cumsum")
        ok, ov = O.oracle_compact(layer.k, layer.v, layer.cu_seqlens, okept, ooffs, oidx)
        assert np.array_equal(p["kept"], okept)
        for u in range(units):
            c, o = int(okept[u]), int(ooffs[u])
            assert np.array_equal(p["k_out"][u * pad:u * pad + c], ok[o:o + c])
            assert np.array_equal(p["v_out"][u * pad:u * pad + c], ov[o:o + c])
            assert np.array_equal(p["idx"][u * pad:u * pad + c], oidx[o:o + c])
        assert np.array_equal(p["out_offsets"], np.arange(units + 1) * pad)
        for u in range(units):
            c, o = int(r["kept"][u]), int(r["out_offsets"][u])
            assert np.array_equal(p["k_out"][u * pad:u * pad + c], r["k_out"][o:o + c])
            assert np.array_equal(p["v_out"][u * pad:u * pad + c], r["v_out"][o:o + c])
            assert np.array_equal(p["idx"][u * pad:u * pad + c], r["idx"][o:o + c])
            assert np.all(p["k_out"][u * pad + c:(u + 1) * pad] == 0xFFFF)      # pad rows are left untouched


def test_layer_cut_and_padding_rejections():
    import torch
    t = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")
    cu = np.array([0, 100], np.int32)
    p = B.make_params(1, 8, 2, 128, 16, "bf16", out_pad_rows=64)              # shorter than the sequence
    st = B.rfkv_compress_layer(p, t, t, t, cu, t, None, t, t, None, t, t, 200, t, 1 << 16, check=False)
    assert st == B.RFKV_OUTPUT_TOO_SMALL
    p = B.make_params(1, 8, 2, 128, 16, "bf16", out_pad_rows=128)             # 2 units x 128 rows > capacity 200
    st = B.rfkv_compress_layer(p, t, t, t, cu, t, None, t, t, None, t, t, 200, t, 1 << 16, check=False)
    assert st == B.RFKV_OUTPUT_TOO_SMALL
    p = B.make_params(1, 8, 2, 128, 16, "bf16", granularity=5)
    st = B.rfkv_compress_layer(p, t, t, t, cu, t, None, t, t, None, t, t, 200, t, 1 << 16, check=False)
    assert st == B.RFKV_INVALID_ARG
