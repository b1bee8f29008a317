"""GPU parity: librfkv (through its C ABI) against the float64 oracle, element by element, on
the same seeded inputs.  Sizes: small shapes that still span several MFMA tiles, workgroup spans
and a ragged tail; the five workload configurations plus the headline shape at full size (one or
a few layers each, in the launch geometry the benchmark uses); and the degenerate cases."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import rfkv_harness as H                                   # noqa: E402
from oracle import refreekv_oracle as O                    # noqa: E402
from paper_2502_16886_amd import binding as B              # noqa: E402
from paper_2502_16886_amd import workloads as W            # noqa: E402

pytestmark = pytest.mark.gpu
MODES = [B.RANK_POSITION, B.RANK_SCORE]
FULL = os.environ.get("RFKV_FULL_LAYERS", "0") == "1"


def run_and_compare(layer, mode, **kw):
    dl = H.DeviceLayer(layer, rank_mode=mode, **kw)
    dl.compress()
    gpu = dl.results()
    rep = H.compare_layer(layer, gpu, mode, **kw)
    print(f"\n  cfg={layer.meta.get('cfg_id')} layer={layer.meta.get('layer')} mode={mode} {rep}", flush=True)
    return dl, gpu, rep


def small_cfg(dtype, Hq, Hkv, d, w, **kw):
    return W.Config("small", 1, Hq, Hkv, d, w, dtype, **kw)


# ------------------------------------------------------------------ config 0 and small shapes
@pytest.mark.parametrize("mode", MODES)
def test_config0_tiny_fp32(mode):
    _, gpu, rep = run_and_compare(W.make_layer(0, 0), mode)
    assert rep["max_rel_score_err"] < 1e-4


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("dtype,Hq,Hkv,d,w,lens", [
    ("bf16", 8, 2, 128, 32, [777]),                 # several tiles + ragged tail
    ("bf16", 28, 4, 128, 32, [1500, 333]),          # G = 7: 224 rows -> two 128-row blocks of the wide-window kernels
    ("bf16", 8, 8, 64, 16, [300, 1, 45, 1029]),     # G = 1, d = 64, a length-1 sequence
    ("fp32", 8, 2, 128, 8, [513, 64]),              # fp32 d = 128
    ("fp32", 4, 4, 64, 1, [260]),                   # the paper's k = 1
    ("bf16", 32, 8, 128, 64, [40, 2100]),           # n < window for the first sequence; 256 rows
    ("bf16", 4, 1, 128, 5, [3, 2, 4, 70]),          # n <= m (sinks) and odd window
    ("bf16", 8, 2, 128, 24, [900, 20]),             # 96 rows: padded to the 4-row-tile kernels
    ("bf16", 8, 2, 128, 40, [1100]),                # 160 rows: wide-window kernels, second block mostly padding
    ("bf16", 8, 2, 64, 72, [700, 300]),             # 288 rows, d = 64: three blocks
    ("fp32", 8, 2, 128, 32, [600, 50]),             # fp32 d = 128, 128 rows: the register-operand kernels of score.hip
    ("fp32", 8, 2, 128, 64, [450]),                 # fp32 d = 128, 256 rows (the most its 512-byte rows allow in LDS is 288)
    ("fp32", 8, 2, 64, 32, [640, 33]),              # fp32 d = 64, 128 rows
    ("bf16", 16, 4, 64, 32, [2050]),                # bf16 d = 64, 128 rows
    ("bf16", 32, 8, 128, 1, [1500, 333, 1, 40]),    # the paper's k = 1 with GQA 4: logits kept, one K pass
    ("bf16", 8, 2, 128, 2, [777, 2, 1]),            # 8 rows, two window positions: causal masking in the kept logits
    ("bf16", 28, 4, 128, 1, [900]),                 # k = 1, G = 7
    ("fp32", 8, 1, 128, 1, [513, 64]),              # k = 1, G = 8, fp32 d = 128
])
def test_small_shapes(mode, dtype, Hq, Hkv, d, w, lens):
    cfg = small_cfg(dtype, Hq, Hkv, d, w, batch=len(lens))
    layer = W.make_layer(0, 17, cfg=cfg, lengths=lens)
    run_and_compare(layer, mode)


@pytest.mark.parametrize("mode", MODES)
def test_thresholds_and_min_keep(mode):
    cfg = small_cfg("bf16", 8, 2, 128, 16, batch=2)
    layer = W.make_layer(0, 3, cfg=cfg, lengths=[600, 90])
    n_units = np.repeat([600, 90], 2)
    for T in (0.0, 1e-4, 0.05, 0.5, 1.0, 2.0):
        _, gpu, _ = run_and_compare(layer, mode, threshold=T)
        if T == 0.0:      # full budget reproduces the cache bit for bit
            assert np.array_equal(gpu["kept"], n_units)
            o = 0
            for u, b, h, s, e in H.unit_slices(layer):
                assert np.array_equal(gpu["k_out"][o:o + e - s], layer.k[s:e, h])
                assert np.array_equal(gpu["v_out"][o:o + e - s], layer.v[s:e, h])
                o += e - s
        if T >= 1.0:
            assert np.all(gpu["kept"] == 1)
    _, gpu, _ = run_and_compare(layer, mode, threshold=0.5, min_keep=100)
    assert np.array_equal(gpu["kept"], np.minimum(np.maximum(gpu["kept"], 100), n_units))
    assert np.all(gpu["kept"][:2] >= 100) and np.all(gpu["kept"][2:] == 90)


@pytest.mark.parametrize("m", [0, 1, 33, 70, 200, 5000])
def test_sink_counts(m):
    """n_sink (the paper's m, positions ranked first) other than 4: none, one, more than a tile, more
    than a wavefront, more than the sequence; thresholds that put the cut among the sinks and past them."""
    cfg = small_cfg("bf16", 8, 2, 128, 16, batch=2)
    layer = W.make_layer(0, 9, cfg=cfg, lengths=[1200, 150])
    for T in (0.01, 0.3, 0.9):
        for mode in MODES:
            dl = H.DeviceLayer(layer, rank_mode=mode, threshold=T, n_sink=m)
            dl.compress()
            H.compare_layer(layer, dl.results(), mode, threshold=T, n_sink=m)
    # the per-layer cut takes the same sink paths
    T32 = H.threshold_as_float32(0.3)
    dl = H.DeviceLayer(layer, threshold=0.3, n_sink=m, granularity=B.PER_LAYER)
    dl.compress()
    gpu = dl.results()
    kept, offs, idx = O.oracle_select_layer(gpu["scores"].astype(np.float64), layer.cu_seqlens, O.RANK_POSITION, m, T32, 0,
                                            form="cumsum")
    assert np.array_equal(gpu["kept"], kept) and np.array_equal(gpu["idx"], idx)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("kv_layout", ["token_major", "head_major"])
def test_model_loop_keeps_the_bottom_layers_whole(mode, kv_layout):
    """Sec. 3.3 "Retaining Bottom Layers": compress_model leaves the first two layers unpruned (the
    library is handed no queries for them and scores nothing: it only re-lays the cache out per
    unit) and compresses the rest."""
    cfg = small_cfg("bf16", 8, 2, 128, 32, batch=3)
    host = [W.make_layer(1, li, cfg=cfg, lengths=[700, 33, 1500]) for li in range(4)]
    dls = [H.DeviceLayer(l, rank_mode=mode, kv_layout=kv_layout) for l in host]
    for dl in dls:                                        # stale contents must not survive
        dl.buf.kept.fill_(-7)
        dl.buf.k_out.fill_(1.0)
    H.compress_model(dls, n_frozen=2)
    ref = O.oracle_compress_model([(l.f64("q_win"), l.f64("k"), l.k, l.v, l.cu_seqlens) for l in host], cfg.n_q_heads,
                                  cfg.n_kv_heads, cfg.window, n_frozen=2, n_sink=cfg.n_sink,
                                  T=H.threshold_as_float32(cfg.threshold), rank_mode=mode, form="cumsum")
    for li, (dl, layer) in enumerate(zip(dls, host)):
        gpu = dl.results()
        if li < 2:
            for key in ("kept", "out_offsets", "idx", "k_out", "v_out"):
                assert np.array_equal(gpu[key], ref[li][key]), (li, key)
        else:
            H.compare_layer(layer, gpu, mode)
            assert gpu["kept"].sum() < ref[0]["kept"].sum()


def test_large_logits_do_not_overflow():
    # logits of magnitude ~80: the running reference exponent must keep exp2 in range
    cfg = small_cfg("fp32", 4, 2, 64, 4, q_shared=0.0, x_sink=(0.0, 0.0), spike_frac=0.0)
    layer = W.make_layer(0, 5, cfg=cfg, lengths=[400])
    layer.q_win *= np.float32(9.0)
    layer.k *= np.float32(9.0)
    dl = H.DeviceLayer(layer)
    dl.compress()
    gpu = dl.results()
    assert np.all(np.isfinite(gpu["scores"]))
    ref = O.oracle_score(layer.f64("q_win"), layer.f64("k"), layer.cu_seqlens, 4, 2, 4)
    assert np.abs(layer.f64("q_win")[0, 0] @ layer.f64("k")[:, 0].T / 8).max() > 60
    rel, nbad = H.score_errors(gpu["scores"], ref)
    assert nbad == 0


@pytest.mark.parametrize("window", [32, 200])
def test_logit_far_above_the_running_reference(window):
    """A key in the middle of a span whose logits lie ~100 binary orders above everything before it:
    the statistics pass sums a tile against the reference exponent it already has and must notice
    that this tile does not fit (both the streaming kernels and the wide-window row blocks)."""
    cfg = small_cfg("bf16", 8, 2, 128, window, x_sink=(0.0, 0.0), spike_frac=0.0)
    layer = W.make_layer(1, 3, cfg=cfg, lengths=[2600])
    q = layer.f64("q_win").reshape(-1, 2, 4, 128)
    k = layer.f64("k")
    for h in range(2):
        qbar = q[:, h].mean(axis=(0, 1))
        for pos in (700, 1911):
            k[pos, h] = qbar * (90.0 * np.sqrt(128.0) / (qbar @ qbar))
    import torch
    layer.k = torch.from_numpy(k).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    logits = np.einsum("rd,nd->rn", q[:, 0, 0], layer.f64("k")[:, 0]) / np.sqrt(128.0)
    assert logits[:, 700].min() - np.delete(logits, (700, 1911), axis=1).max() > 60 * np.log(2.0)
    for mode in MODES:
        run_and_compare(layer, mode)


def test_all_equal_scores_tie_break_lowest_index():
    # feed rfkv_select directly: equal scores -> score ranking keeps positions 0..kept-1
    import torch
    n, Hkv = 5001, 2
    p = B.make_params(1, 2, Hkv, 128, 1, "bf16", threshold=0.1, rank_mode=B.RANK_SCORE)
    cu = np.array([0, n], dtype=np.int32)
    cu_d = torch.from_numpy(cu).cuda()
    scores = torch.full((Hkv, n), 0.25, dtype=torch.float32, device="cuda")
    buf = B.alloc_layer_buffers(p, n, n)
    B.rfkv_select(p, scores, cu, cu_d, buf.kept, buf.out_offsets, buf.idx, buf.ws, buf.ws_bytes)
    torch.cuda.synchronize()
    kept = buf.kept.cpu().numpy()
    expect = O.select_unit(np.full(n, 0.25), O.RANK_SCORE, 4, H.threshold_as_float32(0.1))[0]
    assert np.all(kept == expect) and expect == int(np.floor(0.81 * n)) + 1     # 0.81 n is not an integer
    offs = buf.out_offsets.cpu().numpy()
    assert list(offs) == [0, expect, 2 * expect]
    idx = buf.idx[:2 * expect].cpu().numpy()
    assert np.array_equal(idx[:expect], np.arange(expect)) and np.array_equal(idx[expect:], np.arange(expect))
    # all-zero scores: F = 0 keeps everything
    scores.zero_()
    B.rfkv_select(p, scores, cu, cu_d, buf.kept, buf.out_offsets, buf.idx, buf.ws, buf.ws_bytes)
    torch.cuda.synchronize()
    assert np.all(buf.kept.cpu().numpy() == n)


@pytest.mark.parametrize("T", [0.02, 0.31])
def test_score_ranking_of_long_units_in_a_ragged_batch(T):
    """Units split over several workgroups (longer than 8192 positions) beside short and empty ones of the same
    batch, fed straight to rfkv_select, with score patterns that send the last workgroup of a unit down
    each of its ways: a crossing bucket of a few scores (ranked pair by pair), of thousands (two more radix
    digits) and of more equal scores than its LDS holds (re-read from memory)."""
    import torch
    lens = [20000, 100, 0, 2500, 9001, 12000]
    Hkv = 2
    N = sum(lens)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rng = np.random.default_rng(5)
    host = np.zeros((Hkv, N), np.float32)
    for b, n in enumerate(lens):
        s0 = int(cu[b])
        if n == 0:
            continue
        # head 0: a few large scores over a floor of small ones; head 1: per sequence a different shape
        host[0, s0:s0 + n] = rng.uniform(1e-6, 2e-6, n)
        host[0, s0 + rng.choice(n, max(1, n // 50), replace=False)] = rng.uniform(0.01, 0.5, max(1, n // 50))
        if b % 3 == 0:
            host[1, s0:s0 + n] = rng.uniform(0.25, 0.3, n)              # thousands of scores in one bucket
        elif b % 3 == 1:
            host[1, s0:s0 + n] = 0.125                                  # all equal: ties, lowest positions win
        else:
            host[1, s0:s0 + n] = np.exp(rng.normal(-8.0, 2.0, n))       # spread over many exponents
    p = B.make_params(len(lens), 2, Hkv, 128, 1, "bf16", threshold=T, rank_mode=B.RANK_SCORE)
    cu_d = torch.from_numpy(cu).cuda()
    scores = torch.from_numpy(host).cuda()
    buf = B.alloc_layer_buffers(p, N, max(lens))
    for _ in range(2):                                                  # the second call finds the counters reset
        buf.kept.fill_(-7)
        B.rfkv_select(p, scores, cu, cu_d, buf.kept, buf.out_offsets, buf.idx, buf.ws, buf.ws_bytes)
        torch.cuda.synchronize()
        kept, offs, idx = O.oracle_select(host.astype(np.float64), cu, O.RANK_SCORE, 4, H.threshold_as_float32(T), 0,
                                          form="cumsum")
        assert np.array_equal(buf.kept.cpu().numpy(), kept)
        assert np.array_equal(buf.out_offsets.cpu().numpy(), offs)
        assert np.array_equal(buf.idx[:int(offs[-1])].cpu().numpy(), idx)


@pytest.mark.parametrize("mode", MODES)
def test_staged_calls_equal_fused_call(mode):
    # rfkv_score -> rfkv_select -> rfkv_compact give what rfkv_compress_layer gives; strided
    # (head-major) K/V layouts give the same result as token-major ones
    import torch
    cfg = small_cfg("bf16", 8, 2, 128, 32, batch=2)
    layer = W.make_layer(0, 9, cfg=cfg, lengths=[1200, 257])
    dl = H.DeviceLayer(layer, rank_mode=mode)
    dl.compress()
    fused = dl.results()
    b2 = B.alloc_layer_buffers(dl.params, dl.N, dl.max_len)
    B.rfkv_score(dl.params, dl.q, dl.k, dl.cu_host, dl.cu_dev, b2.scores, b2.ws, b2.ws_bytes)
    B.rfkv_select(dl.params, b2.scores, dl.cu_host, dl.cu_dev, b2.kept, b2.out_offsets, b2.idx, b2.ws, b2.ws_bytes)
    B.rfkv_compact(dl.params, dl.k, dl.v, dl.cu_host, dl.cu_dev, b2.kept, b2.out_offsets, b2.idx, b2.k_out,
                   b2.v_out, b2.capacity_rows)
    torch.cuda.synchronize()
    total = int(b2.out_offsets[-1])
    assert np.array_equal(b2.scores.cpu().numpy(), fused["scores"])
    assert np.array_equal(b2.kept.cpu().numpy(), fused["kept"])
    assert np.array_equal(b2.idx[:total].cpu().numpy(), fused["idx"])
    assert np.array_equal(H.to_host_bits(b2.k_out[:total], "bf16"), fused["k_out"])
    assert np.array_equal(H.to_host_bits(b2.v_out[:total], "bf16"), fused["v_out"])
    # head-major storage [Hkv, N, d] described through the strides
    dl3 = H.DeviceLayer(layer, rank_mode=mode)
    dl3.k = dl3.k.permute(1, 0, 2).contiguous()
    dl3.v = dl3.v.permute(1, 0, 2).contiguous()
    dl3.params.k_stride_tok = dl3.params.v_stride_tok = 128
    dl3.params.k_stride_head = dl3.params.v_stride_head = dl3.N * 128
    dl3.compress()
    again = dl3.results()
    for key in ("scores", "kept", "idx", "k_out", "v_out"):
        assert np.array_equal(again[key], fused[key]), key


def test_repeat_runs_are_bit_identical_and_capacity_is_respected():
    import torch
    cfg = small_cfg("bf16", 32, 8, 128, 32)
    layer = W.make_layer(1, 2, cfg=cfg, lengths=[3000])
    for mode in MODES:
        dl = H.DeviceLayer(layer, rank_mode=mode)
        dl.compress()
        a = dl.results()
        dl.compress()
        b = dl.results()
        for key in a:
            assert np.array_equal(a[key], b[key]), key
        # a too-small output is never overrun: rows past the capacity are simply not written
        total = int(a["out_offsets"][-1])
        cap = total // 2
        dl.buf.k_out.fill_(7.0)
        dl.buf.v_out.fill_(7.0)
        B.rfkv_compress_layer(dl.params, dl.q, dl.k, dl.v, dl.cu_host, dl.cu_dev, None, dl.buf.kept,
                              dl.buf.out_offsets, None, dl.buf.k_out, dl.buf.v_out, cap, dl.buf.ws, dl.buf.ws_bytes)
        torch.cuda.synchronize()
        assert int(dl.buf.out_offsets[-1]) == total                    # the caller can see the overflow
        assert np.array_equal(H.to_host_bits(dl.buf.k_out[:cap], "bf16"), a["k_out"][:cap])
        assert torch.all(dl.buf.k_out[cap:total].float() == 7.0) and torch.all(dl.buf.v_out[cap:total].float() == 7.0)


# ------------------------------------------------------------------ the workload configurations at full size
# (config, layers, K/V storage): the headline shape runs in the storage the benchmark times
FULL_CASES = [(1, [0, 13, 31], "token_major"), (2, [5], "head_major"), (3, [2], "token_major"),
              ("H", [0], "head_major"), (4, [1], "head_major"), ("K1", [0, 7], "head_major")]
# Units of a layer whose retained set may differ from the oracle's (they are never cut-robust ones, and
# compare_layer bounds how far they may move): none on configs 1, 2, 3 and the headline, one on the
# 131072-token config and on k = 1, where single razor-edge units exist among the 32 layers.
MAY_DIFFER = {1: 0, 2: 0, 3: 0, "H": 0, 4: 1, "K1": 1}


@pytest.mark.parametrize("cfg_id,layers,kv_layout", FULL_CASES)
def test_full_size_configs(cfg_id, layers, kv_layout):
    cfg = W.CONFIGS[cfg_id]
    if FULL:
        layers = list(range(cfg.layers))
    for li in layers:
        layer = W.make_layer(cfg_id, li)
        ref_scores = O.oracle_score(layer.f64("q_win"), layer.f64("k"), layer.cu_seqlens, cfg.n_q_heads,
                                    cfg.n_kv_heads, cfg.window)
        for mode in MODES:
            ref = H.oracle_layer(layer, mode, scores=ref_scores)
            dl = H.DeviceLayer(layer, rank_mode=mode, kv_layout=kv_layout)
            dl.compress()
            gpu = dl.results()
            rep = H.compare_layer(layer, gpu, mode, ref=ref)
            print(f"\n  cfg={cfg_id} layer={li} mode={mode} {rep}", flush=True)
            # most units of the score ranking are not cut-robust at these lengths (one step of the rule is
            # ~1e-9 of the mass), so the bit-exact comparison must not hinge on that class alone
            assert rep["exact"] >= rep["units"] - MAY_DIFFER[cfg_id], rep
            del dl, gpu
