"""The seeded input generator: storage-format conversion and reproducibility."""
import numpy as np
import torch

from paper_2502_16886_amd import workloads as W


def test_bf16_rounding_matches_torch_rne():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 7.3
    x[:4] = [0.0, -0.0, 1.0, 65280.0]
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = W.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_layers_are_reproducible_and_distinct():
    a, b, c = W.make_layer(0, 0), W.make_layer(0, 0), W.make_layer(0, 1)
    assert np.array_equal(a.k, b.k) and np.array_equal(a.q_win, b.q_win) and np.array_equal(a.v, b.v)
    assert not np.array_equal(a.k, c.k)
    cfg = a.cfg
    assert a.k.shape == (512, 2, 64) and a.q_win.shape == (16, 8, 64) and a.k.dtype == np.float32
    assert list(a.cu_seqlens) == [0, 512]
    # sinks: the first four keys of a head are identical
    assert np.array_equal(a.k[0], a.k[3])


def test_ragged_config_lengths():
    cfg = W.CONFIGS[3]
    lens = W.seq_lengths(cfg, 3)
    assert len(lens) == 8 and lens.min() >= 2048 and lens.max() <= 32768
    assert np.array_equal(lens, W.seq_lengths(cfg, 3))
    small = W.make_layer(3, 0, lengths=[40, 7, 300, 1])
    assert small.k.dtype == np.uint16 and small.k.shape == (348, 8, 128)
    assert small.q_win.shape == (32 + 7 + 32 + 1, 32, 128)


def test_oracle_on_config0_matches_frozen_fixture():
    import json
    import os
    from oracle import refreekv_oracle as O
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "cfg0_oracle.json")))
    L = W.make_layer(0, 0)
    c = L.cfg
    s = O.oracle_score(L.f64("q_win"), L.f64("k"), L.cu_seqlens, c.n_q_heads, c.n_kv_heads, c.window)
    for p, vals in g["score_samples"].items():
        assert np.allclose(s[:, int(p)], vals, rtol=1e-12)
    for mode, name in ((O.RANK_POSITION, "position"), (O.RANK_SCORE, "score")):
        kept, _, _ = O.oracle_select(s, L.cu_seqlens, mode, c.n_sink, c.threshold)
        assert [int(x) for x in kept] == g[name]["kept"]
