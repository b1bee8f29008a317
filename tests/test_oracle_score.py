"""Pins for the oracle's scoring half (Sec. 3.2 "Reducing Overhead", Eq. 2).

Each test checks the oracle against something it does not compute itself: a
library softmax, the full n x n attention matrix built row by row with
scipy/torch, conservation laws of softmax, or a hand-derived closed form.
"""
import numpy as np
import pytest
import scipy.special
import torch

from oracle import refreekv_oracle as O


def rng(seed):
    return np.random.default_rng(seed)


def test_softmax_rows_sum_to_one_and_are_causal():
    r = rng(1)
    n, w, d = 97, 16, 32
    q, k = r.standard_normal((w, d)), r.standard_normal((n, d))
    P = O.window_attention(q, k, 1 / np.sqrt(d))
    assert np.allclose(P.sum(axis=1), 1.0, atol=1e-12)
    for t in range(w):
        last = n - w + t
        assert np.all(P[t, last + 1:] == 0.0)
        assert np.all(P[t, :last + 1] > 0.0)


def test_window_one_is_the_last_softmax_row_library():
    # k = 1 (the paper's default): A' is just the last row of softmax(QK^T/sqrt d)
    r = rng(2)
    n, d = 301, 64
    q, k = r.standard_normal((1, 1, d)), r.standard_normal((n, d))
    scale = 1 / np.sqrt(d)
    mine = O.score_unit(q, k, scale)
    ref = scipy.special.softmax((k @ q[0, 0]) * scale)
    assert np.allclose(mine, ref, rtol=1e-12, atol=0)
    ref_t = torch.softmax(torch.from_numpy(k @ q[0, 0]) * scale, dim=0).numpy()
    assert np.allclose(mine, ref_t, rtol=1e-12, atol=0)
    assert abs(mine.sum() - 1.0) < 1e-12


def test_matches_full_attention_matrix_with_literal_nonzero_count():
    # Build the whole causal n x n matrix A with torch, take its last k rows and
    # apply Eq. 2 with the literal "entry != 0" indicator as the denominator.
    r = rng(3)
    n, w, d = 40, 7, 16
    q_all, k = r.standard_normal((n, d)), r.standard_normal((n, d))
    scale = 1 / np.sqrt(d)
    logits = torch.from_numpy(q_all @ k.T) * scale
    mask = torch.tril(torch.ones(n, n, dtype=torch.bool))
    A = torch.softmax(logits.masked_fill(~mask, float("-inf")), dim=1).numpy()
    last = A[n - w:, :]
    expect = last.sum(axis=0) / (last != 0).sum(axis=0)
    mine = O.score_unit(q_all[n - w:, None, :], k, scale)
    assert np.allclose(mine, expect, rtol=1e-12, atol=0)


def test_causal_counts_closed_form():
    # 1-based position i is seen by min(w, n - i + 1) of the last w rows
    n, w = 23, 5
    c = O.causal_counts(n, w)
    for i1 in range(1, n + 1):
        assert c[i1 - 1] == min(w, n - i1 + 1)
    # brute force from the mask itself
    vis = np.array([[i <= n - w + t for i in range(n)] for t in range(w)])
    assert np.array_equal(c, vis.sum(axis=0))


def test_weighted_mass_conservation():
    # sum_i cnt_i * A'_g[i] = w'  (each of the w' rows carries unit mass)
    r = rng(4)
    n, w, d = 129, 16, 32
    q, k = r.standard_normal((w, d)), r.standard_normal((n, d))
    a = O.reduced_attention_vector(O.window_attention(q, k, 0.3))
    assert abs((O.causal_counts(n, w) * a).sum() - w) < 1e-10


def test_equal_keys_give_uniform_rows():
    # all keys identical -> every visible entry of row t is 1/(visible count);
    # A'[i] then has the closed form below
    n, w, d = 50, 4, 8
    k = np.tile(rng(5).standard_normal(d), (n, 1))
    q = rng(6).standard_normal((w, 1, d))
    a = O.score_unit(q, k, 0.5)
    expect = np.zeros(n)
    for i in range(n):
        rows = [t for t in range(w) if i <= n - w + t]
        expect[i] = sum(1.0 / (n - w + t + 1) for t in rows) / len(rows)
    assert np.allclose(a, expect, rtol=1e-12)


def test_gqa_is_mean_over_group_heads():
    r = rng(7)
    n, w, d, G = 64, 8, 16, 4
    q, k = r.standard_normal((w, G, d)), r.standard_normal((n, d))
    per_head = [O.score_unit(q[:, g:g + 1, :], k, 0.25) for g in range(G)]
    assert np.allclose(O.score_unit(q, k, 0.25), np.mean(per_head, axis=0), rtol=1e-13)


def test_shift_invariance_and_large_logits_are_safe():
    # adding a constant vector to every key along q changes nothing for w = 1;
    # logits near +-80 must not overflow
    r = rng(8)
    n, d = 77, 16
    q = r.standard_normal((1, 1, d))
    k = r.standard_normal((n, d))
    a = O.score_unit(q, k, 1.0)
    big = O.score_unit(q * 40, k, 1.0)
    assert np.all(np.isfinite(big)) and abs(big.sum() - 1) < 1e-12
    shift = O.score_unit(q, k + 3.0 * q[0, 0] / (q[0, 0] @ q[0, 0]), 1.0)
    assert np.allclose(a, shift, rtol=1e-10)


def test_ragged_batch_layout_and_short_sequences():
    # sequences shorter than the window use min(w, n) rows; units are independent
    r = rng(9)
    Hq, Hkv, d, w = 4, 2, 8, 6
    lens = [3, 1, 11]
    cu = np.concatenate([[0], np.cumsum(lens)])
    k = r.standard_normal((cu[-1], Hkv, d))
    qs = [r.standard_normal((min(w, n), Hq, d)) for n in lens]
    q = np.concatenate(qs)
    s = O.oracle_score(q, k, cu, Hq, Hkv, w)
    assert s.shape == (Hkv, cu[-1])
    for b, n in enumerate(lens):
        for h in range(Hkv):
            alone = O.score_unit(qs[b][:, 2 * h:2 * h + 2, :], k[cu[b]:cu[b + 1], h, :], 1 / np.sqrt(d))
            assert np.array_equal(s[h, cu[b]:cu[b + 1]], alone)
    # a length-1 sequence attends only to itself
    assert np.allclose(s[:, 3], 1.0)


@pytest.mark.parametrize("planted", ["transposed", "no_scale", "mean_over_w"])
def test_pins_catch_planted_mistakes(planted):
    # plausible mistakes, planted in a copy of the computation on the CPU, must
    # break agreement with the independent n x n construction above
    r = rng(10)
    n, w, d = 30, 5, 8
    q_all, k = r.standard_normal((n, d)), r.standard_normal((n, d))
    scale = 1 / np.sqrt(d)
    good = O.score_unit(q_all[n - w:, None, :], k, scale)
    if planted == "transposed":
        bad = O.score_unit(k[n - w:, None, :], q_all, scale)
    elif planted == "no_scale":
        bad = O.score_unit(q_all[n - w:, None, :], k, 1.0)
    else:
        P = O.window_attention(q_all[n - w:], k, scale)
        bad = P.sum(axis=0) / w
    assert not np.allclose(good, bad, rtol=1e-6)
