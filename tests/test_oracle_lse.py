"""Pins of the oracle's scoring from given row normalisers (log-sum-exp of the window rows as an input)."""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import refreekv_oracle as O


def _inputs(seed, lens, Hq, Hkv, d, w):
    rng = np.random.default_rng(seed)
    N = int(sum(lens))
    rows = int(sum(min(w, n) for n in lens))
    q = rng.standard_normal((rows, Hq, d)) * 1.5
    k = rng.standard_normal((N, Hkv, d))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return q, k, cu


def test_window_lse_is_the_library_logsumexp_of_the_visible_logits():
    rng = np.random.default_rng(0)
    n, wp, d = 37, 6, 16
    q, k = rng.standard_normal((wp, d)) * 2, rng.standard_normal((n, d))
    scale = 0.3
    got = O.window_lse(q, k, scale)
    for t in range(wp):
        last = n - wp + t
        assert got[t] == pytest.approx(logsumexp(scale * (k[: last + 1] @ q[t])), rel=1e-13)


def test_large_logits_do_not_overflow():
    q = np.full((1, 4), 30.0)
    k = np.full((5, 4), 30.0)
    lse = O.window_lse(q, k, 1.0)
    assert np.isfinite(lse).all() and lse[0] == pytest.approx(3600.0 + np.log(5.0))


@pytest.mark.parametrize("lens,Hq,Hkv,w", [([50], 4, 2, 8), ([9, 33, 1], 6, 2, 5), ([20, 4], 2, 2, 7)])
def test_scores_from_exact_lse_equal_the_softmax_row_scores(lens, Hq, Hkv, w):
    q, k, cu = _inputs(1, lens, Hq, Hkv, 8, w)
    lse = O.oracle_window_lse(q, k, cu, Hq, Hkv, w)
    a = O.oracle_score(q, k, cu, Hq, Hkv, w)
    b = O.oracle_score_lse(q, lse, k, cu, Hq, Hkv, w)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-300)


def test_k1_scores_from_lse_are_a_library_softmax():
    # window 1, G = 1: the score vector is the softmax of the last row
    q, k, cu = _inputs(2, [40], 1, 1, 8, 1)
    scale = 1 / np.sqrt(8)
    lse = O.oracle_window_lse(q, k, cu, 1, 1, 1)
    got = O.oracle_score_lse(q, lse, k, cu, 1, 1, 1)[0]
    assert np.allclose(got, softmax(scale * (k[:, 0] @ q[0, 0])), rtol=1e-12)


def test_shift_law_a_row_with_lse_plus_ln2_counts_half():
    # G = 2, window 1: score = (p_0 + p_1) / 2; raising head 1's lse by ln 2 halves p_1
    q, k, cu = _inputs(3, [30], 2, 1, 8, 1)
    lse = O.oracle_window_lse(q, k, cu, 2, 1, 1)
    scale = 1 / np.sqrt(8)
    p0 = softmax(scale * (k[:, 0] @ q[0, 0]))
    p1 = softmax(scale * (k[:, 0] @ q[0, 1]))
    lse2 = lse.copy()
    lse2[0, 1] += np.log(2.0)
    got = O.oracle_score_lse(q, lse2, k, cu, 2, 1, 1)[0]
    assert np.allclose(got, (p0 + 0.5 * p1) / 2, rtol=1e-12)


def test_causal_rows_use_their_own_visible_prefix():
    # window 3 over n = 5, G = 1: brute force over the three rows
    q, k, cu = _inputs(4, [5], 1, 1, 4, 3)
    scale = 0.5
    lse = O.oracle_window_lse(q, k, cu, 1, 1, 3, scale=scale)
    got = O.oracle_score_lse(q, lse, k, cu, 1, 1, 3, scale=scale)[0]
    want = np.zeros(5)
    cnt = np.zeros(5)
    for t in range(3):
        last = 5 - 3 + t
        want[: last + 1] += softmax(scale * (k[: last + 1, 0] @ q[t, 0]))
        cnt[: last + 1] += 1
    assert np.allclose(got, want / cnt, rtol=1e-12)
