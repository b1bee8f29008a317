"""Pins of the oracle's per-layer cut (one stopping position per layer and sequence, norm over all
heads): reductions to the per-head rule, closed forms, brute force, invariants."""
import itertools

import numpy as np
import pytest

from oracle import refreekv_oracle as O

MODES = [O.RANK_POSITION, O.RANK_SCORE]


@pytest.mark.parametrize("mode", MODES)
def test_one_head_is_the_per_head_rule(mode):
    rng = np.random.default_rng(1)
    s = rng.random((1, 200)) ** 4
    for T in (0.0, 0.01, 0.2, 0.9, 1.5):
        k1, i1 = O.select_unit(s[0], mode, 4, T)
        k2, i2 = O.select_layer(s, mode, 4, T)
        assert k1 == k2 and np.array_equal(i1, i2[0])


@pytest.mark.parametrize("mode", MODES)
def test_identical_heads_cut_where_each_head_would(mode):
    """H copies of one head scale every norm by sqrt(H): the ratio, hence the cut, is unchanged."""
    rng = np.random.default_rng(2)
    row = rng.random(300) ** 3
    k1, i1 = O.select_unit(row, mode, 4, 0.02)
    k2, i2 = O.select_layer(np.tile(row, (5, 1)), mode, 4, 0.02)
    assert k1 == k2 and all(np.array_equal(i1, x) for x in i2)


def test_uniform_scores_closed_form():
    # every prefix of i ranks holds i/n of the squared mass in every head: i* = floor((1-T)^2 n) + 1
    n, T = 1001, 0.01
    k, idx = O.select_layer(np.full((3, n), 0.7), O.RANK_POSITION, 4, T)
    assert k == int(np.floor((1 - T) ** 2 * n)) + 1
    assert np.array_equal(idx[0], np.concatenate([np.arange(4), np.arange(n - (k - 4), n)]))


def test_a_heavy_head_dominates_the_shared_cut():
    """Head 0 carries almost all the mass in its first rank; head 1 is flat and negligible.  The shared
    cut follows head 0 (keep one position), while head 1 alone would keep almost everything."""
    n = 400
    A = np.full((2, n), 1e-6)
    A[0, 0] = 1.0
    k, idx = O.select_layer(A, O.RANK_SCORE, 4, 0.01)
    assert k == 1 and np.array_equal(idx[0], [0]) and np.array_equal(idx[1], [0])
    k_flat, _ = O.select_unit(A[1], O.RANK_SCORE, 4, 0.01)
    assert k_flat > 0.9 * n


@pytest.mark.parametrize("mode", MODES)
def test_definition_form_equals_cumulative_form(mode):
    rng = np.random.default_rng(3)
    for _ in range(20):
        A = rng.random((rng.integers(1, 5), rng.integers(1, 60))) ** rng.integers(1, 6)
        T = float(rng.choice([0.001, 0.01, 0.1, 0.5]))
        a = O.select_layer(A, mode, 4, T, form="definition")
        b = O.select_layer(A, mode, 4, T, form="cumsum")
        assert a[0] == b[0] and all(np.array_equal(x, y) for x, y in zip(a[1], b[1]))


def test_score_ranking_brute_force_equal_counts():
    """Among all ways to keep the same number c of positions in every head, the per-head top-c keeps
    the most mass; so i* is the smallest c for which ANY equal-count choice meets the rule."""
    rng = np.random.default_rng(4)
    for _ in range(5):
        H, n, T = 2, 6, 0.15
        A = rng.random((H, n)) ** 3
        F2 = np.sum(A * A)
        best = n
        for c in range(1, n + 1):
            ok = False
            for sets in itertools.product(itertools.combinations(range(n), c), repeat=H):
                mass = sum(np.sum(A[h, list(sets[h])] ** 2) for h in range(H))
                if 1 - np.sqrt(mass / F2) < T:
                    ok = True
                    break
            if ok:
                best = c
                break
        k, idx = O.select_layer(A, O.RANK_SCORE, 4, T)
        assert k == best
        mass = sum(np.sum(A[h, idx[h]] ** 2) for h in range(H))
        assert 1 - np.sqrt(mass / F2) < T


def test_position_ranking_literal_prefixes():
    rng = np.random.default_rng(5)
    A = rng.random((3, 40)) ** 4
    m, T = 4, 0.05
    order = list(range(m)) + list(range(39, m - 1, -1))
    F = np.sqrt(np.sum(A * A))
    want = next(i for i in range(1, 41) if 1 - np.sqrt(np.sum(A[:, order[:i]] ** 2)) / F < T)
    k, idx = O.select_layer(A, O.RANK_POSITION, m, T)
    assert k == want and all(np.array_equal(x, np.sort(order[:want])) for x in idx)


@pytest.mark.parametrize("mode", MODES)
def test_limits_and_invariants(mode):
    rng = np.random.default_rng(6)
    A = rng.random((4, 150)) ** 3
    assert O.select_layer(A, mode, 4, 0.0)[0] == 150          # strict inequality: T = 0 keeps everything
    assert O.select_layer(A, mode, 4, 1.0)[0] == 1
    assert O.select_layer(np.zeros((2, 9)), mode, 4, 0.01)[0] == 9
    ks = [O.select_layer(A, mode, 4, T)[0] for T in (0.001, 0.01, 0.05, 0.2, 0.6)]
    assert ks == sorted(ks, reverse=True)
    assert O.select_layer(3.7 * A, mode, 4, 0.01)[0] == O.select_layer(A, mode, 4, 0.01)[0]
    assert O.select_layer(A, mode, 4, 0.5, min_keep=120)[0] == 120


def test_batched_form_offsets_and_equal_counts():
    rng = np.random.default_rng(7)
    cu = np.array([0, 50, 50, 130])
    S = rng.random((3, 130)) ** 4
    kept, offs, idx = O.oracle_select_layer(S, cu, O.RANK_POSITION, 4, 0.02)
    assert kept.shape == (9,) and np.all(kept[0:3] == kept[0]) and np.all(kept[3:6] == 0) and np.all(kept[6:9] == kept[6])
    assert np.array_equal(offs, np.concatenate([[0], np.cumsum(kept)]))
    assert len(idx) == offs[-1]
