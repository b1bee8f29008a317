"""Pins for the oracle's ranking + Uni-Metric budget rule (Sec. 3.2, Eq. 1, Eq. 3)
and for compaction (Alg. 1).  Closed forms are derived by hand in the comments;
brute force enumerates subsets / prefixes straight from the paper's wording."""
import itertools
import math

import numpy as np
import pytest

from oracle import refreekv_oracle as O

POS, SCO = O.RANK_POSITION, O.RANK_SCORE


# ---------------------------------------------------------------- ranking
def test_position_rank_is_first_m_then_reversed_rest():
    # X^ = {x1..xm, xn, xn-1, ..., xm+1} (1-based) with m = 4, n = 9
    r = O.rank_positions(np.zeros(9), POS, 4)
    assert list(r + 1) == [1, 2, 3, 4, 9, 8, 7, 6, 5]
    assert list(O.rank_positions(np.zeros(3), POS, 4)) == [0, 1, 2]          # n <= m
    assert list(O.rank_positions(np.zeros(4), POS, 4)) == [0, 1, 2, 3]
    assert list(O.rank_positions(np.zeros(5), POS, 0)) == [4, 3, 2, 1, 0]


def test_score_rank_descending_ties_lowest_index():
    s = np.array([0.2, 0.5, 0.2, 0.9, 0.5, 0.0])
    assert list(O.rank_positions(s, SCO, 4)) == [3, 1, 4, 0, 2, 5]


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("n,T", [(512, 0.01), (1000, 0.05), (37, 0.2), (8192, 0.01)])
def test_uniform_scores_closed_form(n, T):
    # all s equal: ||A_i|| / ||A|| = sqrt(i/n); 1 - sqrt(i/n) < T  <=>  i > (1-T)^2 n
    s = np.full(n, 1.0 / n)
    x = (1 - T) ** 2 * n
    assert abs(x - round(x)) > 1e-6          # keep away from an exact tie
    expect = math.floor(x) + 1
    assert O.budget_cumsum(s, T) == expect
    if n <= 1000:
        assert O.budget_definition(s, T) == expect
    if n == 512:
        assert expect == 502


def test_strict_inequality_at_exact_equality():
    # n = 4, s = 1: ratios 1 - sqrt(i/4) = 0.5, 0.2929, 0.1340, 0.  With T = 0.5 the
    # first i satisfying the strict "< T" of Eq. 1 is i = 2 (a "<=" would give 1).
    s = np.ones(4)
    assert O.budget_cumsum(s, 0.5) == 2
    assert O.budget_definition(s, 0.5) == 2


@pytest.mark.parametrize("r", [1, 3, 10])
def test_one_hot_at_rank_r(r):
    s = np.zeros(10)
    s[r - 1] = 0.7
    assert O.budget_cumsum(s, 0.01) == r
    assert O.budget_definition(s, 0.01) == r


@pytest.mark.parametrize("q,n,T", [(0.9, 200, 0.01), (0.5, 40, 0.001), (0.99, 3000, 0.01)])
def test_geometric_closed_form(q, n, T):
    # s[r] = q^r: P_i / F^2 = (1 - q^{2i}) / (1 - q^{2n}); first i with P_i/F^2 > (1-T)^2
    s = q ** np.arange(1, n + 1)
    tau = (1 - T) ** 2
    x = math.log(1 - tau * (1 - q ** (2 * n))) / math.log(q * q)   # P_i/F^2 > tau <=> i > x
    assert abs(x - round(x)) > 1e-6
    expect = min(n, math.floor(x) + 1)
    assert O.budget_cumsum(s, T) == expect
    if n <= 200:
        assert O.budget_definition(s, T) == expect


def test_two_level_closed_form():
    # a sinks of weight alpha followed by (n - a) ones:
    # P_i = a alpha^2 + (i - a) for i >= a;  F^2 = a alpha^2 + n - a
    a, alpha, n, T = 4, 30.0, 1000, 0.01
    s = np.concatenate([np.full(a, alpha), np.ones(n - a)])
    F2 = a * alpha ** 2 + n - a
    x = (1 - T) ** 2 * F2 - a * alpha ** 2 + a      # need i > x
    expect = math.floor(x) + 1
    assert a < expect < n
    assert O.budget_cumsum(s, T) == expect
    assert O.budget_definition(s, T) == expect
    # sinks heavy enough -> the cut falls inside the sinks: need j alpha^2 > tau F^2
    s2 = np.concatenate([np.full(a, 1000.0), np.ones(n - a)])
    F2 = a * 1000.0 ** 2 + n - a
    expect2 = math.floor((1 - T) ** 2 * F2 / 1000.0 ** 2) + 1
    assert expect2 == 4
    assert O.budget_cumsum(s2, T) == expect2


# ---------------------------------------------------------------- definition vs Eq. 3
@pytest.mark.parametrize("seed", range(6))
def test_definition_form_equals_cumsum_form(seed):
    r = np.random.default_rng(seed)
    n = int(r.integers(1, 700))
    s = r.lognormal(0, 2, n)
    for T in (0.0, 1e-4, 0.01, 0.1, 0.5, 0.999, 1.0, 1.5):
        assert O.budget_definition(s, T) == O.budget_cumsum(s, T)


def test_norm_of_masked_vector_is_sqrt_of_cumsum():
    # Eq. 3's identity itself, element by element
    r = np.random.default_rng(11)
    s = r.random(50)
    C = np.sqrt(np.cumsum(s * s))
    for i in range(1, 51):
        m = s.copy()
        m[i:] = 0
        assert abs(np.linalg.norm(m) - C[i - 1]) < 1e-14


# ---------------------------------------------------------------- limits / invariants
def test_threshold_limits_and_monotonicity():
    r = np.random.default_rng(12)
    s = r.lognormal(0, 1.5, 300)
    for mode in (POS, SCO):
        kept0, idx0 = O.select_unit(s, mode, 4, 0.0)
        assert kept0 == 300 and np.array_equal(idx0, np.arange(300))       # T = 0 keeps all
        assert O.select_unit(s, mode, 4, 1.0)[0] == 1                      # 1 - x < 1 at i = 1
        assert O.select_unit(s, mode, 4, 2.0)[0] == 1
        last = 301
        for T in (0.0, 1e-5, 1e-3, 0.01, 0.05, 0.2, 0.6, 1.0):
            kept = O.select_unit(s, mode, 4, T)[0]
            assert kept <= last
            last = kept
        # rescaling A' (sum instead of mean over heads / rows) changes nothing
        assert O.select_unit(s * 37.5, mode, 4, 0.01)[0] == O.select_unit(s, mode, 4, 0.01)[0]
    # descending order maximises every prefix mass -> never keeps more than position order
    assert O.select_unit(s, SCO, 4, 0.01)[0] <= O.select_unit(s, POS, 4, 0.01)[0]


def test_zero_scores_and_min_keep():
    assert O.select_unit(np.zeros(9), POS, 4, 0.01)[0] == 9          # F = 0 -> keep all
    s = np.zeros(20)
    s[0] = 1.0
    assert O.select_unit(s, POS, 4, 0.01)[0] == 1
    kept, idx = O.select_unit(s, POS, 4, 0.01, min_keep=7)
    assert kept == 7 and list(idx) == [0, 1, 2, 3, 17, 18, 19]
    assert O.select_unit(s, POS, 4, 0.01, min_keep=50)[0] == 20


def test_all_equal_scores_keep_lowest_indices_in_score_mode():
    n, T = 101, 0.1          # 0.81 * 101 is not an integer: no razor edge
    kept, idx = O.select_unit(np.full(n, 0.01), SCO, 4, T)
    assert kept == math.floor(0.81 * n) + 1
    assert np.array_equal(idx, np.arange(kept))


def test_position_mode_retained_set_is_sinks_plus_suffix():
    r = np.random.default_rng(13)
    s = r.random(200)
    kept, idx = O.select_unit(s, POS, 4, 0.05)
    assert 4 < kept < 200
    assert np.array_equal(idx, np.concatenate([np.arange(4), np.arange(200 - (kept - 4), 200)]))


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("seed", range(8))
def test_score_mode_is_minimum_cardinality_subset(seed):
    # over ALL subsets S: smallest |S| with 1 - ||A'_S|| / ||A'|| < T
    r = np.random.default_rng(100 + seed)
    n = int(r.integers(2, 15))
    s = r.lognormal(0, 1.0, n)
    T = float(r.choice([0.01, 0.05, 0.2]))
    F = np.sqrt((s * s).sum())
    best = n
    for bits in range(1, 1 << n):
        sel = np.array([(bits >> j) & 1 for j in range(n)], dtype=bool)
        if 1.0 - np.sqrt((s[sel] ** 2).sum()) / F < T:
            best = min(best, int(sel.sum()))
    kept, idx = O.select_unit(s, SCO, 4, T)
    assert kept == best
    assert 1.0 - np.sqrt((s[idx] ** 2).sum()) / F < T             # and the oracle's set attains it


@pytest.mark.parametrize("seed", range(8))
def test_position_mode_prefix_enumeration(seed):
    # enumerate the prefixes of X^ built literally from the paper's 1-based wording
    r = np.random.default_rng(200 + seed)
    n = int(r.integers(1, 64))
    m = int(r.integers(0, 7))
    s = r.lognormal(0, 1.5, n)
    T = float(r.choice([0.01, 0.1]))
    order = list(range(1, min(m, n) + 1)) + list(range(n, min(m, n), -1))      # 1-based X^
    F = math.sqrt(sum(x * x for x in s))
    expect = n
    for i in range(1, n + 1):
        norm = math.sqrt(sum(s[p - 1] ** 2 for p in order[:i]))
        if 1 - norm / F < T:
            expect = i
            break
    kept, idx = O.select_unit(s, POS, m, T)
    assert kept == expect
    assert sorted(p - 1 for p in order[:expect]) == list(idx)


# ---------------------------------------------------------------- batch layout + compaction
def _random_batch(seed, lens, Hq=4, Hkv=2, d=8, w=5):
    r = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    q = np.concatenate([r.standard_normal((min(w, n), Hq, d)) for n in lens])
    k = r.standard_normal((cu[-1], Hkv, d))
    v = r.standard_normal((cu[-1], Hkv, d))
    return q, k, v, cu, Hq, Hkv, d, w


def test_full_budget_reproduces_cache_exactly():
    q, k, v, cu, Hq, Hkv, d, w = _random_batch(20, [17, 5, 33])
    k32, v32 = k.astype(np.float32), v.astype(np.float32)
    for mode in (POS, SCO):
        out = O.oracle_compress_layer(q, k, k32, v32, cu, Hq, Hkv, w, T=0.0, rank_mode=mode)
        assert np.array_equal(out["kept"], np.repeat(np.diff(cu), Hkv))
        o = 0
        for b in range(len(cu) - 1):
            for h in range(Hkv):
                n = cu[b + 1] - cu[b]
                assert np.array_equal(out["k_out"][o:o + n].view(np.uint32),
                                      k32[cu[b]:cu[b + 1], h].view(np.uint32))
                assert np.array_equal(out["v_out"][o:o + n].view(np.uint32),
                                      v32[cu[b]:cu[b + 1], h].view(np.uint32))
                o += n


def test_model_loop_retains_the_bottom_layers_whole():
    # Sec. 3.3 "Retaining Bottom Layers": the first two layers are not pruned, the others are;
    # a retained layer holds every row of every head in order, whatever its attention looks like
    layers = []
    for li in range(4):
        q, k, v, cu, Hq, Hkv, d, w = _random_batch(30 + li, [23, 6, 31])
        k[cu[:-1]] *= 6.0                                    # a heavy first key: the rule would prune a lot
        layers.append((q, k, k.astype(np.float32), v.astype(np.float32), cu))
    res = O.oracle_compress_model(layers, Hq, Hkv, w, n_frozen=2, T=0.2)
    lens = np.repeat(np.diff(cu), Hkv)
    for li, (r, (q, k, k32, v32, _)) in enumerate(zip(res, layers)):
        alone = O.oracle_compress_layer(q, k, k32, v32, cu, Hq, Hkv, w, T=0.2)
        if li < 2:
            assert np.array_equal(r["kept"], lens) and alone["kept"].sum() < lens.sum()
            o = 0
            for b in range(len(cu) - 1):
                for h in range(Hkv):
                    n = cu[b + 1] - cu[b]
                    assert np.array_equal(r["idx"][o:o + n], np.arange(n))
                    assert np.array_equal(r["k_out"][o:o + n].view(np.uint32), k32[cu[b]:cu[b + 1], h].view(np.uint32))
                    assert np.array_equal(r["v_out"][o:o + n].view(np.uint32), v32[cu[b]:cu[b + 1], h].view(np.uint32))
                    o += n
        else:
            for key in ("kept", "out_offsets", "idx", "k_out", "v_out"):
                assert np.array_equal(r[key], alone[key])
    # n_frozen = 0 prunes every layer
    assert O.oracle_compress_model(layers[:1], Hq, Hkv, w, n_frozen=0, T=0.2)[0]["kept"].sum() < lens.sum()


@pytest.mark.parametrize("mode", [POS, SCO])
def test_attention_over_compacted_cache_equals_masked_full_attention(mode):
    q, k, v, cu, Hq, Hkv, d, w = _random_batch(21, [64, 9, 40])
    out = O.oracle_compress_layer(q, k, k, v, cu, Hq, Hkv, w, T=0.2, rank_mode=mode)
    r = np.random.default_rng(5)
    assert out["out_offsets"][0] == 0 and np.array_equal(np.diff(out["out_offsets"]), out["kept"])
    shrunk = 0
    for b in range(len(cu) - 1):
        n = cu[b + 1] - cu[b]
        for h in range(Hkv):
            u = b * Hkv + h
            o, c = out["out_offsets"][u], out["kept"][u]
            idx = out["idx"][o:o + c]
            assert np.all(np.diff(idx) > 0) and idx.min() >= 0 and idx.max() < n
            shrunk += c < n
            qn = r.standard_normal((3, d))
            mask = np.zeros(n, dtype=bool)
            mask[idx] = True
            full = O.attention_output(qn, k[cu[b]:cu[b + 1], h], v[cu[b]:cu[b + 1], h], 0.35, mask)
            comp = O.attention_output(qn, out["k_out"][o:o + c], out["v_out"][o:o + c], 0.35)
            assert np.allclose(full, comp, rtol=1e-12, atol=1e-12)
            # any row order gives the same attention output
            perm = r.permutation(c)
            comp2 = O.attention_output(qn, out["k_out"][o:o + c][perm], out["v_out"][o:o + c][perm], 0.35)
            assert np.allclose(full, comp2, rtol=1e-12, atol=1e-12)
    assert shrunk > 0


def test_cut_robustness_flags_razor_edges():
    # uniform scores where (1-T)^2 n is an integer: the crossing sits exactly on a step edge
    n, T = 100, 0.1
    robust, i_star = O.cut_robustness(np.full(n, 0.01), POS, 0, T)
    assert not robust
    s = np.random.default_rng(3).lognormal(0, 1, 500)
    robust, i_star = O.cut_robustness(s, POS, 4, 0.01)
    assert i_star == O.select_unit(s, POS, 4, 0.01)[0]
