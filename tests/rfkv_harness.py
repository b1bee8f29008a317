"""Shared helpers of the GPU parity tests and the smoke check: run a synthetic layer through librfkv
(paper_2502_16886_amd.device) and compare the results with the float64 oracle.  Not collected by pytest."""
from __future__ import annotations

import numpy as np

from oracle import refreekv_oracle as O
from paper_2502_16886_amd import binding as B
from paper_2502_16886_amd import workloads as W
from paper_2502_16886_amd.device import DeviceLayer, LayerSet, compress_model, threshold_as_float32, to_device, to_host_bits, unit_slices  # noqa: F401

# Relative error allowed on a score (bf16 or fp32 inputs, fp32 accumulation); scores below
# `SCORE_ATOL` (far under anything that can influence a cut) are compared absolutely.
SCORE_RTOL = 1e-3
SCORE_ATOL = 1e-30
# Bound used to decide whether a cut may legitimately move: the fp32 pipeline (MFMA accumulate,
# one fused multiply-add, one hardware exp2 per term) keeps every score within this relative
# error of the exact value; measured errors are reported next to it by the tests (up to 1.3e-6 with
# a 32-row window; up to 2.3e-6 with the paper's k = 1, where a score is the mean of only G terms and
# the fp32 accumulation error of a large sink logit, ~3 ulp of a raw q.k near 100, does not average out).
SCORE_EPS_FOR_CUT = 4e-6



def oracle_layer(layer: W.Layer, rank_mode, threshold=None, min_keep=0, n_sink=None, scores=None) -> dict:
    c = layer.cfg
    T = threshold_as_float32(c.threshold if threshold is None else threshold)
    m = c.n_sink if n_sink is None else n_sink
    if scores is None:
        scores = O.oracle_score(layer.f64("q_win"), layer.f64("k"), layer.cu_seqlens, c.n_q_heads, c.n_kv_heads,
                                c.window)
    kept, offs, idx = O.oracle_select(scores, layer.cu_seqlens, rank_mode, m, T, min_keep, form="cumsum")
    k_out, v_out = O.oracle_compact(layer.k, layer.v, layer.cu_seqlens, kept, offs, idx)
    return dict(scores=scores, kept=kept, out_offsets=offs, idx=idx, k_out=k_out, v_out=v_out)


def score_errors(gpu_scores: np.ndarray, ref_scores: np.ndarray):
    """(max relative error over entries above SCORE_ATOL, number of violations of the tolerance)."""
    ref = ref_scores
    err = np.abs(gpu_scores.astype(np.float64) - ref)
    bad = err > SCORE_RTOL * np.abs(ref) + SCORE_ATOL
    big = np.abs(ref) > 1e-25
    rel = float((err[big] / np.abs(ref[big])).max()) if big.any() else 0.0
    return rel, int(bad.sum())


def cut_is_robust(scores_unit, rank_mode, n_sink, T, eps=SCORE_EPS_FOR_CUT):
    """The oracle's cut cannot move when every score is perturbed by up to `eps` relative
    (and, in score ranking, the scores on both sides of the cut differ by more than 1e-3)."""
    n = len(scores_unit)
    if n == 0:
        return True
    robust, i_star = O.cut_robustness(scores_unit, rank_mode, n_sink, T, rel=1e-3)
    if not robust or T <= 0 or T >= 1:
        return robust
    rank = O.rank_positions(scores_unit, rank_mode, n_sink)
    s = np.asarray(scores_unit, np.float64)[rank]
    P = np.cumsum(s * s)
    F2 = P[-1]
    if F2 == 0:
        return True
    tau = (1 - T) ** 2
    g_hi = P[i_star - 1] / F2
    g_lo = P[i_star - 2] / F2 if i_star >= 2 else 0.0
    # scaling the kept part by (1+eps) and the rest by (1-eps) moves g by about 4 eps g (1 - g)
    slack = 4 * eps * max(g_hi * (1 - g_hi), g_lo * (1 - g_lo))
    return min(g_hi - tau, tau - g_lo) > slack


def compare_layer(layer: W.Layer, gpu: dict, rank_mode, threshold=None, min_keep=0, n_sink=None,
                  ref: dict | None = None) -> dict:
    """Full parity check of one rfkv_compress_layer result; raises AssertionError on a violation.

    1. scores: every entry within SCORE_RTOL of the oracle.
    2. selection, stage-exact: the oracle's rule applied to the GPU's own scores must give exactly
       the GPU's kept counts and index lists (integer work: bit-exact, every unit).
    3. compaction: the GPU's K/V rows are, bit for bit, the input rows at the GPU's indices.
    4. end to end: on every cut-robust unit the retained set (hence the compacted K/V) equals the
       oracle's computed from scratch in float64; on the others the cut may move by a few ranks.
    """
    c = layer.cfg
    T = threshold_as_float32(c.threshold if threshold is None else threshold)
    m = c.n_sink if n_sink is None else n_sink
    if ref is None:
        ref = oracle_layer(layer, rank_mode, threshold, min_keep, n_sink)
    rel, nbad = score_errors(gpu["scores"], ref["scores"])
    assert nbad == 0, f"{nbad} scores off by more than {SCORE_RTOL} relative (max {rel:.3e})"

    # 2. oracle select on the GPU's scores
    own = oracle_layer(layer, rank_mode, threshold, min_keep, n_sink, scores=gpu["scores"].astype(np.float64))
    assert np.array_equal(gpu["kept"], own["kept"]), \
        f"kept differs from the rule applied to the GPU's scores: {gpu['kept']} vs {own['kept']}"
    assert np.array_equal(gpu["out_offsets"], own["out_offsets"])
    assert np.array_equal(gpu["idx"], own["idx"]), "index lists differ from the rule applied to the GPU's scores"
    # 3. compaction is a bit-exact gather
    assert np.array_equal(gpu["k_out"], own["k_out"]) and np.array_equal(gpu["v_out"], own["v_out"])

    # 4. end to end against the oracle's own scores
    n_units = n_robust = n_exact = 0
    worst_shift = 0
    for u, b, h, s, e in unit_slices(layer):
        n_units += 1
        su = ref["scores"][h, s:e]
        robust = min_keep > 0 or cut_is_robust(su, rank_mode, m, T)
        go, gk = int(gpu["out_offsets"][u]), int(gpu["kept"][u])
        ro, rk = int(ref["out_offsets"][u]), int(ref["kept"][u])
        same = gk == rk and np.array_equal(gpu["idx"][go:go + gk], ref["idx"][ro:ro + rk])
        n_exact += same
        n_robust += robust
        worst_shift = max(worst_shift, abs(gk - rk))
        if robust:
            assert same, f"unit {u} (b={b}, h={h}) is cut-robust but kept {gk} vs oracle {rk}"
            assert np.array_equal(gpu["k_out"][go:go + gk], ref["k_out"][ro:ro + rk])
            assert np.array_equal(gpu["v_out"][go:go + gk], ref["v_out"][ro:ro + rk])
        else:
            if rank_mode == O.RANK_POSITION:
                assert abs(gk - rk) <= 2, f"unit {u}: razor-edge cut moved by {gk - rk}"
            else:
                # the symmetric difference may only hold positions whose score ties the cut score
                a, bset = set(gpu["idx"][go:go + gk].tolist()), set(ref["idx"][ro:ro + rk].tolist())
                diff = np.array(sorted(a ^ bset), dtype=np.int64)
                if len(diff):
                    cut_score = np.sort(su)[::-1][max(rk, 1) - 1]
                    assert np.all(np.abs(su[diff] - cut_score) <= 2e-3 * cut_score + 1e-30), \
                        f"unit {u}: sets differ away from the cut"
    return dict(units=n_units, robust=int(n_robust), exact=int(n_exact), robust_frac=round(n_robust / max(1, n_units), 4),
                not_robust_frac=round(1.0 - n_robust / max(1, n_units), 4), max_rel_score_err=rel,
                worst_shift=worst_shift,
                retained=float(gpu["kept"].sum()) / max(1, layer.cfg.n_kv_heads * int(layer.cu_seqlens[-1])))
