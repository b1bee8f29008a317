"""Float64 CPU oracle for the ReFreeKV post-prefill compression pass.

TEST INFRASTRUCTURE ONLY.  This module is the yardstick the HIP path is judged
against; it is imported by the tests, by the smoke check and by the benchmark's
CPU-baseline leg, and by nothing else.  It shares no code with the GPU path and
must never be used as a fallback for it.

Everything here is written from the paper's definitions, slowly and plainly:

* window attention rows  -- causal softmax(Q K^T / sqrt(d)) for the last k query
  positions (Sec. 3.2 "Reducing Overhead"; Alg. 1, the `Attention(Q[-1], K^T)` step);
* the reduced vector A'  -- column mean of those rows over the rows that can see
  the column (Eq. 2);
* GQA reduction          -- mean of A' over the query heads sharing a KV head
  (the paper is silent; any positive rescaling leaves the budget rule unchanged);
* initial ranking        -- position based, first m then the rest reversed
  (Sec. 3.2 "Initial Ranking"), or by descending score (Sec. 4.4 ablation);
* Uni-Metric budget rule -- leftmost ranked prefix whose Frobenius norm is
  within T of the full norm (Eq. 1), in the masked-norm *definition* form and in
  the cumulative square-sum form (Eq. 3);
* compaction             -- gather of the retained K/V rows (Alg. 1, last steps),
  emitted in ascending original position;
* decode attention       -- softmax(q K_c^T / sqrt(d)) V_c of new queries over the compacted
  ragged cache, and the same over the full cache with evicted positions masked;
* scores from given row normalisers -- the window rows' log-sum-exp as an input (what the
  prefill's attention forward keeps), exp(logit - lse) in place of the softmax rows.

All floating point is float64.  Inputs arrive already upcast (bf16/fp32 -> fp64
is exact), so the oracle sees the same values the GPU sees.

Pinned by tests/test_oracle_*.py: softmax row sums, the k = 1 special case
against a library softmax, the full n x n attention matrix on tiny inputs,
closed forms of the budget rule (uniform / one-hot / geometric / two-level),
definition-form == cumsum-form, exhaustive subset search for the score ranking,
literal prefix enumeration for the position ranking, T = 0 / T >= 1 limits,
attention over the compacted cache == masked full attention, and the decode
attention against a library scaled-dot-product attention, a single-key cache and an
all-equal-keys cache; the log-sum-exp against scipy's, scores from it against the
softmax-row scores, and its shift law (lse + ln 2 halves a row's share).  The paper
prints no worked numeric example of the rule, so there is no paper-value pin;
results on the paper's real datasets/models are parity-unpinned.
"""
from __future__ import annotations

import numpy as np

RANK_POSITION = 0   # Sec. 3.2 "Initial Ranking" (paper default)
RANK_SCORE = 1      # Sec. 4.4 "Initial Ranking Strategies" (ablation)

# above this length the O(n^2) definition form is skipped in favour of Eq. 3
DEFINITION_FORM_MAX_N = 4096


# ----------------------------------------------------------------------------
# scoring  (Sec. 3.2 "Reducing Overhead", Eq. 2)
# ----------------------------------------------------------------------------
def window_attention(q_rows: np.ndarray, k_rows: np.ndarray, scale: float) -> np.ndarray:
    """Causal softmax attention of the last w' query positions over all n keys.

    q_rows [w', d], k_rows [n, d] (float64).  Row t is the query at absolute
    position n - w' + t; it sees keys 0 .. n - w' + t.  Returns P [w', n] with
    exact zeros at the causally hidden entries.
    """
    q_rows = np.asarray(q_rows, dtype=np.float64)
    k_rows = np.asarray(k_rows, dtype=np.float64)
    wp, n = q_rows.shape[0], k_rows.shape[0]
    assert wp <= n
    logits = (q_rows @ k_rows.T) * scale
    P = np.zeros((wp, n), dtype=np.float64)
    for t in range(wp):
        last = n - wp + t                      # last visible key of this row
        row = logits[t, : last + 1]
        e = np.exp(row - row.max())
        P[t, : last + 1] = e / e.sum()
    return P


def causal_counts(n: int, wp: int) -> np.ndarray:
    """Number of window rows that can see key i (denominator of Eq. 2)."""
    i = np.arange(n)
    return np.minimum(wp, n - i).astype(np.float64)


def reduced_attention_vector(P: np.ndarray) -> np.ndarray:
    """Eq. 2: per-column mean of the window rows over the rows that see the column."""
    wp, n = P.shape
    return P.sum(axis=0) / causal_counts(n, wp)


def score_unit(q_unit: np.ndarray, k_unit: np.ndarray, scale: float) -> np.ndarray:
    """A' for one (sequence, KV head).  q_unit [w', G, d], k_unit [n, d]."""
    wp, G, _ = q_unit.shape
    n = k_unit.shape[0]
    acc = np.zeros(n, dtype=np.float64)
    for g in range(G):
        acc += reduced_attention_vector(window_attention(q_unit[:, g, :], k_unit, scale))
    return acc / G


def oracle_score(q_win, k, cu_seqlens, n_q_heads, n_kv_heads, window, scale=None):
    """Scores [Hkv, N] for a packed ragged batch.

    q_win [sum_b min(window, n_b), Hq, d] holds, per sequence, the queries of its
    last min(window, n_b) positions; k [N, Hkv, d]; cu_seqlens [B+1].
    """
    q_win = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    N, Hkv, d = k.shape
    assert Hkv == n_kv_heads and n_q_heads % n_kv_heads == 0
    G = n_q_heads // n_kv_heads
    if scale is None or scale == 0:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((Hkv, N), dtype=np.float64)
    q0 = 0
    for b in range(len(cu_seqlens) - 1):
        s, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        n = e - s
        wp = min(window, n)
        for h in range(Hkv):
            if n > 0:
                out[h, s:e] = score_unit(q_win[q0:q0 + wp, h * G:(h + 1) * G, :], k[s:e, h, :], scale)
        q0 += wp
    return out


# ----------------------------------------------------------------------------
# scoring from given row normalisers  (Sec. 3.2 "Reducing Overhead", Eq. 2)
#
# The rows Eq. 2 averages are softmax rows of the causal attention the prefill has just computed;
# an attention forward pass keeps each row's normaliser as a log-sum-exp.  These functions state
# what the scores are when that normaliser is an INPUT: p[t, i] = exp(logit[t, i] - lse[t]).
# ----------------------------------------------------------------------------
def window_lse(q_rows: np.ndarray, k_rows: np.ndarray, scale: float) -> np.ndarray:
    """ln sum_{i <= pos(t)} exp(scale q_t . k_i) for the last w' query positions, [w']."""
    q_rows = np.asarray(q_rows, dtype=np.float64)
    k_rows = np.asarray(k_rows, dtype=np.float64)
    wp, n = q_rows.shape[0], k_rows.shape[0]
    logits = (q_rows @ k_rows.T) * scale
    out = np.empty(wp, dtype=np.float64)
    for t in range(wp):
        row = logits[t, : n - wp + t + 1]
        m = row.max()
        out[t] = m + np.log(np.exp(row - m).sum())
    return out


def oracle_window_lse(q_win, k, cu_seqlens, n_q_heads, n_kv_heads, window, scale=None):
    """The log-sum-exp of every window row, [sum_b min(window, n_b), Hq] (rows as in q_win)."""
    q_win = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    d = k.shape[2]
    G = n_q_heads // n_kv_heads
    if scale is None or scale == 0:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((q_win.shape[0], n_q_heads), dtype=np.float64)
    q0 = 0
    for b in range(len(cu_seqlens) - 1):
        s, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        wp = min(window, e - s)
        for hq in range(n_q_heads):
            if wp > 0:
                out[q0:q0 + wp, hq] = window_lse(q_win[q0:q0 + wp, hq, :], k[s:e, hq // G, :], scale)
        q0 += wp
    return out


def score_unit_from_lse(q_unit: np.ndarray, k_unit: np.ndarray, lse_unit: np.ndarray, scale: float) -> np.ndarray:
    """A' for one (sequence, KV head) with the rows' normalisers given.  q_unit [w', G, d],
    k_unit [n, d], lse_unit [w', G]."""
    wp, G, _ = q_unit.shape
    n = k_unit.shape[0]
    acc = np.zeros(n, dtype=np.float64)
    for g in range(G):
        logits = (q_unit[:, g, :] @ k_unit.T) * scale
        P = np.zeros((wp, n), dtype=np.float64)
        for t in range(wp):
            last = n - wp + t
            P[t, : last + 1] = np.exp(logits[t, : last + 1] - lse_unit[t, g])
        acc += reduced_attention_vector(P)
    return acc / G


def oracle_score_lse(q_win, lse_win, k, cu_seqlens, n_q_heads, n_kv_heads, window, scale=None):
    """Scores [Hkv, N] as oracle_score, with lse_win [sum_b min(window, n_b), Hq] given."""
    q_win = np.asarray(q_win, dtype=np.float64)
    lse_win = np.asarray(lse_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    N, Hkv, d = k.shape
    G = n_q_heads // n_kv_heads
    if scale is None or scale == 0:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((Hkv, N), dtype=np.float64)
    q0 = 0
    for b in range(len(cu_seqlens) - 1):
        s, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        n = e - s
        wp = min(window, n)
        for h in range(Hkv):
            if n > 0:
                out[h, s:e] = score_unit_from_lse(q_win[q0:q0 + wp, h * G:(h + 1) * G, :], k[s:e, h, :],
                                                  lse_win[q0:q0 + wp, h * G:(h + 1) * G], scale)
        q0 += wp
    return out


# ----------------------------------------------------------------------------
# ranking  (Sec. 3.2 "Initial Ranking"; Sec. 4.4 ablation)
# ----------------------------------------------------------------------------
def rank_positions(scores_unit: np.ndarray, rank_mode: int, n_sink: int) -> np.ndarray:
    """Permutation: rank r (0-based) -> position (0-based)."""
    n = len(scores_unit)
    if rank_mode == RANK_POSITION:
        if n <= n_sink:
            return np.arange(n)
        return np.concatenate([np.arange(n_sink), np.arange(n - 1, n_sink - 1, -1)])
    if rank_mode == RANK_SCORE:
        # descending score, equal scores keep ascending position
        return np.argsort(-np.asarray(scores_unit, dtype=np.float64), kind="stable")
    raise ValueError("rank_mode")


# ----------------------------------------------------------------------------
# Uni-Metric budget rule  (Eq. 1, Eq. 3)
# ----------------------------------------------------------------------------
def budget_definition(s_ranked: np.ndarray, T: float) -> int:
    """Eq. 1 literally: for each i build the vector with ranks > i masked out, take
    its norm afresh, stop at the first i with 1 - norm_i / norm_full < T.
    Returns i* in 1..n (n if no i qualifies or the full norm is zero)."""
    s = np.asarray(s_ranked, dtype=np.float64)
    n = len(s)
    F = np.sqrt(np.sum(s * s))
    if n == 0 or F == 0.0:
        return n
    for i in range(1, n + 1):
        masked = s.copy()
        masked[i:] = 0.0
        if 1.0 - np.sqrt(np.sum(masked * masked)) / F < T:
            return i
    return n


def budget_cumsum(s_ranked: np.ndarray, T: float) -> int:
    """Eq. 3: the same rule through the cumulative square-sum."""
    s = np.asarray(s_ranked, dtype=np.float64)
    n = len(s)
    if n == 0:
        return 0
    C = np.sqrt(np.cumsum(s * s))
    F = C[-1]
    if F == 0.0:
        return n
    hit = np.nonzero(1.0 - C / F < T)[0]
    return int(hit[0]) + 1 if len(hit) else n


def select_unit(scores_unit, rank_mode, n_sink, T, min_keep=0, form="auto"):
    """(kept, idx): number of retained positions and their indices, ascending."""
    n = len(scores_unit)
    if n == 0:
        return 0, np.zeros(0, dtype=np.int64)
    rank = rank_positions(scores_unit, rank_mode, n_sink)
    s_ranked = np.asarray(scores_unit, dtype=np.float64)[rank]
    if form == "auto":
        form = "definition" if n <= DEFINITION_FORM_MAX_N else "cumsum"
    i_star = budget_definition(s_ranked, T) if form == "definition" else budget_cumsum(s_ranked, T)
    kept = min(n, max(i_star, int(min_keep)))
    return kept, np.sort(rank[:kept])


def oracle_select(scores, cu_seqlens, rank_mode, n_sink, T, min_keep=0, form="auto"):
    """Per unit u = b*Hkv + h: kept[u]; out_offsets = exclusive scan of kept;
    idx = retained positions (relative to the sequence start), ascending,
    packed unit after unit."""
    Hkv = scores.shape[0]
    B = len(cu_seqlens) - 1
    kept = np.zeros(B * Hkv, dtype=np.int64)
    chunks = []
    for b in range(B):
        s, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        for h in range(Hkv):
            c, idx = select_unit(scores[h, s:e], rank_mode, n_sink, T, min_keep, form)
            kept[b * Hkv + h] = c
            chunks.append(idx)
    offs = np.concatenate([[0], np.cumsum(kept)]).astype(np.int64)
    idx = np.concatenate(chunks) if chunks else np.zeros(0, dtype=np.int64)
    return kept, offs, idx


def select_layer(scores_seq, rank_mode, n_sink, T, min_keep=0, form="auto"):
    """One cut per (layer, sequence) instead of one per head (Fig. 1 evicts "per layer"; Sec. 3.3
    finds "the stopping positions of all layers"): the reduced attention matrix of the layer is
    A' [Hkv, n], every head's row is ranked on its own, the vector masked at rank i keeps ranks
    1..i of every head, and i* is the leftmost i with 1 - ||A~'_i||_F / ||A'||_F < T, the norms
    taken over the whole matrix.  Returns (kept, [idx_h ascending for each head])."""
    A = np.asarray(scores_seq, dtype=np.float64)
    Hkv, n = A.shape
    if n == 0:
        return 0, [np.zeros(0, dtype=np.int64) for _ in range(Hkv)]
    ranks = [rank_positions(A[h], rank_mode, n_sink) for h in range(Hkv)]
    ranked = np.stack([A[h][ranks[h]] for h in range(Hkv)])            # [Hkv, n], rank order per head
    if form == "auto":
        form = "definition" if n * Hkv <= DEFINITION_FORM_MAX_N else "cumsum"
    F = np.sqrt(np.sum(A * A))
    i_star = n
    if F > 0.0:
        if form == "definition":
            for i in range(1, n + 1):
                masked = ranked.copy()
                masked[:, i:] = 0.0
                if 1.0 - np.sqrt(np.sum(masked * masked)) / F < T:
                    i_star = i
                    break
        else:
            C = np.sqrt(np.cumsum(np.sum(ranked * ranked, axis=0)))
            hit = np.nonzero(1.0 - C / C[-1] < T)[0]
            i_star = int(hit[0]) + 1 if len(hit) else n
    kept = min(n, max(i_star, int(min_keep)))
    return kept, [np.sort(ranks[h][:kept]) for h in range(Hkv)]


def oracle_select_layer(scores, cu_seqlens, rank_mode, n_sink, T, min_keep=0, form="auto"):
    """oracle_select with one cut per (layer, sequence): same outputs, every head of a sequence
    keeps the same number of positions."""
    Hkv = scores.shape[0]
    B = len(cu_seqlens) - 1
    kept = np.zeros(B * Hkv, dtype=np.int64)
    chunks = []
    for b in range(B):
        s, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        c, idxs = select_layer(scores[:, s:e], rank_mode, n_sink, T, min_keep, form)
        kept[b * Hkv:(b + 1) * Hkv] = c
        chunks.extend(idxs)
    offs = np.concatenate([[0], np.cumsum(kept)]).astype(np.int64)
    idx = np.concatenate(chunks) if chunks else np.zeros(0, dtype=np.int64)
    return kept, offs, idx


# ----------------------------------------------------------------------------
# compaction  (Alg. 1, "Compress K / V by R")
# ----------------------------------------------------------------------------
def oracle_compact(k, v, cu_seqlens, kept, out_offsets, idx):
    """Gather rows.  k, v [N, Hkv, d] in any storage dtype (moved bit for bit).
    Returns k_out, v_out [sum kept, d]."""
    N, Hkv, d = k.shape
    total = int(out_offsets[-1])
    k_out = np.zeros((total, d), dtype=k.dtype)
    v_out = np.zeros((total, d), dtype=v.dtype)
    B = len(cu_seqlens) - 1
    for b in range(B):
        s = int(cu_seqlens[b])
        for h in range(Hkv):
            u = b * Hkv + h
            o = int(out_offsets[u])
            for t in range(int(kept[u])):
                p = s + int(idx[o + t])
                k_out[o + t] = k[p, h]
                v_out[o + t] = v[p, h]
    return k_out, v_out


def oracle_compress_layer(q_win_f64, k_f64, k_raw, v_raw, cu_seqlens, n_q_heads, n_kv_heads,
                          window, n_sink=4, T=0.01, rank_mode=RANK_POSITION, min_keep=0,
                          scale=None, form="auto"):
    """One layer: score -> rank -> budget rule -> compact (Alg. 1 loop body)."""
    scores = oracle_score(q_win_f64, k_f64, cu_seqlens, n_q_heads, n_kv_heads, window, scale)
    kept, offs, idx = oracle_select(scores, cu_seqlens, rank_mode, n_sink, T, min_keep, form)
    k_out, v_out = oracle_compact(k_raw, v_raw, cu_seqlens, kept, offs, idx)
    return dict(scores=scores, kept=kept, out_offsets=offs, idx=idx, k_out=k_out, v_out=v_out)


def oracle_compress_model(layers, n_q_heads, n_kv_heads, window, n_frozen=2, **kw):
    """Alg. 1's loop over layers with Sec. 3.3 "Retaining Bottom Layers": the first n_frozen
    layers are not pruned (every position of every head is retained, in order), the others go
    through oracle_compress_layer.  `layers`: per layer a tuple (q_win_f64, k_f64, k_raw, v_raw,
    cu_seqlens).  Returns the per-layer result dicts (scores None for the retained layers)."""
    out = []
    for li, (q_win, k_f64, k_raw, v_raw, cu) in enumerate(layers):
        if li >= n_frozen:
            out.append(oracle_compress_layer(q_win, k_f64, k_raw, v_raw, cu, n_q_heads, n_kv_heads, window, **kw))
            continue
        lens = np.diff(np.asarray(cu, dtype=np.int64))
        kept = np.repeat(lens, n_kv_heads)
        offs = np.concatenate([[0], np.cumsum(kept)]).astype(np.int64)
        idx = np.concatenate([np.arange(n, dtype=np.int64) for n in kept]) if len(kept) else np.zeros(0, np.int64)
        k_out, v_out = oracle_compact(k_raw, v_raw, cu, kept, offs, idx)
        out.append(dict(scores=None, kept=kept, out_offsets=offs, idx=idx, k_out=k_out, v_out=v_out))
    return out


# ----------------------------------------------------------------------------
# helpers for the invariants the tests use
# ----------------------------------------------------------------------------
def attention_output(q_new, k_rows, v_rows, scale, keep_mask=None):
    """softmax(q K^T * scale) V for queries that see every key; positions with
    keep_mask == False get logit -inf.  Used for the compaction invariant."""
    logits = (np.asarray(q_new, np.float64) @ np.asarray(k_rows, np.float64).T) * scale
    if keep_mask is not None:
        logits = np.where(keep_mask[None, :], logits, -np.inf)
    logits = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(logits)
    return (e / e.sum(axis=1, keepdims=True)) @ np.asarray(v_rows, np.float64)


def oracle_decode_attention(q_new, k_c, v_c, out_offsets, n_q_heads, n_kv_heads, scale=None):
    """Attention of new queries over the compacted ragged cache (the consumer of Alg. 1's
    compressed K / V; Sec. 4.3 measures its cost): q_new [B, n_new, Hq, d]; the retained rows
    of unit u = b * Hkv + h are k_c / v_c [out_offsets[u] : out_offsets[u + 1]].  Every new
    query sees the whole cache of its sequence and nothing else.  Returns float64
    [B, n_new, Hq, d]; a unit without rows gives zeros."""
    q_new = np.asarray(q_new, np.float64)
    B, n_new, Hq, d = q_new.shape
    G = n_q_heads // n_kv_heads
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    out = np.zeros((B, n_new, Hq, d))
    for b in range(B):
        for h in range(n_kv_heads):
            u = b * n_kv_heads + h
            lo, hi = int(out_offsets[u]), int(out_offsets[u + 1])
            if hi == lo:
                continue
            for g in range(G):
                out[b, :, h * G + g, :] = attention_output(q_new[b, :, h * G + g, :], k_c[lo:hi], v_c[lo:hi], scale)
    return out


def oracle_masked_attention(q_new, k, v, cu_seqlens, keep_mask, n_q_heads, n_kv_heads, scale=None):
    """The same attention over the uncompressed cache with the evicted positions masked to
    -inf: k, v [N, Hkv, d] packed, keep_mask [Hkv, N] bool.  By the permutation invariance of
    attention it equals oracle_decode_attention on the compacted rows."""
    q_new = np.asarray(q_new, np.float64)
    B, n_new, Hq, d = q_new.shape
    G = n_q_heads // n_kv_heads
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    out = np.zeros((B, n_new, Hq, d))
    for b in range(B):
        s, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        for h in range(n_kv_heads):
            m = np.asarray(keep_mask[h, s:e], bool)
            if not m.any():
                continue
            for g in range(G):
                out[b, :, h * G + g, :] = attention_output(q_new[b, :, h * G + g, :], k[s:e, h], v[s:e, h], scale, m)
    return out


def cut_robustness(scores_unit, rank_mode, n_sink, T, rel=1e-3):
    """Is the oracle's cut far enough from a rounding edge that a correct fp32
    implementation must reproduce it exactly?  Returns (robust, i_star).

    With g(i) = P_i / F^2 and tau = (1 - T)^2 the rule picks the step of g that
    straddles tau.  The unit is robust when tau sits more than `rel` of that
    step's height away from both of its edges and, in score ranking, the scores
    on the two sides of the cut differ by more than `rel` relative.
    """
    n = len(scores_unit)
    rank = rank_positions(scores_unit, rank_mode, n_sink)
    s = np.asarray(scores_unit, np.float64)[rank]
    i_star = budget_cumsum(s, T)
    if n == 0:
        return True, 0
    P = np.cumsum(s * s)
    F2 = P[-1]
    if F2 == 0.0 or T <= 0.0 or T >= 1.0:
        return True, i_star          # keep-all / keep-one limits do not depend on rounding
    tau = (1.0 - T) ** 2
    g_hi = P[i_star - 1] / F2
    g_lo = P[i_star - 2] / F2 if i_star >= 2 else 0.0
    step = g_hi - g_lo
    robust = step > 0 and min(g_hi - tau, tau - g_lo) > rel * step
    if rank_mode == RANK_SCORE and i_star < n:
        robust = robust and abs(s[i_star - 1] - s[i_star]) > rel * abs(s[i_star - 1])
    return bool(robust), i_star
