"""Pins of the oracle's decode attention (new queries over the compacted ragged cache, and the
masked form over the full cache).  None of them re-types the oracle's formula: they compare it
with a library attention routine, with closed forms, and with itself across the two forms."""
import numpy as np
import pytest
import torch

from oracle import refreekv_oracle as O
from paper_2502_16886_amd import workloads as W


def _random_case(seed, B=2, n_new=5, Hq=4, Hkv=2, d=16, lens=(37, 12)):
    rng = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    N = int(cu[-1])
    q = rng.standard_normal((B, n_new, Hq, d))
    k = rng.standard_normal((N, Hkv, d))
    v = rng.standard_normal((N, Hkv, d))
    return q, k, v, cu


def _compact(k, v, cu, keep):
    """Rows of the retained positions, unit-major (b, h), ascending position."""
    Hkv = k.shape[1]
    ks, vs, offs = [], [], [0]
    for b in range(len(cu) - 1):
        for h in range(Hkv):
            pos = np.nonzero(keep[h, cu[b]:cu[b + 1]])[0] + cu[b]
            ks.append(k[pos, h])
            vs.append(v[pos, h])
            offs.append(offs[-1] + len(pos))
    return np.concatenate(ks), np.concatenate(vs), np.asarray(offs, np.int64)


def test_full_cache_equals_library_sdpa():
    """Nothing evicted: every (sequence, query head) is plain scaled-dot-product attention
    (torch's CPU routine in float64) of the new queries over the sequence's keys of the KV head."""
    q, k, v, cu = _random_case(1)
    B, n_new, Hq, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    keep = np.ones((Hkv, k.shape[0]), bool)
    k_c, v_c, offs = _compact(k, v, cu, keep)
    got = O.oracle_decode_attention(q, k_c, v_c, offs, Hq, Hkv)
    for b in range(B):
        kk = torch.from_numpy(k[cu[b]:cu[b + 1]]).permute(1, 0, 2)       # [Hkv, n, d]
        vv = torch.from_numpy(v[cu[b]:cu[b + 1]]).permute(1, 0, 2)
        qq = torch.from_numpy(q[b]).permute(1, 0, 2)                       # [Hq, n_new, d]
        ref = torch.nn.functional.scaled_dot_product_attention(
            qq, kk.repeat_interleave(G, dim=0), vv.repeat_interleave(G, dim=0))
        np.testing.assert_allclose(got[b], ref.permute(1, 0, 2).numpy(), rtol=1e-12, atol=1e-13)


def test_compacted_equals_masked_full():
    """Random retained sets: attention over the gathered rows == masked attention over all rows."""
    q, k, v, cu = _random_case(2)
    Hq, Hkv = q.shape[2], k.shape[1]
    rng = np.random.default_rng(3)
    keep = rng.random((Hkv, k.shape[0])) < 0.4
    keep[:, cu[:-1]] = True                                  # no unit is empty
    k_c, v_c, offs = _compact(k, v, cu, keep)
    a = O.oracle_decode_attention(q, k_c, v_c, offs, Hq, Hkv, scale=0.3)
    b = O.oracle_masked_attention(q, k, v, cu, keep, Hq, Hkv, scale=0.3)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)


def test_single_key_returns_its_value_row():
    q, k, v, cu = _random_case(4)
    Hq, Hkv = q.shape[2], k.shape[1]
    G = Hq // Hkv
    keep = np.zeros((Hkv, k.shape[0]), bool)
    chosen = {}
    for b in range(len(cu) - 1):
        for h in range(Hkv):
            p = int(cu[b]) + (3 * b + 5 * h) % int(cu[b + 1] - cu[b])
            keep[h, p] = True
            chosen[(b, h)] = p
    k_c, v_c, offs = _compact(k, v, cu, keep)
    out = O.oracle_decode_attention(q, k_c, v_c, offs, Hq, Hkv)
    for (b, h), p in chosen.items():
        for g in range(G):
            np.testing.assert_allclose(out[b, :, h * G + g], np.broadcast_to(v[p, h], out[b, :, 0].shape), rtol=1e-13)


def test_equal_keys_average_the_values():
    """All keys equal: uniform weights whatever the query, so the output is the mean value row."""
    q, k, v, cu = _random_case(5)
    Hq, Hkv = q.shape[2], k.shape[1]
    k[:] = k[0:1, 0:1]
    keep = np.ones((Hkv, k.shape[0]), bool)
    k_c, v_c, offs = _compact(k, v, cu, keep)
    out = O.oracle_decode_attention(q, k_c, v_c, offs, Hq, Hkv)
    G = Hq // Hkv
    for b in range(len(cu) - 1):
        for hq in range(Hq):
            mean = v[cu[b]:cu[b + 1], hq // G].mean(axis=0)
            np.testing.assert_allclose(out[b, :, hq], np.broadcast_to(mean, out[b, :, hq].shape), rtol=1e-12, atol=1e-14)


def test_planted_mistakes_are_caught():
    """A transposed head mapping or a forgotten scale changes the result (the pins above would
    notice): guard against the comparison being insensitive."""
    q, k, v, cu = _random_case(6)
    Hq, Hkv = q.shape[2], k.shape[1]
    keep = np.ones((Hkv, k.shape[0]), bool)
    k_c, v_c, offs = _compact(k, v, cu, keep)
    good = O.oracle_decode_attention(q, k_c, v_c, offs, Hq, Hkv)
    no_scale = O.oracle_decode_attention(q, k_c, v_c, offs, Hq, Hkv, scale=1.0)
    swapped = O.oracle_decode_attention(q[:, :, ::-1], k_c, v_c, offs, Hq, Hkv)
    assert np.abs(good - no_scale).max() > 1e-3
    assert np.abs(good - swapped).max() > 1e-3


def test_empty_unit_gives_zeros():
    q, k, v, cu = _random_case(7)
    Hq, Hkv = q.shape[2], k.shape[1]
    keep = np.ones((Hkv, k.shape[0]), bool)
    keep[1, cu[1]:cu[2]] = False                              # unit (b=1, h=1) keeps nothing
    k_c, v_c, offs = _compact(k, v, cu, keep)
    out = O.oracle_decode_attention(q, k_c, v_c, offs, Hq, Hkv)
    G = Hq // Hkv
    assert np.all(out[1, :, G:2 * G] == 0)
    assert np.abs(out[1, :, 0:G]).max() > 0


def test_new_queries_generator_is_deterministic_and_typed():
    a = W.make_new_queries(1, 3, n_new=8)
    b = W.make_new_queries(1, 3, n_new=8)
    assert a.dtype == np.uint16 and a.shape == (1, 8, 32, 128) and np.array_equal(a, b)
    c = W.make_new_queries(0, 0, n_new=4)
    assert c.dtype == np.float32 and c.shape == (1, 4, 8, 64)
    assert not np.array_equal(a, W.make_new_queries(1, 4, n_new=8))
