"""GPU parity at a size where 32-bit element offsets no longer reach: one layer whose K (and V) holds
more than 2^31 elements (2.2 M tokens x 8 KV heads x 128, bf16, 4.5 GB each), a second short sequence
behind it so that a sequence start lies beyond 2^31 elements too.  The inputs are made on the GPU by
torch's seeded generator (a generator outside both paths) and the very same bits are downloaded for
the oracle.  Checked: one KV head's scores of the long sequence and the whole short sequence against
the float64 oracle, Eq. 2's mass identity on every head, the selection stage-exact on every unit (both
rankings), the compacted rows bit for bit (gathered again with torch indexing on the device), and decode
attention over that compacted cache for three units against the oracle."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import rfkv_harness as H                                   # noqa: E402
from oracle import refreekv_oracle as O                    # noqa: E402
from paper_2502_16886_amd import binding as B              # noqa: E402

pytestmark = pytest.mark.gpu

LENS = (2_200_017, 1000)
HQ, HKV, D, WIN, M, T = 32, 8, 128, 32, 4, 0.01


def bf16_to_f64(t):
    import torch
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("mode", [B.RANK_POSITION, B.RANK_SCORE])
def test_more_than_2g_elements(mode):
    import torch
    G = HQ // HKV
    cu = np.concatenate([[0], np.cumsum(LENS)]).astype(np.int32)
    N = int(cu[-1])
    assert N * HKV * D > 2 ** 31
    gen = torch.Generator(device="cuda").manual_seed(20250216)
    k = torch.randn((N, HKV, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((N, HKV, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    shared = torch.randn((1, HKV, 1, D), generator=gen, device="cuda")
    q = (0.6 * torch.randn((2 * WIN, HKV, G, D), generator=gen, device="cuda") + shared).reshape(2 * WIN, HQ, D)
    q = q.to(torch.bfloat16).contiguous()
    for b in range(2):                                     # sinks: the first keys point along the shared query part
        s0 = int(cu[b])
        k[s0:s0 + M] = (2.5 * shared[0, :, 0, :]).to(torch.bfloat16)
    cu_dev = torch.from_numpy(cu).cuda()

    p = B.make_params(2, HQ, HKV, D, WIN, "bf16", n_sink=M, threshold=T, rank_mode=mode)
    buf = B.alloc_layer_buffers(p, N, max(LENS))
    print(f"\n  N={N} mode={mode}: launching", flush=True)
    B.rfkv_compress_layer(p, q, k, v, cu, cu_dev, buf.scores, buf.kept, buf.out_offsets, buf.idx, buf.k_out,
                          buf.v_out, buf.capacity_rows, buf.ws, buf.ws_bytes, None)
    torch.cuda.synchronize()
    print("  done; checking", flush=True)
    scores = buf.scores.cpu().numpy()
    kept = buf.kept.cpu().numpy().astype(np.int64)
    offs = buf.out_offsets.cpu().numpy()
    idx = buf.idx[:int(offs[-1])].cpu().numpy().astype(np.int64)

    # scores: KV head 5 of the long sequence and every head of the short one, against the oracle
    h = 5
    ref = O.oracle_score(bf16_to_f64(q[:WIN, h * G:(h + 1) * G]), bf16_to_f64(k[:LENS[0], h:h + 1]),
                         np.array([0, LENS[0]]), G, 1, WIN)[0]
    got = scores[h, :LENS[0]].astype(np.float64)
    assert np.all(np.abs(got - ref) <= H.SCORE_RTOL * ref + 1e-300), float(np.max(np.abs(got - ref) / ref))
    ref2 = O.oracle_score(bf16_to_f64(q[WIN:]), bf16_to_f64(k[LENS[0]:]), np.array([0, LENS[1]]), HQ, HKV, WIN)
    got2 = scores[:, LENS[0]:].astype(np.float64)
    assert np.all(np.abs(got2 - ref2) <= H.SCORE_RTOL * ref2 + 1e-300)
    # Eq. 2: every window row is a distribution, so sum_i cnt_i A'[i] = w' on every head (cnt_i = rows that see i)
    for b, n in enumerate(LENS):
        cnt = np.minimum(WIN, n - np.arange(n)).astype(np.float64)
        mass = (scores[:, cu[b]:cu[b + 1]].astype(np.float64) * cnt).sum(axis=1)
        assert np.allclose(mass, min(WIN, n), rtol=1e-4), mass

    # selection, stage-exact on the GPU's own scores: counts, offsets and index lists of all 16 units
    kept_o, offs_o, idx_o = O.oracle_select(scores.astype(np.float64), cu, mode, M, H.threshold_as_float32(T), 0,
                                            form="cumsum")
    assert np.array_equal(kept, kept_o) and np.array_equal(offs, offs_o) and np.array_equal(idx, idx_o)
    assert 0 < kept.min() and kept[:HKV].max() <= LENS[0]

    # the consumer over the same cache: 8 new queries, one KV head of the long sequence and the short
    # sequence against the oracle (rows of the compacted cache beyond 2^31 elements)
    if mode == B.RANK_POSITION:
        n_new = 8
        qn = (0.6 * torch.randn((2, n_new, HKV, G, D), generator=gen, device="cuda") + shared[None, 0]).reshape(
            2, n_new, HQ, D).to(torch.bfloat16).contiguous()
        out = torch.full((2, n_new, HQ, D), float("nan"), dtype=torch.float32, device="cuda")
        dws_bytes = B.rfkv_decode_workspace_bytes(p, n_new, max(LENS))
        dws = torch.empty(dws_bytes, dtype=torch.uint8, device="cuda")
        B.rfkv_decode_attention(p, qn, n_new, buf.k_out, buf.v_out, cu, buf.out_offsets, None, out, dws, dws_bytes)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        for u in (h, HKV + 2, 2 * HKV - 1):                  # units of both sequences; the last one ends the cache
            b, hh = divmod(u, HKV)
            o0, o1 = int(offs[u]), int(offs[u + 1])
            k_u, v_u = bf16_to_f64(buf.k_out[o0:o1]), bf16_to_f64(buf.v_out[o0:o1])
            q_u = bf16_to_f64(qn[b:b + 1, :, hh * G:(hh + 1) * G])
            ref_o = O.oracle_decode_attention(q_u, k_u, v_u, np.array([0, o1 - o0]), G, 1)
            bound = 2.0 ** -8 * O.oracle_decode_attention(q_u, k_u, np.abs(v_u), np.array([0, o1 - o0]), G, 1)
            err = np.abs(got[b:b + 1, :, hh * G:(hh + 1) * G] - ref_o)
            assert np.all(err <= 1.05 * bound + 1e-5), (u, float(err.max()))

    # compaction: the rows at those positions, bit for bit (gathered again by torch on the device)
    idx_dev = torch.from_numpy(idx).cuda()
    for u in range(2 * HKV):
        b, hh = divmod(u, HKV)
        o0, o1 = int(offs[u]), int(offs[u + 1])
        for src, out in ((k, buf.k_out), (v, buf.v_out)):
            for c0 in range(o0, o1, 1 << 20):
                c1 = min(o1, c0 + (1 << 20))
                rows = src[:, hh][idx_dev[c0:c1] + int(cu[b])]
                assert torch.equal(rows.view(torch.int16), out[c0:c1].view(torch.int16)), (u, c0)
