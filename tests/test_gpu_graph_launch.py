"""GPU parity in the launch configuration the benchmark times: the headline workload at full size,
several layers' calls captured into ONE HIP graph that forks over four streams (all at the default
priority), replayed several times with eager work and synchronisations in between.  Every replay
must reproduce the eager calls bit for bit, and one layer is checked against the float64 oracle."""
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
LAYERS, STREAMS = 4, 4
KEYS = ("scores", "kept", "out_offsets", "idx", "k_out", "v_out")


def clear_outputs(dl):
    b = dl.buf
    for t in (b.scores, b.kept, b.out_offsets, b.idx, b.k_out, b.v_out):
        t.zero_()                                          # a fill kernel, not a memset node


@pytest.mark.parametrize("mode,with_lse", [(B.RANK_POSITION, False), (B.RANK_SCORE, False), (B.RANK_POSITION, True)])
def test_graph_over_four_streams_replays_the_eager_results(mode, with_lse):
    import torch
    cfg = W.CONFIGS["H"]
    host = [W.make_layer("H", li) for li in range(LAYERS)]
    dls = [H.DeviceLayer(l, rank_mode=mode, kv_layout="head_major") for l in host]
    lse = [None] * LAYERS
    if with_lse:
        for i, l in enumerate(host):
            ref = O.oracle_window_lse(l.f64("q_win"), l.f64("k"), l.cu_seqlens, cfg.n_q_heads, cfg.n_kv_heads, cfg.window)
            lse[i] = torch.from_numpy(np.ascontiguousarray(ref, dtype=np.float32)).cuda()

    eager = []
    for dl, x in zip(dls, lse):
        dl.compress(None, lse_win=x)
        eager.append(dl.results())
    # the eager result of one layer against the oracle (retained sets, compacted rows, scores)
    if with_lse:
        ref_scores = O.oracle_score_lse(host[1].f64("q_win"), lse[1].cpu().numpy().astype(np.float64), host[1].f64("k"),
                                        host[1].cu_seqlens, cfg.n_q_heads, cfg.n_kv_heads, cfg.window)
    else:
        ref_scores = O.oracle_score(host[1].f64("q_win"), host[1].f64("k"), host[1].cu_seqlens, cfg.n_q_heads,
                                    cfg.n_kv_heads, cfg.window)
    rep = H.compare_layer(host[1], eager[1], mode, ref=H.oracle_layer(host[1], mode, scores=ref_scores))
    print(f"\n  eager layer 1, mode={mode}, lse={with_lse}: {rep}", flush=True)

    side = [torch.cuda.Stream() for _ in range(STREAMS)]   # default priority

    def all_layers():
        cur = torch.cuda.current_stream()
        for st in side:
            st.wait_stream(cur)
        for j, (dl, x) in enumerate(zip(dls, lse)):
            with torch.cuda.stream(side[j % STREAMS]):
                dl.compress(None, lse_win=x)
        for st in side:
            cur.wait_stream(st)

    all_layers()                                           # the streams exist and are warm before capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=None):
        all_layers()
    torch.cuda.synchronize()

    for replay in range(3):
        for dl in dls:
            clear_outputs(dl)
        torch.cuda.synchronize()
        graph.replay()
        for j, dl in enumerate(dls):
            got = dl.results()                             # synchronises
            for key in KEYS:
                assert np.array_equal(got[key], eager[j][key]), (replay, j, key)
        # eager work of the program between replays: another call outside the graph, then a sync
        dls[replay % LAYERS].compress(None, lse_win=lse[replay % LAYERS])
        torch.cuda.synchronize()
