"""Writes tests/golden/cfg0_oracle.json from the CPU oracle alone.

The paper prints no worked numeric example of its budget rule, so this fixture is
not a paper value: it freezes what the float64 oracle returns on the tiny fp32
configuration so that an accidental change to the oracle or to the input
generator is noticed.  Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import refreekv_oracle as O                     # noqa: E402
from paper_2502_16886_amd import workloads as W             # noqa: E402


def main():
    L = W.make_layer(0, 0)
    c = L.cfg
    scores = O.oracle_score(L.f64("q_win"), L.f64("k"), L.cu_seqlens, c.n_q_heads, c.n_kv_heads, c.window)
    out = {"config": 0, "layer": 0, "threshold": c.threshold, "n_sink": c.n_sink,
           "score_samples": {str(p): [float(scores[h, p]) for h in range(c.n_kv_heads)]
                             for p in (0, 3, 4, 100, 255, 496, 497, 510, 511)},
           "score_row_sums": [float(scores[h].sum()) for h in range(c.n_kv_heads)]}
    for mode, name in ((O.RANK_POSITION, "position"), (O.RANK_SCORE, "score")):
        kept, offs, idx = O.oracle_select(scores, L.cu_seqlens, mode, c.n_sink, c.threshold)
        out[name] = {"kept": [int(x) for x in kept],
                     "idx_checksum": [int(np.sum(idx[offs[u]:offs[u + 1]] * (np.arange(kept[u]) + 1)))
                                      for u in range(len(kept))]}
    with open(os.path.join(os.path.dirname(__file__), "cfg0_oracle.json"), "w") as f:
        json.dump(out, f, indent=1)
    print(json.dumps(out)[:300])


if __name__ == "__main__":
    main()
