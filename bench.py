#!/usr/bin/env python3
"""Benchmark of the ReFreeKV compression pass on one MI355X.

A step is one rfkv_compress_layer call (score -> rank -> budget rule -> gather-compact) over one
transformer layer of the headline workload: Llama3-8B attention shape (32 query / 8 KV heads,
d = 128, bf16), one 32768-token sequence, observation window 32, T = 1 %, m = 4, position ranking
(the paper's method).  Steps rotate over several layers' distinct buffers so that no step finds
its inputs in the 256 MB Infinity Cache left there by the previous one.  Inputs are synthetic
(paper_2502_16886_amd.workloads) and resident in HBM before timing starts.

Timing: the steps are captured into one HIP graph over all layer buffers (forked over a few streams,
layers are independent) and the graph is replayed at least five times; every replay is bracketed by
HIP events, `ms_per_step` is the median replay divided by the steps in it, and the spread is
reported.  `--steps K` asks for K steps; the run rounds up to whole replays and says what it ran.

Prints one JSON line: throughput, the roofline figures of the whole pass and of its dominant kernel,
the CPU oracle timed on the same workload, and legs for the score ranking, a single stream, the
prefill's log-sum-exp hand-over, all layers in one call, the other workload configurations, the
decode attention over the compacted cache and the ablation's wide window.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E bandwidth
MIN_REPLAYS = 5


def algorithmic_bytes(N, Hkv, d, e, Hq, wrows, kept_rows, units, score_mode):
    """Bytes the method itself must move for one layer-pass (K counted once)."""
    k_read = N * Hkv * d * e
    q_read = wrows * Hq * d * e
    scores = 2 * N * Hkv * 4
    gather = 4 * kept_rows * d * e
    idx = kept_rows * 8 if score_mode else 0
    return k_read + q_read + scores + gather + idx + 12 * units


def kernel_bytes(name, N, Hkv, d, e, Hq, wrows, kept_rows):
    """Algorithmic bytes of one kernel launch."""
    if name == "score_stats":
        return N * Hkv * d * e + wrows * Hq * d * e
    if name == "score_reduce":
        return N * Hkv * d * e + wrows * Hq * d * e + N * Hkv * 4
    if name == "select":
        return N * Hkv * 4
    if name == "compact":
        return 4 * kept_rows * d * e
    return 0


def read_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` measured offline with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (scaled by a plain copy of known size); the summary lives in profiles/.  None if there is no
    summary for this kernel and workload."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{kernel}_{workload}.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for ln in open(path):
        if "=" in ln and not ln.lstrip().startswith("#"):
            k, v = ln.split("=", 1)
            try:
                vals[k.strip()] = float(v.split()[0])
            except ValueError:
                pass
    if "fetch_bytes_per_launch" in vals and "write_bytes_per_launch" in vals:
        return {"fetch_bytes": int(vals["fetch_bytes_per_launch"]), "write_bytes": int(vals["write_bytes_per_launch"]),
                "total_bytes": int(vals["fetch_bytes_per_launch"] + vals["write_bytes_per_launch"]),
                "source": os.path.relpath(path, ROOT)}
    return None


class Stepper:
    """`layers` device buffers of one workload and the means to run steps over them: eagerly, on one
    or several streams, or as replays of one HIP graph that holds one step per buffer."""

    def __init__(self, torch, objs, streams):
        self.torch = torch
        self.objs = objs                                   # things with .compress(stream)
        self.side = [torch.cuda.Stream() for _ in range(streams)] if streams > 1 else []

    def run_steps(self, count, start=0):
        torch, n = self.torch, len(self.objs)
        if not self.side:
            for i in range(count):
                self.objs[(start + i) % n].compress(None)          # torch's current stream
            return
        # layer j always uses stream j % S, hence two uses of one layer's buffers stay ordered
        cur = torch.cuda.current_stream()
        for st in self.side:
            st.wait_stream(cur)
        for i in range(count):
            j = (start + i) % n
            with torch.cuda.stream(self.side[j % len(self.side)]):
                self.objs[j].compress(None)
        for st in self.side:
            cur.wait_stream(st)

    def timed(self, steps, warmup, graph=True, min_replays=MIN_REPLAYS):
        """Per-step milliseconds: median, min and max over replays, steps run, replays, wall ms per step."""
        import numpy as np
        torch, n = self.torch, len(self.objs)
        self.run_steps(max(warmup, 1))
        torch.cuda.synchronize()
        g = None
        if graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=None):
                self.run_steps(n)
            torch.cuda.synchronize()
        replays = max(min_replays, (steps + n - 1) // n)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(replays + 1)]
        torch.cuda.synchronize()
        t = time.perf_counter()
        marks[0].record()
        for r in range(replays):
            if g is not None:
                g.replay()
            else:
                self.run_steps(n)
            marks[r + 1].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t) * 1e3 / (replays * n)
        per = np.array([marks[r].elapsed_time(marks[r + 1]) for r in range(replays)]) / n
        return dict(ms=float(np.median(per)), ms_min=float(per.min()), ms_max=float(per.max()), steps=replays * n,
                    replays=replays, wall_ms=wall)


def kernel_times(np, B, dls, reps):
    """Per-kernel durations from HIP events recorded on the launch stream between the kernels
    (rfkv_compress_layer_timed; serial, one call at a time)."""
    kms = np.zeros(len(B.KERNEL_NAMES))
    for i in range(reps):
        dl = dls[i % len(dls)]
        b = dl.buf
        _, ms = B.rfkv_compress_layer_timed(dl.params, dl.q, dl.k, dl.v, dl.cu_host, dl.cu_dev, b.scores, b.kept,
                                            b.out_offsets, b.idx, b.k_out, b.v_out, b.capacity_rows, b.ws, b.ws_bytes,
                                            None)
        kms += np.array(ms)
    return dict(zip(B.KERNEL_NAMES, (kms / reps).tolist()))


def with_score_mode(H, B, dl):
    """The same inputs and output buffers as `dl`, ranked by score."""
    d2 = H.DeviceLayer.__new__(H.DeviceLayer)
    d2.__dict__.update(dl.__dict__)
    d2.params = B.RfkvParams.from_buffer_copy(dl.params)
    d2.params.rank_mode = B.RANK_SCORE
    return d2


def time_decode_attention(torch, np, H, B, W, cfg_id=4, n_new=64, reps=20):
    """Consumer of the compressed cache: attention of `n_new` new queries over the compacted ragged
    cache of one layer of config 4 (131072 tokens), next to masked attention over the full cache."""
    layer = W.make_layer(cfg_id, 0)
    cfg = layer.cfg
    qn = W.make_new_queries(cfg_id, 0, n_new=n_new)
    dl = H.DeviceLayer(layer, kv_layout="head_major")
    dl.compress()
    res = dl.results()
    N, Hkv, d = dl.N, cfg.n_kv_heads, cfg.head_dim
    kept_rows = int(res["out_offsets"][-1])
    keep = np.zeros((Hkv, N), np.uint8)
    for u, b, h, s0, e0 in H.unit_slices(layer):
        o, c = int(res["out_offsets"][u]), int(res["kept"][u])
        keep[h, s0 + res["idx"][o:o + c]] = 1
    mask = torch.from_numpy(keep).cuda()
    q = H.to_device(qn, cfg.dtype)
    out = torch.empty((dl.batch, n_new, cfg.n_q_heads, d), dtype=torch.float32, device="cuda")
    ws_bytes = B.rfkv_decode_workspace_bytes(dl.params, n_new, dl.max_len)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    b = dl.buf
    t_c = timed(lambda: B.rfkv_decode_attention(dl.params, q, n_new, b.k_out, b.v_out, dl.cu_host, b.out_offsets, None,
                                                out, ws, ws_bytes))
    t_m = timed(lambda: B.rfkv_masked_attention(dl.params, q, n_new, dl.k, dl.v, dl.cu_host, dl.cu_dev, mask, out, ws,
                                                ws_bytes))
    flop_per_key = 4 * n_new * (cfg.n_q_heads // Hkv) * d          # QK^T and PV, multiply-add = 2
    tf = flop_per_key * kept_rows / (t_c * 1e-3) / 1e12
    return {"workload": f"{cfg.name}: {N} tokens, {n_new} new queries, position ranking, T={cfg.threshold}",
            "retained_fraction": round(kept_rows / (N * Hkv), 4),
            "compacted_ms": round(t_c, 5), "masked_full_ms": round(t_m, 5), "speedup": round(t_m / t_c, 3),
            "compacted_kv_GBps": round(2 * kept_rows * d * 2 / (t_c * 1e-3) / 1e9, 1),
            "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": 2500.0, "unit": "TFLOP/s",
                         "frac": round(tf / 2500.0, 4), "traffic": None},
            "masked_mfma_TFLOPs": round(flop_per_key * N * Hkv / (t_m * 1e-3) / 1e12, 1)}


def time_wide_window(np, H, B, W, window=328, reps=12):
    """The ablation's large window (k = 1 % of n) on the headline shape: the window contraction is a
    real GEMM, so the kernels are priced against the dense bf16 MFMA peak (2 passes over Q_win K^T)."""
    base = W.CONFIGS["H"]
    cfg = W.Config(f"{base.name}-w{window}", base.layers, base.n_q_heads, base.n_kv_heads, base.head_dim, window,
                   base.dtype, batch=1, context=base.context)
    layer = W.make_layer("H", 0, cfg=cfg)
    dl = H.DeviceLayer(layer, kv_layout="head_major")
    for _ in range(2):
        dl.compress()
    k = kernel_times(np, B, [dl], reps)
    n, G, d, Hkv = cfg.context, cfg.n_q_heads // cfg.n_kv_heads, cfg.head_dim, cfg.n_kv_heads
    # logits a pass has to form: row t of the window sees n - w + t + 1 keys
    visible = sum(n - window + t + 1 for t in range(window)) * G * Hkv
    flop = 2.0 * visible * d
    peak = 2500.0
    return {"workload": f"{cfg.name}: {n} tokens, window {window} ({window * G} score rows per KV head), position ranking",
            "ms_per_step": round(float(sum(k.values())), 5), "kernel_ms": {a: round(v, 5) for a, v in k.items()},
            "flop_per_pass": flop,
            "roofline": {"bound": "mfma", "kernel": "score_reduce", "achieved": round(flop / (k["score_reduce"] * 1e-3) / 1e12, 1),
                         "peak": peak, "unit": "TFLOP/s",
                         "frac": round(flop / (k["score_reduce"] * 1e-3) / 1e12 / peak, 4), "traffic": None},
            "stats_TFLOPs": round(flop / (k["score_stats"] * 1e-3) / 1e12, 1)}


def time_all_layers(torch, np, H, B, W, host_layers, cfg, n_layers=30, replays=MIN_REPLAYS):
    """The post-prefill pass over the whole model in ONE rfkv_compress_layers call on one stream:
    `n_layers` layers (the paper keeps the first two of 32 whole, Sec. 3.3 "Retaining Bottom Layers"),
    each with its own cache and outputs; the library runs the layers' passes side by side.  The
    generated layers repeat to fill the 30."""
    if len(host_layers[0].cu_seqlens) < 2:
        return None
    dls = [H.DeviceLayer(host_layers[i % len(host_layers)], kv_layout="head_major") for i in range(n_layers)]
    ls = H.LayerSet(dls)
    for _ in range(2):
        ls.compress(with_scores=False, with_idx=False)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(replays + 1)]
    marks[0].record()
    for r in range(replays):
        ls.compress(with_scores=False, with_idx=False)
        marks[r + 1].record()
    torch.cuda.synchronize()
    per = np.array([marks[r].elapsed_time(marks[r + 1]) for r in range(replays)])
    ms = float(np.median(per))
    kept = float(np.mean([int(d.buf.out_offsets[-1]) for d in dls]))
    n = dls[0].N
    e = 2 if cfg.dtype == "bf16" else 4
    wrows = int(np.minimum(cfg.window, np.diff(host_layers[0].cu_seqlens)).sum())
    alg = algorithmic_bytes(n, cfg.n_kv_heads, cfg.head_dim, e, cfg.n_q_heads, wrows, kept, dls[0].batch * cfg.n_kv_heads, False)
    del ls, dls
    torch.cuda.empty_cache()
    as_batch = time_layers_as_batch(torch, np, H, W, host_layers, cfg, n_layers, replays, alg)
    return {"entry_point": "rfkv_compress_layers", "layers_per_call": n_layers, "streams": 1, "as_batch": as_batch,
            "retained_fraction": round(kept / (n * cfg.n_kv_heads), 4),
            "ms_per_call": round(ms, 4), "ms_per_layer": round(ms / n_layers, 5),
            "ms_per_layer_min_max": [round(float(per.min()) / n_layers, 5), round(float(per.max()) / n_layers, 5)],
            "tokens_per_s_per_layer_pass": round(n / (ms / n_layers * 1e-3), 1),
            "frac": round(alg / (ms / n_layers * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}


def time_layers_as_batch(torch, np, H, W, host_layers, cfg, n_layers, replays, alg_per_layer):
    """The same layers once more, as a batch: a layer is to rfkv_compress_layer what a sequence is, so caches
    that sit in one allocation ([layer, token, head, d]) are compressed by ONE call of the per-layer entry
    point with one launch of each kernel over all layers (no ramp, launch gap or tail per layer)."""
    src = [host_layers[i % len(host_layers)] for i in range(n_layers)]
    n = int(src[0].cu_seqlens[-1])
    cat = W.Layer(cfg=cfg, q_win=np.concatenate([l.q_win for l in src]), k=np.concatenate([l.k for l in src]),
                  v=np.concatenate([l.v for l in src]),
                  cu_seqlens=np.concatenate([[0], np.cumsum(np.concatenate([np.diff(l.cu_seqlens) for l in src]))]).astype(np.int32))
    dl = H.DeviceLayer(cat, kv_layout="token_major")       # [layer * token, head, d]
    del cat
    for _ in range(2):
        dl.compress()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(replays + 1)]
    marks[0].record()
    for r in range(replays):
        dl.compress()
        marks[r + 1].record()
    torch.cuda.synchronize()
    per = np.array([marks[r].elapsed_time(marks[r + 1]) for r in range(replays)]) / n_layers
    ms = float(np.median(per))
    out = {"entry_point": "rfkv_compress_layer, the layers as a batch of sequences in one allocation", "streams": 1,
           "ms_per_layer": round(ms, 5), "ms_per_layer_min_max": [round(float(per.min()), 5), round(float(per.max()), 5)],
           "tokens_per_s_per_layer_pass": round(n / (ms * 1e-3), 1),
           "frac": round(alg_per_layer / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    del dl
    torch.cuda.empty_cache()
    return out


def time_config(torch, np, H, B, W, cfg_id, streams, buffers=8, gen=2):
    """One of the other workload configurations, a few replays: position and score ranking."""
    cfg = W.CONFIGS[cfg_id]
    host = [W.make_layer(cfg_id, li) for li in range(gen)]
    dls = [H.DeviceLayer(host[i % gen], kv_layout="head_major") for i in range(buffers)]
    N = dls[0].N
    e = 2 if cfg.dtype == "bf16" else 4
    wrows = int(np.minimum(cfg.window, np.diff(host[0].cu_seqlens)).sum())
    units = dls[0].batch * cfg.n_kv_heads
    out = {"workload": f"{cfg.name}: {cfg.n_q_heads}q/{cfg.n_kv_heads}kv heads, d={cfg.head_dim}, batch {dls[0].batch}, "
                       f"{N} tokens, window {cfg.window}, {cfg.dtype}", "tokens": N}
    for name, objs, score_mode in (("position", dls, False), ("score", [with_score_mode(H, B, d) for d in dls], True)):
        r = Stepper(torch, objs, streams).timed(buffers, 2)
        kept = float(np.mean([int(d.buf.out_offsets[-1]) for d in dls]))
        alg = algorithmic_bytes(N, cfg.n_kv_heads, cfg.head_dim, e, cfg.n_q_heads, wrows, kept, units, score_mode)
        out[name] = {"ms_per_step": round(r["ms"], 5), "ms_min_max": [round(r["ms_min"], 5), round(r["ms_max"], 5)],
                     "tokens_per_s": round(N / (r["ms"] * 1e-3), 1), "retained_fraction": round(kept / (N * cfg.n_kv_heads), 4),
                     "frac": round(alg / (r["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    del dls
    torch.cuda.empty_cache()
    return out


def oracle_seconds(np, O, H, layer, threads=None):
    """Best of a few oracle layer-passes (inputs already upcast), optionally with the numerical
    libraries limited to `threads` threads."""
    c = layer.cfg
    q, k = layer.f64("q_win"), layer.f64("k")

    def once():
        t = time.perf_counter()
        O.oracle_compress_layer(q, k, layer.k, layer.v, layer.cu_seqlens, c.n_q_heads, c.n_kv_heads, c.window,
                                n_sink=c.n_sink, T=H.threshold_as_float32(c.threshold), rank_mode=O.RANK_POSITION,
                                form="cumsum")
        return time.perf_counter() - t

    def best():
        return min(once() for _ in range(3))
    if threads is None:
        return best()
    try:
        from threadpoolctl import threadpool_limits
    except Exception:
        return None
    with threadpool_limits(limits=threads):
        return best()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--layers", type=int, default=40, help="distinct layer buffers to rotate over (one graph holds them all)")
    ap.add_argument("--gen-layers", type=int, default=8, help="layers generated on the host (the buffers repeat them)")
    ap.add_argument("--config", default="H", help="workload id in paper_2502_16886_amd.workloads.CONFIGS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kv-layout", default="head_major", choices=["head_major", "token_major"],
                    help="storage of K/V: [Hkv, N, d] (the [B, H, n, d] cache of the paper's setting) or [N, Hkv, d]")
    ap.add_argument("--modes", default="both", choices=["both", "position"],
                    help="also time score ranking (both) or only the paper's position ranking")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 128 MiB device copy a few times (a kernel of known traffic, for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--decode", type=int, default=1,
                    help="also time the decode attention of 64 new queries over the compacted cache of the "
                         "long-context workload (config 4) against masked attention over the full cache (0 = skip)")
    ap.add_argument("--prefill-lse", type=int, default=1,
                    help="also time the pass when the prefill hands over the window rows' log-sum-exp (0 = skip)")
    ap.add_argument("--all-layers", type=int, default=30,
                    help="also time this many layers compressed by one rfkv_compress_layers call (0 = skip)")
    ap.add_argument("--wide", type=int, default=1,
                    help="also time the ablation's wide window (k = 1 %% of n) on the headline shape (0 = skip)")
    ap.add_argument("--configs", default="0,1,2,3,4,K1",
                    help="other workload configurations to time briefly, comma separated ('' = none)")
    ap.add_argument("--streams", type=int, default=4,
                    help="HIP streams the steps are spread over (layers are independent; step i runs on stream i %% S)")
    ap.add_argument("--graph", type=int, default=1, help="replay the timed steps from a HIP graph (1) or launch eagerly (0)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU (the units of a layer are independent and would shard by "
              "KV head, sequence or layer without communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2502_16886_amd import device as H
    from paper_2502_16886_amd import binding as B
    from paper_2502_16886_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.load_library()
    cfg_id = int(args.config) if args.config.isdigit() else args.config
    cfg = W.CONFIGS[cfg_id]
    e = 2 if cfg.dtype == "bf16" else 4

    t0 = time.time()
    # `layers` device buffers to rotate over; at most `gen_layers` of them are generated on the host, the
    # rest are further uploads of the same layers in turn (their own buffers, inputs and outputs)
    host_layers = [W.make_layer(cfg_id, li) for li in range(min(args.layers, args.gen_layers))]
    pos_dls = [H.DeviceLayer(host_layers[i % len(host_layers)], rank_mode=B.RANK_POSITION, kv_layout=args.kv_layout)
               for i in range(args.layers)]
    gen_s = time.time() - t0
    N = pos_dls[0].N
    wrows = int(np.minimum(cfg.window, np.diff(host_layers[0].cu_seqlens)).sum())
    units = pos_dls[0].batch * cfg.n_kv_heads
    shape = (N, cfg.n_kv_heads, cfg.head_dim, e, cfg.n_q_heads, wrows)

    def kept_rows_of(dls):
        return float(np.mean([int(dl.buf.out_offsets[-1]) for dl in dls]))

    # ---- headline: position ranking, graph over all buffers, several streams
    head = Stepper(torch, pos_dls, args.streams)
    try:
        pos = head.timed(args.steps, args.warmup, graph=bool(args.graph))
    except Exception as ex:          # graph capture unavailable: fall back to eager launches
        if not args.graph:
            raise
        print(f"bench.py: graph replay failed ({ex}); timing eager launches", file=sys.stderr)
        args.graph = 0
        pos = head.timed(args.steps, args.warmup, graph=False)
    pos["kernel_ms"] = kernel_times(np, B, pos_dls, max(args.layers, 40))
    pos["kept_rows"] = kept_rows_of(pos_dls)
    ms_per_step = pos["ms"]
    value = N / (ms_per_step * 1e-3)
    alg = algorithmic_bytes(*shape, pos["kept_rows"], units, False)
    dom = max(pos["kernel_ms"], key=pos["kernel_ms"].get)       # dominant kernel = longest average duration
    dom_bytes = kernel_bytes(dom, *shape, pos["kept_rows"])
    dom_gbs = dom_bytes / (pos["kernel_ms"][dom] * 1e-3) / 1e9
    pipe_gbs = alg / (ms_per_step * 1e-3) / 1e9
    roofline = {"bound": "hbm", "scope": "whole pass: algorithmic bytes of a step's kernels / step time",
                "achieved": round(pipe_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(pipe_gbs / HBM_PEAK_GBS, 4), "algorithmic_bytes": int(alg),
                "traffic": read_traffic("step", cfg.name),
                "dominant_kernel": {"kernel": dom, "algorithmic_bytes": int(dom_bytes),
                                    "ms": round(pos["kernel_ms"][dom], 5), "achieved": round(dom_gbs, 1),
                                    "kernel_frac": round(dom_gbs / HBM_PEAK_GBS, 4),
                                    "traffic": read_traffic(dom, cfg.name)},
                "kernel_ms": {k: round(v, 5) for k, v in pos["kernel_ms"].items()}}

    # ---- score ranking on the same inputs
    score_mode = None
    sdls = None
    if args.modes == "both":
        sdls = [with_score_mode(H, B, dl) for dl in pos_dls]
        sco = Stepper(torch, sdls, args.streams).timed(args.layers, 2, graph=bool(args.graph))
        kms = kernel_times(np, B, sdls, args.layers)
        kr = kept_rows_of(sdls)
        alg_s = algorithmic_bytes(*shape, kr, units, True)
        score_mode = {"value": round(N / (sco["ms"] * 1e-3), 1), "ms_per_step": round(sco["ms"], 5),
                      "ms_min_max": [round(sco["ms_min"], 5), round(sco["ms_max"], 5)],
                      "retained_fraction": round(kr / (N * cfg.n_kv_heads), 4),
                      "kernel_ms": {k: round(v, 5) for k, v in kms.items()},
                      "frac": round(alg_s / (sco["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # ---- the same steps on one stream (no overlap between layers): per-layer latency
    single = None
    if args.streams > 1:
        for dl in pos_dls:
            dl.compress()
        s1 = Stepper(torch, pos_dls, 1).timed(args.layers, 2, graph=bool(args.graph))
        single = {"ms_per_step": round(s1["ms"], 5), "ms_min_max": [round(s1["ms_min"], 5), round(s1["ms_max"], 5)],
                  "frac": round(alg / (s1["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # ---- the prefill hands over the window rows' log-sum-exp
    with_lse = None
    lse_objs = None
    if args.prefill_lse:
        # Stand-in for the prefill's attention kernel: the window rows' log-sum-exp, by torch, outside
        # every timed region.  Position ranking on the same inputs and buffers as the headline.
        class WithLse:
            def __init__(self, dl):
                self.dl = dl
                c = dl.layer.cfg
                G = c.n_q_heads // c.n_kv_heads
                scale = 1.0 / float(np.sqrt(c.head_dim))
                parts, q0 = [], 0
                k = dl.k if args.kv_layout == "head_major" else dl.k.permute(1, 0, 2)        # [Hkv, N, d]
                for bb in range(dl.batch):
                    s0, e0 = int(dl.cu_host[bb]), int(dl.cu_host[bb + 1])
                    n, wp = e0 - s0, min(c.window, e0 - s0)
                    q = dl.q[q0:q0 + wp].float().view(wp, c.n_kv_heads, G, c.head_dim)
                    logits = torch.einsum("rhgd,hnd->rhgn", q, k[:, s0:e0].float()) * scale
                    vis = torch.arange(n, device="cuda")[None, :] <= (n - wp + torch.arange(wp, device="cuda"))[:, None]
                    logits = logits.masked_fill(~vis[:, None, None, :], float("-inf"))
                    parts.append(torch.logsumexp(logits, dim=-1).reshape(wp, c.n_q_heads))
                    q0 += wp
                self.lse = torch.cat(parts).contiguous()

            def compress(self, stream):
                return self.dl.compress(stream, lse_win=self.lse)
        lse_objs = [WithLse(dl) for dl in pos_dls]
        r = Stepper(torch, lse_objs, args.streams).timed(args.layers, 2, graph=bool(args.graph))
        kr = kept_rows_of(pos_dls)
        alg_l = algorithmic_bytes(*shape, kr, units, False) + 4 * wrows * cfg.n_q_heads
        r1 = Stepper(torch, lse_objs, 1).timed(args.layers, 2, graph=bool(args.graph)) if args.streams > 1 else None
        with_lse = {"note": "window rows' log-sum-exp supplied by the caller (rfkv_compress_layer_lse): no statistics pass, "
                            "K read once; the lse itself comes from torch outside the timed region",
                    "value": round(N / (r["ms"] * 1e-3), 1), "ms_per_step": round(r["ms"], 5),
                    "ms_min_max": [round(r["ms_min"], 5), round(r["ms_max"], 5)],
                    "retained_fraction": round(kr / (N * cfg.n_kv_heads), 4),
                    "frac": round(alg_l / (r["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                    "single_stream_ms_per_step": round(r1["ms"], 5) if r1 else None}

    # ---- the CPU oracle on the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import refreekv_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        t = time.perf_counter()
        out = None
        passes = 0
        while passes == 0 or (time.perf_counter() - t < 10.0 and passes < 8 * len(host_layers)):
            L = host_layers[passes % len(host_layers)]   # the layers in turn, again from the first until ~10 s are spent
            res = O.oracle_compress_layer(L.f64("q_win"), L.f64("k"), L.k, L.v, L.cu_seqlens, cfg.n_q_heads,
                                          cfg.n_kv_heads, cfg.window, n_sink=cfg.n_sink,
                                          T=H.threshold_as_float32(cfg.threshold), rank_mode=O.RANK_POSITION,
                                          form="cumsum")
            if out is None:
                out = res                                # layer 0's result doubles as a parity check below
            passes += 1
        dt = (time.perf_counter() - t) / passes
        # the run doubles as a last parity check of the benchmarked launch configuration
        dl = pos_dls[0]
        dl.compress(None)
        gpu = dl.results()
        agree = bool(np.array_equal(gpu["kept"], out["kept"]))
        # the small configurations with the numerical libraries held to one thread, and unrestricted
        small = {}
        for cid in (0, 1):
            L = W.make_layer(cid, 0)
            one, many = oracle_seconds(np, O, H, L, threads=1), oracle_seconds(np, O, H, L)
            small[f"config{cid}"] = {"tokens": int(L.cu_seqlens[-1]),
                                     "one_thread_ms_per_layer_pass": None if one is None else round(one * 1e3, 3),
                                     "all_threads_ms_per_layer_pass": round(many * 1e3, 3)}
        cpu = {"value": round(N / dt, 1), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"{passes} layer-passes over {len(host_layers)} layers of the same workload ({N} tokens, all "
                         f"{cfg.n_kv_heads} KV heads each, upcast to float64 included), float64 numpy, {dt:.2f} s per layer-pass",
               "kept_counts_match_gpu": agree, "small_configs": small}

    decode = time_decode_attention(torch, np, H, B, W) if args.decode else None
    all_layers = time_all_layers(torch, np, H, B, W, host_layers, cfg, args.all_layers) if args.all_layers else None
    wide = time_wide_window(np, H, B, W) if args.wide else None

    per_config = None
    if args.configs:
        del head, pos_dls, lse_objs, sdls                # make room: the other configurations bring their own buffers
        torch.cuda.empty_cache()
        per_config = {}
        for cid in args.configs.split(","):
            cid = int(cid) if cid.isdigit() else cid
            if cid == cfg_id:
                continue
            per_config[str(cid)] = time_config(torch, np, H, B, W, cid, args.streams)

    if args.calibrate_copy:
        src = torch.empty(128 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()

    line = {
        "metric": "tokens/s compressed per layer-pass at Llama3-8B shape, 32K ctx; % peak HBM BW",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": pos["steps"], "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_q_heads}q/{cfg.n_kv_heads}kv heads, d={cfg.head_dim}, "
                               f"batch {units // cfg.n_kv_heads}, {N} tokens, window {cfg.window}, T={cfg.threshold}, "
                               f"m={cfg.n_sink}, position ranking, K/V {args.kv_layout}, {args.layers} rotating layer buffers",
                   "rank_mode": "position", "retained_fraction": round(pos["kept_rows"] / (N * cfg.n_kv_heads), 4),
                   "launch": "hip_graph" if args.graph else "eager", "streams": args.streams,
                   "steps_requested": args.steps, "steps_run": pos["steps"], "replays": pos["replays"],
                   "timing": "median over replays of the HIP-event time of one replay / steps in it",
                   "ms_per_step_min_max": [round(pos["ms_min"], 5), round(pos["ms_max"], 5)],
                   "wall_ms_per_step": round(pos["wall_ms"], 5), "input_generation_s": round(gen_s, 1)},
        "percent_peak_hbm": round(100 * roofline["frac"], 2),
        "roofline": roofline, "cpu_baseline": cpu, "score_ranking": score_mode, "single_stream": single,
        "with_prefill_lse": with_lse, "all_layers_one_call": all_layers, "per_config": per_config,
        "decode_attention": decode, "wide_window": wide,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
