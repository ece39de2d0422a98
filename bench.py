#!/usr/bin/env python3
"""Benchmark of the token-importance hot path on one MI355X.

One "step" is one pass of the whole path -- sp_score (sp_score_batch for the
ragged batch), sp_select, sp_project -- over synthetic prompts already resident
in HBM. The default workload is the 128K-token long-context configuration (16
layers, 32 query / 8 kv heads, head_dim 64, 16 lookahead rows): the one the
bandwidth target is quoted on.

Prints ONE JSON line with the throughput (prompt tokens scored per second
through all layers), the HBM roofline of sp_score (algorithmic K bytes read
once / measured duration, against the 8 TB/s peak and against the streaming-read
rate the library's own probe reaches on the same buffers) and the CPU oracle
timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
ROTATE_BYTES = 2 << 30          # K buffers are rotated over at least this much memory, so that no cache serves K

# HBM traffic of one sp_score call on the default workload, recorded from hardware counters (rocprofv3 --pmc
# FETCH_SIZE, then WRITE_SIZE, each scaled by what the counter reads for the 1 GiB calibration copy).
# It is reported only while the kernel sources are the ones the counters were taken on.
TRAFFIC = {
    "workload": "long-128k",
    "sources_sha256": "971240212852ba369836edad355ea8676dc7853e40188034fee0d7762d77563b",
    "fetch_bytes": 1090799.0 * 2048,      # FETCH_SIZE 1090799.0 per dispatch; the 1 GiB copy reads 524314 -> 2 KiB per count
    "write_bytes": 16960.0 * 1024,        # WRITE_SIZE 16960.0 per dispatch; the 1 GiB copy writes 1048576 -> 1 KiB per count
}
KERNEL_SOURCES = ["sp_score_fused.hip", "sp_score_fused.hpp", "sp_score_dev.hpp"]     # the dominant kernel and its headers


def kernel_sources_sha256() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2603_02631_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload: str):
    if TRAFFIC["sources_sha256"] is None or TRAFFIC["workload"] != workload:
        return None
    if kernel_sources_sha256() != TRAFFIC["sources_sha256"]:
        return None
    return float(TRAFFIC["fetch_bytes"] + TRAFFIC["write_bytes"])


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="untimed: the step is repeated for this long before the warm-up steps, so that the device's "
                         "power management has settled at its sustained clock (after an idle period the first few "
                         "dispatches run ~2 %% faster than sustained, the next ~40 up to 25 %% slower)")
    ap.add_argument("--first-calls", type=int, default=20,
                    help="steps timed right after the inputs are ready, before the settle phase: what a caller's "
                         "first calls cost (reported beside the sustained figure, never instead of it)")
    ap.add_argument("--probe-passes", type=int, default=10)
    ap.add_argument("--workload", default="long-128k")
    ap.add_argument("--layer-agg", default="mean", choices=["mean", "max"])
    ap.add_argument("--k-dtype", default="bf16", choices=["bf16", "fp8"],
                    help="fp8: the keys quantised to E4M3 codes with one scale per layer and kv head, scored by "
                         "sp_score_fp8 (a line of its own beside the bf16 one, never instead of it)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--batch-post", default="batch", choices=["batch", "graph", "eager"],
                    help="ragged batch: sp_select_batch + sp_project_batch (three launches for all prompts), or "
                         "sp_select + sp_project per prompt replayed from a HIP graph / launched call by call")
    ap.add_argument("--cpu-sample-layers", type=int, default=0,
                    help="layers the CPU oracle is timed on with all cores (0 = all layers of the workload)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 1 GiB device copy before the timed region (reference for HBM counters)")
    ap.add_argument("--print-sources-hash", action="store_true")
    args = ap.parse_args()
    if args.print_sources_hash:
        print(kernel_sources_sha256())
        return 0
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import synth
    import paper_2603_02631_amd as sp

    sp.load_library()            # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = "cuda:0"
    w = synth.get_config(args.workload)
    mode = sp.SP_LAYER_MEAN if args.layer_agg == "mean" else sp.SP_LAYER_MAX
    ragged = w.batch > 0
    fp8 = args.k_dtype == "fp8"
    if fp8 and ragged:
        print("bench.py: 8-bit keys are scored one prompt at a time (sp_score_fp8)", file=sys.stderr)
        return 2

    # ---- inputs: generated on the host by the seeded generator, uploaded once ----
    t0 = time.time()
    lengths = synth.gen_prompt_lengths(w)
    B = int(lengths.size)
    offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    T = int(offsets[-1])                     # tokens per step (all prompts)
    hh = synth.heavy_hitter_positions(w, lengths)
    q_bits = synth.gen_q(w, B)
    k_bytes = float(w.k_bytes_per_token) * T / (2 if fp8 else 1)
    # short workloads: the same K replicated n_rot times and walked round-robin, so that every call streams
    # from HBM rather than from the 256 MB memory-side cache
    n_rot = 1 if k_bytes >= ROTATE_BYTES else int(-(-ROTATE_BYTES // int(k_bytes)))
    if args.cpu_sample_layers <= 0:
        args.cpu_sample_layers = w.n_layers
    qd = torch.from_numpy((q_bits if ragged else q_bits[0]).view(np.int16)).to(dev)
    # all layers of a copy sit in one allocation (the probe then streams a copy with one launch)
    k_big = torch.empty((n_rot, w.n_layers, w.n_kv_heads, T, w.head_dim), dtype=torch.uint8 if fp8 else torch.int16,
                        device=dev)
    k_sample = []                # host copies of the layers the CPU baseline uses
    kscale = np.ones((w.n_layers, w.n_kv_heads), dtype=np.float32)
    for l in range(w.n_layers):
        k = synth.gen_k_layer(w, l, q_bits, lengths, hh)
        if fp8:
            k, kscale[l] = synth.quantise_k_e4m3(k)
        if l < args.cpu_sample_layers and not args.no_cpu_baseline:
            k_sample.append(k)
        k_big[:, l] = torch.from_numpy(k if fp8 else k.view(np.int16)).to(dev).unsqueeze(0)
    kscale_dev = torch.from_numpy(kscale).to(dev)
    k_sets = [[k_big[r, l] for l in range(w.n_layers)] for r in range(n_rot)]
    chars = [synth.gen_char_offsets(w, int(lengths[b]), prompt=b) for b in range(B)]
    M_all = [int(t.size - 1) for _, t in chars]
    log(f"[bench] inputs for {w.name} ready in {time.time() - t0:.1f}s ({B} prompt(s), {T} tokens, "
        f"K = {k_bytes / 2**30:.2f} GiB x {n_rot} rotating copies, {sum(M_all)} target tokens)")

    desc = sp.ScoreDesc(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_q, w.scale, mode,
                        w.head_dim, T * w.head_dim)
    ws1 = torch.empty(sp.sp_score_workspace(desc, T, B), dtype=torch.uint8, device=dev)
    scores = torch.empty(T, dtype=torch.float32, device=dev)
    off_host = [int(v) for v in offsets]
    off_dev = torch.from_numpy(offsets).to(dev)
    per = []                     # per prompt: buffers of sp_select / sp_project
    for b in range(B):
        Lb, (doff, toff) = int(lengths[b]), chars[b]
        C = (Lb + w.chunk - 1) // w.chunk
        kk = sp.sp_keep_count(C, w.keep_num, w.keep_den)
        per.append(dict(
            L=Lb, M=M_all[b], k=kk, scores=scores[off_host[b]:off_host[b + 1]],
            ws=torch.empty(sp.sp_select_workspace(Lb, w.chunk), dtype=torch.uint8, device=dev),
            sel=torch.empty(kk, dtype=torch.int32, device=dev), spans=torch.empty((kk, 2), dtype=torch.int64, device=dev),
            n_spans=torch.zeros(1, dtype=torch.int32, device=dev), dd=torch.from_numpy(doff).to(dev),
            td=torch.from_numpy(toff).to(dev), tsp=torch.empty((kk, 2), dtype=torch.int64, device=dev),
            n_t=torch.zeros(1, dtype=torch.int32, device=dev), mask=torch.empty(M_all[b], dtype=torch.uint8, device=dev),
            n_kept=torch.zeros(1, dtype=torch.int64, device=dev)))
    stream = torch.cuda.current_stream()
    if ragged:
        fused = 1 if sp.sp_score_batch_is_fused(desc, off_host) > 0 else 0
    else:
        fused = sp.sp_score_fp8_is_fused(desc, T) if fp8 else sp.sp_score_is_fused(desc, T)
    calls = [0]
    # ragged batch: the prompts' select / project chains (one-workgroup kernels) are independent of each other
    # and go round robin onto a few streams of default priority, so that they overlap
    side = [torch.cuda.Stream(device=dev) for _ in range(min(4, B))] if ragged else []

    def enqueue_select_project(main):
        """sp_select + sp_project of every prompt behind whatever is on `main`; `main` waits for all of it."""
        if side:
            scored = torch.cuda.Event()
            scored.record(main)
            for sd in side:
                sd.wait_event(scored)
        for i, p in enumerate(per):
            st = side[i % len(side)] if side else main
            sp.sp_select(p["scores"], p["L"], w.pool, w.chunk, p["k"], p["sel"], p["spans"], p["n_spans"], None,
                         p["ws"], stream=st)
            sp.sp_project(p["dd"], p["L"], p["td"], p["M"], p["spans"], p["n_spans"], p["k"], p["tsp"], p["n_t"],
                          p["mask"], p["n_kept"], stream=st)
        for sd in side:     # the next step's score call overwrites the scores: it waits for all of them
            e = torch.cuda.Event()
            e.record(sd)
            main.wait_event(e)

    graph = [None]
    batch_post = None
    if ragged and args.batch_post == "batch":
        # all prompts in three launches: packed inputs and outputs
        kept_host = [0]
        for p in per:
            kept_host.append(kept_host[-1] + p["k"])
        moff_host = [0]
        for p in per:
            moff_host.append(moff_host[-1] + p["M"])
        K = kept_host[-1]
        i64 = dict(dtype=torch.int64, device=dev)
        batch_post = dict(
            kept_host=kept_host, moff_host=moff_host, kept_dev=torch.tensor(kept_host, **i64),
            moff_dev=torch.tensor(moff_host, **i64), dd=torch.cat([p["dd"] for p in per]), td=torch.cat([p["td"] for p in per]),
            sel=torch.empty(K, dtype=torch.int32, device=dev), spans=torch.empty((K, 2), **i64),
            n_spans=torch.zeros(B, dtype=torch.int32, device=dev), tsp=torch.empty((K, 2), **i64),
            n_t=torch.zeros(B, dtype=torch.int32, device=dev), mask=torch.empty(moff_host[-1], dtype=torch.uint8, device=dev),
            n_kept=torch.zeros(B, **i64),
            ws=torch.empty(sp.sp_select_batch_workspace(T, B, w.chunk), dtype=torch.uint8, device=dev))

    def step(ev=None):
        # two events per step bracket the score call on its stream; the rest of the step follows from the wall clock
        k_dev = k_sets[calls[0] % n_rot]
        calls[0] += 1
        if ev is not None:
            ev[0].record(stream)
        if ragged:
            sp.sp_score_batch(desc, qd, k_dev, off_host, off_dev, scores, ws1, stream=stream)
        elif fp8:
            sp.sp_score_fp8(desc, qd, k_dev, kscale_dev, T, scores, ws1, stream=stream)
        else:
            sp.sp_score(desc, qd, k_dev, T, scores, ws1, stream=stream)
        if ev is not None:
            ev[1].record(stream)
        if batch_post is not None:
            bp = batch_post
            sp.sp_select_batch(scores, off_host, off_dev, w.pool, w.chunk, bp["kept_host"], bp["kept_dev"], bp["sel"],
                               bp["spans"], bp["n_spans"], None, bp["ws"], stream=stream)
            sp.sp_project_batch(bp["dd"], off_host, off_dev, bp["td"], bp["moff_host"], bp["moff_dev"], bp["spans"],
                                bp["n_spans"], bp["kept_host"], bp["kept_dev"], bp["tsp"], bp["n_t"], bp["mask"],
                                bp["n_kept"], stream=stream)
        elif graph[0] is not None:
            graph[0].replay()
        else:
            enqueue_select_project(stream)

    def post_outputs():
        return [(int(p["n_spans"].item()), p["spans"].cpu().numpy().copy(), int(p["n_t"].item()),
                 p["tsp"].cpu().numpy().copy(), p["mask"].cpu().numpy().copy(), int(p["n_kept"].item())) for p in per]

    def same_outputs(a, b):
        for x, y in zip(a, b):
            if x[0] != y[0] or x[2] != y[2] or x[5] != y[5]:
                return False
            if not (np.array_equal(x[1][:x[0]], y[1][:y[0]]) and np.array_equal(x[3][:x[2]], y[3][:y[2]])
                    and np.array_equal(x[4], y[4])):
                return False
        return True

    def build_graph():
        """The launch-bound select / project stage (3 one-workgroup launches per prompt, nothing else: the
        library enqueues no memory sets or copies) recorded once as a HIP graph, parallel chains for a ragged
        batch. Every replay below is checked against the eager result, with eager work in between."""
        step()
        torch.cuda.synchronize()
        want = post_outputs()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            enqueue_select_project(torch.cuda.current_stream())
        for trial in range(3):
            for p in per:
                p["n_spans"].zero_(); p["n_t"].zero_(); p["n_kept"].zero_(); p["mask"].fill_(9); p["tsp"].fill_(-7)
            step()                       # eager work (score + select + project) between the replays
            torch.cuda.synchronize()
            for p in per:
                p["n_spans"].zero_(); p["n_t"].zero_(); p["n_kept"].zero_(); p["mask"].fill_(9); p["tsp"].fill_(-7)
            g.replay()
            torch.cuda.synchronize()
            if not same_outputs(post_outputs(), want):
                log(f"[bench] graph replay {trial} differs from the eager result: graph not used")
                return None
        return g

    def timed(n):
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n)]
        t_a = time.perf_counter()
        for i in range(n):
            step(events[i])
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t_a) * 1e3 / max(n, 1)
        return wall_ms, np.array([e[0].elapsed_time(e[1]) for e in events], dtype=np.float64)

    if args.calibration_copy:
        a_src = torch.ones(2**28, dtype=torch.float32, device=dev)       # 1 GiB read + 1 GiB written
        a_dst = torch.empty_like(a_src)
        torch.cuda.synchronize()
        a_dst.copy_(a_src)
        torch.cuda.synchronize()
        del a_src, a_dst
    torch.cuda.synchronize()
    if ragged and args.batch_post == "graph":
        graph[0] = build_graph()
        time.sleep(1.0)          # the first calls below are meant to follow an idle period
    first_wall, first_score = timed(args.first_calls) if args.first_calls > 0 else (None, np.zeros(0))
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ms_per_step, score_all = timed(args.steps)
    score_ms, score_mean = float(np.median(score_all)), float(np.mean(score_all))
    rest_ms = ms_per_step - score_mean
    achieved = k_bytes / (score_ms * 1e-3) / 1e9
    status = int(ws1[:4].cpu().numpy().view(np.uint32)[0])
    if status != 0 or not bool(torch.isfinite(scores).all()):
        print(f"bench.py: invalid scores after the timed steps (status word {status})", file=sys.stderr)
        return 4
    if batch_post is not None:
        # the batch calls against the per-prompt calls on the same scores: identical results
        torch.cuda.synchronize()
        got = (batch_post["n_kept"].cpu().numpy().copy(), batch_post["mask"].cpu().numpy().copy())
        enqueue_select_project(stream)
        torch.cuda.synchronize()
        want_kept = np.array([int(p["n_kept"].item()) for p in per])
        want_mask = np.concatenate([p["mask"].cpu().numpy() for p in per])
        if not (np.array_equal(got[0], want_kept) and np.array_equal(got[1], want_mask)):
            print("bench.py: sp_select_batch / sp_project_batch differ from the per-prompt calls", file=sys.stderr)
            return 4
        n_kept = int(got[0].sum())
    else:
        n_kept = sum(int(p["n_kept"].item()) for p in per)

    # ---- streaming-read probe over the same K buffers: the achievable rate on this device ----
    sink = torch.zeros(1, dtype=torch.int64, device=dev)
    probe_ms = []
    for i in range(args.probe_passes + 2):
        kt = k_big[i % n_rot]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        sp.sp_hbm_read_probe(kt, kt.numel() * kt.element_size(), sink, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        if i >= 2:
            probe_ms.append(e0.elapsed_time(e1))
    probe_gbs = k_bytes / (float(np.median(probe_ms)) * 1e-3) / 1e9 if probe_ms else None
    log(f"[bench] {args.steps} steps: {ms_per_step:.3f} ms/step; score {score_ms:.3f} ms median / {score_mean:.3f} mean "
        f"({achieved:.0f} GB/s algorithmic; probe {probe_gbs or 0:.0f} GB/s), select+project {rest_ms:.3f} ms; "
        f"kept {n_kept} of {sum(M_all)}"
        + (f"; first {args.first_calls} calls: score {float(np.median(first_score)):.3f} ms median" if first_score.size else ""))

    score_name = "sp_score_batch" if ragged else ("sp_score_fp8" if fp8 else "sp_score")
    stage_ms = {score_name: score_ms, score_name + "_mean": score_mean, "sp_select+sp_project": rest_ms}
    if first_score.size:
        stage_ms[score_name + "_first_calls_median"] = float(np.median(first_score))
        stage_ms[score_name + "_first_calls_max"] = float(np.max(first_score))
        stage_ms["step_first_calls"] = first_wall
    cfg = {"workload": w.name, "n_layers": w.n_layers, "n_q_heads": w.n_q_heads,
           "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "n_q": w.n_q, "pool": w.pool, "chunk": w.chunk,
           "keep": f"{w.keep_num}/{w.keep_den}", "layer_agg": args.layer_agg, "k_layout": "HND", "k_dtype": args.k_dtype,
           "k_rotating_copies": n_rot, "score_path": "single-launch" if fused == 1 else "three-kernel",
           "select_project_launch": ("batch calls" if batch_post is not None else
                                     "hip graph" if graph[0] is not None else "per prompt")}
    if ragged:
        cfg.update({"prompts": B, "total_tokens": T, "min_len": int(lengths.min()), "max_len": int(lengths.max())})
    else:
        cfg["L"] = T
    out = {
        "metric": "prompt tokens scored/sec (all layers)",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_ms": args.settle_ms,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp8" if fp8 else "bf16",
        "data": "synthetic",
        "config": cfg,
        "stage_ms": stage_ms,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(w.name),
                     "traffic_source": "recorded rocprofv3 counters, valid for the kernel sources they were taken on",
                     "probe_gbs": probe_gbs, "frac_of_probe": (achieved / probe_gbs) if probe_gbs else None,
                     "kernel": score_name + " (all its launches, median of the timed steps)",
                     "algorithmic_bytes": k_bytes},
    }

    if not args.no_cpu_baseline:
        import oracle
        n_all = oracle.max_threads()
        n_s = min(args.cpu_sample_layers, w.n_layers)

        def oracle_score_seconds(n_layers):
            t_a = time.perf_counter()
            res = []
            for b in range(B):
                sl = slice(off_host[b], off_host[b + 1])
                kb = [np.ascontiguousarray(k[:, sl, :]) for k in k_sample[:n_layers]] if ragged else k_sample[:n_layers]
                if fp8:
                    res.append(oracle.score_fp8(q_bits[b, :n_layers], kb, kscale[:n_layers].astype(np.float64), w.scale, mode))
                else:
                    res.append(oracle.score(q_bits[b, :n_layers], kb, w.scale, mode))
            return time.perf_counter() - t_a, res

        t_score, I_all = oracle_score_seconds(n_s)
        t0 = time.perf_counter()
        for b in range(B):
            _, o_spans, _ = oracle.select(I_all[b], w.pool, w.chunk, per[b]["k"])
            oracle.project(chars[b][0], chars[b][1], o_spans)
        t_rest = time.perf_counter() - t0
        oracle.set_threads(1)
        try:
            t_one, _ = oracle_score_seconds(1)
        finally:
            oracle.set_threads(n_all)
        t_full = t_score * w.n_layers / n_s + t_rest
        t_full_1 = t_one * w.n_layers + t_rest
        out["cpu_baseline"] = {
            "value": T / t_full, "unit": "tokens/s", "cores": n_all, "kind": "oracle",
            "value_1thread": T / t_full_1,
            "sample": f"{n_all} threads: score pass on {n_s} of {w.n_layers} layers, all {T} tokens ({t_score:.1f}s); "
                      f"1 thread: score pass on 1 layer ({t_one:.1f}s); both scaled linearly to {w.n_layers} layers, "
                      f"plus the full select/project ({t_rest:.2f}s, single-threaded code)",
        }
        log(f"[bench] oracle: {t_score:.1f}s for {n_s} layer(s) on {n_all} threads, {t_one:.1f}s for 1 layer on 1 thread")
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
