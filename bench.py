#!/usr/bin/env python3
"""Benchmark of the token-importance hot path on one MI355X.

One "step" is one pass of the whole path -- sp_score, sp_select, sp_project --
over one synthetic prompt already resident in HBM. The default workload is the
128K-token long-context configuration (16 layers, 32 query / 8 kv heads,
head_dim 64, 16 lookahead rows): the one the bandwidth target is quoted on.

Prints ONE JSON line with the throughput (prompt tokens scored per second
through all layers), the HBM roofline of sp_score (algorithmic K bytes read
once / measured duration, against the 8 TB/s peak) and the CPU oracle timed on
a bounded sample of the same workload.
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

# HBM traffic of one sp_score call on the default workload, from hardware counters (rocprofv3 --pmc
# FETCH_SIZE, then WRITE_SIZE, each scaled by what the counter reads for the 1 GiB calibration copy).
# It is reported only while the kernel sources are the ones the counters were taken on.
TRAFFIC = {
    "workload": "long-128k",
    "sources_sha256": "3f583bcc070e7a9b61a94a09f9e918ee01e130fc5da73d9b45b7b1fd390008bd",
    "fetch_bytes": 1090789.5 * 2048,      # FETCH_SIZE 1090789.5 per dispatch; the 1 GiB copy reads 524307 -> 2 KiB per count
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
    ap.add_argument("--workload", default="long-128k")
    ap.add_argument("--layer-agg", default="mean", choices=["mean", "max"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-layers", type=int, default=0,
                    help="layers the CPU oracle is timed on (0 = all layers of the workload)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 1 GiB device copy before the timed region (reference for HBM counters)")
    ap.add_argument("--print-sources-hash", action="store_true")
    args = ap.parse_args()
    if args.print_sources_hash:
        print(kernel_sources_sha256())
        return 0
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
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
    if w.batch > 0:
        print("bench.py: the ragged batch is a parity-test case, not a bench workload", file=sys.stderr)
        return 2
    mode = sp.SP_LAYER_MEAN if args.layer_agg == "mean" else sp.SP_LAYER_MAX
    L = w.L
    if args.cpu_sample_layers <= 0:
        args.cpu_sample_layers = w.n_layers

    # ---- inputs: generated on the host by the seeded generator, uploaded once ----
    t0 = time.time()
    lengths = synth.gen_prompt_lengths(w)
    hh = synth.heavy_hitter_positions(w, lengths)
    q_bits = synth.gen_q(w, 1)
    qd = torch.from_numpy(q_bits[0].view(np.int16)).to(dev)
    k_dev = []
    k_sample = []                # host copies of the layers the CPU baseline uses
    for l in range(w.n_layers):
        k = synth.gen_k_layer(w, l, q_bits, lengths, hh)
        if l < args.cpu_sample_layers and not args.no_cpu_baseline:
            k_sample.append(k)
        k_dev.append(torch.from_numpy(k.view(np.int16)).to(dev))
    doff, toff = synth.gen_char_offsets(w, L)
    M = toff.size - 1
    log(f"[bench] inputs for {w.name} ready in {time.time() - t0:.1f}s "
        f"(K = {w.k_bytes_per_token * L / 2**30:.2f} GiB, M = {M} target tokens)")

    C = (L + w.chunk - 1) // w.chunk
    k_keep = sp.sp_keep_count(C, w.keep_num, w.keep_den)
    desc = sp.ScoreDesc(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_q, w.scale, mode,
                        w.head_dim, L * w.head_dim)
    ws1 = torch.empty(sp.sp_score_workspace(desc, L, 1), dtype=torch.uint8, device=dev)
    ws2 = torch.empty(sp.sp_select_workspace(L, w.chunk), dtype=torch.uint8, device=dev)
    scores = torch.empty(L, dtype=torch.float32, device=dev)
    sel = torch.empty(k_keep, dtype=torch.int32, device=dev)
    spans = torch.empty((k_keep, 2), dtype=torch.int64, device=dev)
    n_spans = torch.zeros(1, dtype=torch.int32, device=dev)
    dd = torch.from_numpy(doff).to(dev)
    td = torch.from_numpy(toff).to(dev)
    tsp = torch.empty((k_keep, 2), dtype=torch.int64, device=dev)
    n_t = torch.zeros(1, dtype=torch.int32, device=dev)
    mask = torch.empty(M, dtype=torch.uint8, device=dev)
    n_kept = torch.zeros(1, dtype=torch.int64, device=dev)
    stream = torch.cuda.current_stream()

    def step(ev=None):
        # two events per step bracket sp_score on its stream; the rest of the step follows from the wall clock
        if ev is not None:
            ev[0].record(stream)
        sp.sp_score(desc, qd, k_dev, L, scores, ws1, stream=stream)
        if ev is not None:
            ev[1].record(stream)
        sp.sp_select(scores, L, w.pool, w.chunk, k_keep, sel, spans, n_spans, None, ws2, stream=stream)
        sp.sp_project(dd, L, td, M, spans, n_spans, k_keep, tsp, n_t, mask, n_kept, stream=stream)

    if args.calibration_copy:
        a_src = torch.ones(2**28, dtype=torch.float32, device=dev)       # 1 GiB read + 1 GiB written
        a_dst = torch.empty_like(a_src)
        torch.cuda.synchronize()
        a_dst.copy_(a_src)
        torch.cuda.synchronize()
        del a_src, a_dst
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    score_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    rest_ms = ms_per_step - score_ms
    k_bytes = float(w.k_bytes_per_token) * L
    achieved = k_bytes / (score_ms * 1e-3) / 1e9
    log(f"[bench] {args.steps} steps: {ms_per_step:.3f} ms/step; sp_score {score_ms:.3f} ms "
        f"({achieved:.0f} GB/s algorithmic), select+project {rest_ms:.3f} ms; kept {int(n_kept.item())} of {M}")

    out = {
        "metric": "prompt tokens scored/sec (all layers)",
        "value": L / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_ms": args.settle_ms,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "n_layers": w.n_layers, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "n_q": w.n_q, "L": L,
                   "pool": w.pool, "chunk": w.chunk, "keep": f"{w.keep_num}/{w.keep_den}",
                   "layer_agg": args.layer_agg, "k_layout": "HND"},
        "stage_ms": {"sp_score": score_ms, "sp_select+sp_project": rest_ms},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(w.name),
                     "kernel": "sp_score (all its launches)", "algorithmic_bytes": k_bytes},
    }

    if not args.no_cpu_baseline:
        import oracle
        n_s = min(args.cpu_sample_layers, w.n_layers)
        t0 = time.perf_counter()
        I = oracle.score(q_bits[0, :n_s], k_sample, w.scale, mode)
        t_score = time.perf_counter() - t0
        t0 = time.perf_counter()
        o_sel, o_spans, _ = oracle.select(I, w.pool, w.chunk, k_keep)
        oracle.project(doff, toff, o_spans)
        t_rest = time.perf_counter() - t0
        t_full = t_score * w.n_layers / n_s + t_rest
        out["cpu_baseline"] = {
            "value": L / t_full, "unit": "tokens/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"score pass on {n_s} of {w.n_layers} layers at full L={L} ({t_score:.1f}s, scaled "
                      f"linearly to all layers) + full select/project ({t_rest:.2f}s)",
        }
        log(f"[bench] oracle: {t_score:.1f}s for {n_s} layer(s) on {oracle.max_threads()} threads")
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
