"""End-to-end GPU parity of the whole path (score -> select -> project) on the
synthetic workloads, chained on the device the way the benchmark runs it."""
from __future__ import annotations

import sys
import time

import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run_pipeline_gpu(w, q_bits, k_dev, L, doff, toff, mode):
    """One pass of the hot path with every intermediate left on the device."""
    import torch
    import paper_2603_02631_amd as sp
    from gpu_util import DEV, dev_bits, make_desc, workspace
    C = (L + w.chunk - 1) // w.chunk
    k = sp.sp_keep_count(C, w.keep_num, w.keep_den)
    M = toff.size - 1
    desc = make_desc(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_q, w.scale, mode, "HND", L)
    qd = dev_bits(q_bits)
    ws1 = workspace(sp.sp_score_workspace(desc, L, 1))
    ws2 = workspace(sp.sp_select_workspace(L, w.chunk))
    scores = torch.empty(L, dtype=torch.float32, device=DEV)
    sel = torch.empty(k, dtype=torch.int32, device=DEV)
    spans = torch.empty((k, 2), dtype=torch.int64, device=DEV)
    n_spans = torch.zeros(1, dtype=torch.int32, device=DEV)
    cs = torch.empty(C, dtype=torch.float32, device=DEV)
    dd = torch.from_numpy(doff).to(DEV)
    td = torch.from_numpy(toff).to(DEV)
    tsp = torch.empty((k, 2), dtype=torch.int64, device=DEV)
    n_t = torch.zeros(1, dtype=torch.int32, device=DEV)
    mask = torch.empty(M, dtype=torch.uint8, device=DEV)
    n_kept = torch.zeros(1, dtype=torch.int64, device=DEV)
    sp.sp_score(desc, qd, k_dev, L, scores, ws1)
    sp.sp_select(scores, L, w.pool, w.chunk, k, sel, spans, n_spans, cs, ws2)
    sp.sp_project(dd, L, td, M, spans, n_spans, k, tsp, n_t, mask, n_kept)
    torch.cuda.synchronize()
    ns, nt = int(n_spans.item()), int(n_t.item())
    return dict(scores=scores.cpu().numpy(), sel=sel.cpu().numpy().astype(np.int64), spans=spans[:ns].cpu().numpy(),
                cs=cs.cpu().numpy(), tspans=tsp[:nt].cpu().numpy(), mask=mask.cpu().numpy(),
                n_kept=int(n_kept.item()), k=k)


def check_pipeline(w, out, I, doff, toff, eps=2e-3):
    from gpu_util import assert_scores_close
    L = I.size
    assert_scores_close(out["scores"], I)
    o_sel, o_spans, o_cs = oracle.select(I, w.pool, w.chunk, out["k"])
    np.testing.assert_allclose(out["cs"].astype(np.float64), o_cs, rtol=1e-3)
    # selection: exact on the GPU's own chunk scores, and equal to the oracle's modulo near-ties
    np.testing.assert_array_equal(out["sel"], oracle.topk(out["cs"].astype(np.float64), out["k"]))
    tau = np.sort(o_cs)[::-1][out["k"] - 1]
    kept = np.zeros(o_cs.size, bool)
    kept[out["sel"]] = True
    assert kept[o_cs > tau * (1 + eps)].all() and not kept[o_cs < tau * (1 - eps)].any()
    diff = np.setxor1d(out["sel"], o_sel).size
    # spans and projection: exact given the GPU's selection
    np.testing.assert_array_equal(out["spans"], oracle.merge(out["sel"], w.chunk, L))
    ts, mask, n = oracle.project(doff, toff, out["spans"])
    np.testing.assert_array_equal(out["tspans"], ts)
    np.testing.assert_array_equal(out["mask"], mask)
    assert out["n_kept"] == n
    return diff


@pytest.mark.parametrize("name", ["tiny", "llama1b-8k", "qwen06b-32k"])
def test_pipeline_small_configs(name):
    from gpu_util import dev_bits
    w = synth.get_config(name)
    say(f"[pipeline] {name}: generating")
    inp = synth.make_score_inputs(w)
    doff, toff = synth.gen_char_offsets(w, w.L)
    k_dev = [dev_bits(k) for k in inp["k"]]
    for mode in (0, 1):
        t0 = time.time()
        I = oracle.score(inp["q"][0], inp["k"], w.scale, mode)
        say(f"[pipeline] {name} mode {mode}: oracle {time.time() - t0:.1f}s")
        out = run_pipeline_gpu(w, inp["q"][0], k_dev, w.L, doff, toff, mode)
        diff = check_pipeline(w, out, I, doff, toff)
        say(f"[pipeline] {name} mode {mode}: ok, selection differs from oracle in {diff} chunks, "
            f"kept {out['n_kept']} of {toff.size - 1} target tokens")


@pytest.mark.timeout(400)
def test_pipeline_full_size_benchmark_workload():
    """The 128K-token workload the benchmark times, in the benchmark's launch configuration (one
    prompt, HND keys, default stream, the single-launch score kernel): every score, then the chained
    selection and projection, against the oracle; both aggregation modes."""
    import paper_2603_02631_amd as sp
    from gpu_util import assert_scores_close, dev_bits, gpu_score, make_desc
    w = synth.get_config("long-128k")
    say(f"[pipeline] {w.name}: generating {w.k_bytes_per_token * w.L / 2**30:.2f} GiB of keys")
    inp = synth.make_score_inputs(w)
    doff, toff = synth.gen_char_offsets(w, w.L)
    assert sp.sp_score_is_fused(make_desc(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_q, w.scale, 0,
                                          "HND", w.L), w.L) == 1
    k_dev = [dev_bits(k) for k in inp["k"]]
    t0 = time.time()
    I = oracle.score(inp["q"][0], inp["k"], w.scale, oracle.LAYER_MEAN)
    say(f"[pipeline] {w.name} mean: oracle {time.time() - t0:.1f}s")
    out = run_pipeline_gpu(w, inp["q"][0], k_dev, w.L, doff, toff, oracle.LAYER_MEAN)
    diff = check_pipeline(w, out, I, doff, toff)
    say(f"[pipeline] {w.name} mean: ok, max rel err {np.max(np.abs(out['scores'] - I) / I):.2e}, selection differs "
        f"from oracle in {diff} chunks, kept {out['n_kept']} of {toff.size - 1} target tokens")
    del k_dev
    t0 = time.time()
    I = oracle.score(inp["q"][0], inp["k"], w.scale, oracle.LAYER_MAX)
    say(f"[pipeline] {w.name} max: oracle {time.time() - t0:.1f}s")
    got = gpu_score(inp["q"][0], inp["k"], w.scale, oracle.LAYER_MAX)
    assert_scores_close(got, I)
    say(f"[pipeline] {w.name} max: ok, max rel err {np.max(np.abs(got - I) / I):.2e}")


@pytest.mark.timeout(400)
def test_pipeline_full_size_quarter_million_tokens_chunk_128():
    """262144 tokens, chunk 128 (the code-debugging setting of Appendix A.3): too long for the
    single-launch kernel, so the general score path at full size with no layer split, then selection
    and projection; and the same prompt scored with the lookahead keys in the normaliser."""
    import paper_2603_02631_amd as sp
    from gpu_util import assert_scores_close, dev_bits, gpu_score_look, make_desc
    w = synth.get_config("long-256k")
    say(f"[pipeline] {w.name}: generating {w.k_bytes_per_token * w.L / 2**30:.2f} GiB of keys")
    inp = synth.make_score_inputs(w)
    doff, toff = synth.gen_char_offsets(w, w.L)
    assert sp.sp_score_is_fused(make_desc(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_q, w.scale, 0,
                                          "HND", w.L), w.L) == 0
    k_dev = [dev_bits(k) for k in inp["k"]]
    t0 = time.time()
    I = oracle.score(inp["q"][0], inp["k"], w.scale, oracle.LAYER_MEAN)
    say(f"[pipeline] {w.name} mean: oracle {time.time() - t0:.1f}s")
    out = run_pipeline_gpu(w, inp["q"][0], k_dev, w.L, doff, toff, oracle.LAYER_MEAN)
    diff = check_pipeline(w, out, I, doff, toff)
    say(f"[pipeline] {w.name} mean: ok, max rel err {np.max(np.abs(out['scores'] - I) / I):.2e}, selection differs "
        f"from oracle in {diff} chunks, kept {out['n_kept']} of {toff.size - 1} target tokens")
    kl = synth.gen_look_keys(w, inp["q"])
    t0 = time.time()
    I = oracle.score_look(inp["q"][0], inp["k"], kl, 1, w.scale, oracle.LAYER_MAX)
    say(f"[pipeline] {w.name} lookahead keys, max: oracle {time.time() - t0:.1f}s")
    got = gpu_score_look(inp["q"][0], inp["k"], kl, 1, w.scale, oracle.LAYER_MAX, k_dev=k_dev)
    assert_scores_close(got, I)
    say(f"[pipeline] {w.name} lookahead keys, max: ok, max rel err {np.max(np.abs(got - I) / I):.2e}")


@pytest.mark.timeout(400)
def test_score_batch_full_size_ragged_workload():
    """The 16-prompt ragged batch (2K to 64K tokens, 332K in all) at full size: every prompt's
    scores against the oracle run on that prompt alone."""
    from gpu_util import assert_scores_close, gpu_score_batch
    w = synth.get_config("ragged-16")
    lengths = synth.gen_prompt_lengths(w)
    say(f"[score_batch] {w.name}: {lengths.size} prompts, {int(lengths.sum())} tokens")
    hh = synth.heavy_hitter_positions(w, lengths)
    q = synth.gen_q(w, lengths.size)
    ks = [synth.gen_k_layer(w, l, q, lengths, hh) for l in range(w.n_layers)]
    offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    got = gpu_score_batch(q, ks, offsets, w.scale, oracle.LAYER_MEAN)
    t0 = time.time()
    worst = 0.0
    for b in range(lengths.size):
        sl = slice(int(offsets[b]), int(offsets[b + 1]))
        kb = [np.ascontiguousarray(k[:, sl, :]) for k in ks]
        want = oracle.score(q[b], kb, w.scale, oracle.LAYER_MEAN)
        assert_scores_close(got[sl], want)
        worst = max(worst, float(np.max(np.abs(got[sl] - want) / want)))
    say(f"[score_batch] {w.name}: ok, oracle {time.time() - t0:.1f}s, max rel err {worst:.2e}")
