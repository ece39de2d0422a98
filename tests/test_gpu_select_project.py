"""GPU parity of sp_select and sp_project against the CPU oracle.

Chunk scores are compared within 1e-3 relative. Selection is integer work that
floating point decides, so it is checked three ways: (a) exactly, against the
oracle's top-k applied to the GPU's own fp32 chunk scores (same precision on
both sides of the decision); (b) exactly, on inputs whose ties are exact in
both precisions; (c) end to end "modulo ties": every chunk clearly above the
k-th oracle score is kept and none clearly below. Spans and projections are
compared exactly."""
from __future__ import annotations

import sys

import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def check_select(scores32: np.ndarray, pool_w: int, chunk: int, k: int, eps: float = 2e-3):
    from gpu_util import gpu_select
    L = scores32.size
    sel, spans, cs = gpu_select(scores32, pool_w, chunk, k)
    o_sel, o_spans, o_cs = oracle.select(scores32.astype(np.float64), pool_w, chunk, k)
    # chunk scores within tolerance
    np.testing.assert_allclose(cs.astype(np.float64), o_cs, rtol=1e-3, atol=1e-30)
    # (a) kernel-exact: oracle top-k on the GPU's own fp32 chunk scores
    exact = oracle.topk(cs.astype(np.float64), k)
    np.testing.assert_array_equal(sel.astype(np.int64), exact)
    # spans are exactly the merge of the GPU's selection
    np.testing.assert_array_equal(spans, oracle.merge(exact, chunk, L))
    # (c) modulo ties against the float64 oracle
    tau = np.sort(o_cs)[::-1][k - 1]
    kept = np.zeros(o_cs.size, bool)
    kept[sel] = True
    assert kept.sum() == k
    assert kept[o_cs > tau * (1 + eps)].all()
    assert not kept[o_cs < tau * (1 - eps)].any()
    return sel, spans, o_sel


@pytest.mark.parametrize("L,pool_w,chunk,keep", [
    (1024, 13, 32, (25, 100)), (1000, 13, 32, (20, 100)), (8192, 13, 32, (20, 100)),
    (131072, 13, 64, (10, 100)), (70000, 13, 16, (15, 100)),     # > 1024 chunks: multi-segment scans
    (40000, 13, 4, (10, 100)),                                   # 10000 chunks: keys re-read per pass, not cached
    (5, 13, 32, (100, 100)), (12, 13, 4, (50, 100)), (300, 1, 7, (30, 100)), (300, 129, 32, (30, 100)),
    (4097, 13, 128, (25, 100)), (999, 5, 1, (10, 100)), (2000, 13, 5000, (10, 100)),
])
def test_select_random_scores(L, pool_w, chunk, keep):
    say(f"[select] L={L} pool={pool_w} chunk={chunk} keep={keep}")
    rng = np.random.default_rng(L * 31 + chunk)
    scores = (rng.random(L) ** 8).astype(np.float32) / L          # skewed, like importance scores
    hot = rng.choice(L, size=max(1, L // 100), replace=False)
    scores[hot] += 0.05
    C = (L + chunk - 1) // chunk
    k = oracle.keep_count(C, *keep)
    check_select(scores, pool_w, chunk, k)
    check_select(scores, pool_w, chunk, 1)
    check_select(scores, pool_w, chunk, C)


def test_select_exact_ties_take_lower_index():
    """Constant and integer-valued scores tie exactly in fp32 and fp64."""
    from gpu_util import gpu_select
    say("[select] exact ties")
    L, c = 416, 32
    const = np.full(L, 2.0 ** -9, dtype=np.float32)
    sel, spans, cs = gpu_select(const, 13, c, 4)
    o_sel, o_spans, _ = oracle.select(const.astype(np.float64), 13, c, 4)
    np.testing.assert_array_equal(sel, o_sel)
    np.testing.assert_array_equal(spans, o_spans)
    np.testing.assert_array_equal(sel, [1, 2, 3, 4])
    rng = np.random.default_rng(3)
    for trial in range(6):
        C = int(rng.integers(3, 3000))
        vals = rng.integers(0, 5, size=C).astype(np.float32)        # chunk = 1, pool = 1: scores are the chunk scores
        if trial == 0:
            vals[::7] = -0.0
        for k in (1, C // 3 + 1, C):
            sel, spans, cs = gpu_select(vals, 1, 1, k)
            o_sel, o_spans, _ = oracle.select(vals.astype(np.float64), 1, 1, k)
            np.testing.assert_array_equal(sel, o_sel)
            np.testing.assert_array_equal(spans, o_spans)
    neg = -np.arange(1, 200, dtype=np.float32)                       # negative scores order correctly
    sel, _, _ = gpu_select(neg, 1, 1, 5)
    np.testing.assert_array_equal(sel, [0, 1, 2, 3, 4])


def test_select_without_chunk_score_output_and_determinism():
    from gpu_util import gpu_select
    say("[select] no chunk-score output")
    rng = np.random.default_rng(9)
    s = rng.random(5000).astype(np.float32)
    a = gpu_select(s, 13, 32, 40, want_chunk_scores=False)
    b = gpu_select(s, 13, 32, 40, want_chunk_scores=True)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    assert a[2] is None


def offsets_from_lengths(lens):
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)


def split_same_text(rng, total, max_len, allow_zero=False):
    cuts = [0]
    while cuts[-1] < total:
        step = int(rng.integers(0 if allow_zero else 1, max_len + 1))
        cuts.append(min(total, cuts[-1] + step))
    return np.array(cuts, dtype=np.int64)


def check_project(doff, toff, spans):
    from gpu_util import gpu_project
    ts, mask, n = gpu_project(doff, toff, spans)
    o_ts, o_mask, o_n = oracle.project(doff, toff, spans)
    np.testing.assert_array_equal(ts, o_ts)
    np.testing.assert_array_equal(mask, o_mask)
    assert n == o_n
    ts2, m2, n2 = gpu_project(doff, toff, spans, want_mask=False, max_spans=max(1, spans.shape[0]) + 3)
    np.testing.assert_array_equal(ts2, o_ts)
    assert m2 is None and n2 == o_n
    # a capacity beyond what the one-launch kernel holds in LDS takes the three-launch path
    ts3, m3, n3 = gpu_project(doff, toff, spans, max_spans=1500)
    np.testing.assert_array_equal(ts3, o_ts)
    np.testing.assert_array_equal(m3, o_mask)
    assert n3 == o_n


def random_spans(rng, L, n_max):
    n = int(rng.integers(0, n_max + 1))
    pts = np.sort(rng.choice(L + 1, size=min(2 * n, (L + 1) // 2 * 2), replace=False))
    return pts.reshape(-1, 2).astype(np.int64)


def test_project_random_cases_match_oracle_exactly():
    say("[project] random")
    rng = np.random.default_rng(21)
    for trial in range(40):
        L = int(rng.integers(1, 400))
        doff = offsets_from_lengths(rng.integers(1, 9, size=L))
        toff = split_same_text(rng, int(doff[-1]), 7)
        check_project(doff, toff, random_spans(rng, L, 12))


def test_project_many_spans_and_special_tokenisations():
    say("[project] many spans / identity / chars / single token / zero-length tokens")
    rng = np.random.default_rng(22)
    L = 40000
    doff = offsets_from_lengths(rng.geometric(0.25, size=L))
    toff = split_same_text(rng, int(doff[-1]), 9)
    C = L // 32
    sel = np.sort(rng.choice(C, size=C // 3, replace=False)).astype(np.int64)      # ~ 300 spans: > one scan segment
    spans = oracle.merge(sel, 32, L)
    assert spans.shape[0] > 256
    check_project(doff, toff, spans)
    check_project(doff, doff, spans)                                               # identity tokenisation
    check_project(doff, np.arange(int(doff[-1]) + 1, dtype=np.int64), spans[:50])  # one char per target token
    check_project(doff, np.array([0, doff[-1]], dtype=np.int64), spans[:3])        # a single target token
    check_project(doff, toff, np.array([[0, L]], dtype=np.int64))                  # keep everything
    check_project(doff, toff, np.zeros((0, 2), np.int64))                          # keep nothing
    # zero-length tokens on both sides (offsets only non-decreasing)
    for trial in range(20):
        Ls = int(rng.integers(1, 120))
        d2 = offsets_from_lengths(rng.integers(0, 4, size=Ls))
        if d2[-1] == 0:
            d2[-1] = 1
        t2 = split_same_text(rng, int(d2[-1]), 3, allow_zero=True)
        check_project(d2, t2, random_spans(rng, Ls, 8))


def test_project_long_prompt_coarse_index_strides():
    say("[project] long prompts: coarse-index strides 2 .. 63 and beyond")
    rng = np.random.default_rng(23)
    for L, mean_len in ((6000, 3), (131072, 4), (131072, 6), (131072, 7)):
        doff = offsets_from_lengths(rng.geometric(1.0 / mean_len, size=L))
        toff = split_same_text(rng, int(doff[-1]), 5)
        C = L // 32
        sel = np.sort(rng.choice(C, size=min(C // 10, 400), replace=False)).astype(np.int64)
        spans = oracle.merge(sel, 32, L)
        say(f"  L={L} M={toff.size - 1} spans={spans.shape[0]}")
        check_project(doff, toff, spans)
        check_project(doff, toff, np.array([[0, 1], [L - 1, L]], dtype=np.int64))   # first and last token


def test_project_workload_char_models():
    say("[project] workload char models")
    for name in ("tiny", "llama1b-8k"):
        w = synth.get_config(name)
        doff, toff = synth.gen_char_offsets(w, w.L)
        rng = np.random.default_rng(w.cfg_id)
        C = (w.L + w.chunk - 1) // w.chunk
        k = oracle.keep_count(C, w.keep_num, w.keep_den)
        sel = np.sort(rng.choice(C, size=k, replace=False)).astype(np.int64)
        check_project(doff, toff, oracle.merge(sel, w.chunk, w.L))


BATCHES = [
    # name, prompt lengths, pool, chunk, keep
    ("batch_mixed", [1000, 0, 1, 31, 5000, 40000, 33, 0], 13, 32, (20, 100)),
    ("batch_many_chunks", [70000, 300, 9000], 13, 16, (15, 100)),        # 4375 chunks: eight key segments per thread
    ("batch_keys_reread", [40000, 12], 13, 4, (10, 100)),                # 10000 chunks: keys re-read per pass
    ("batch_single_prompt", [12345], 5, 64, (25, 100)),
    ("batch_all_empty", [0, 0, 0], 13, 32, (20, 100)),
    ("batch_wide_pool_short_prompts", [5, 200, 64, 129], 129, 32, (50, 100)),
]


@pytest.mark.parametrize("case", BATCHES, ids=[c[0] for c in BATCHES])
def test_select_and_project_batch_match_the_per_prompt_calls_and_the_oracle(case):
    """sp_select_batch / sp_project_batch on packed ragged inputs: every prompt bit-identical to
    sp_select / sp_project on that prompt alone (same kernels' arithmetic), selection exact against the
    oracle's top-k on the GPU's chunk scores, projection exact against the oracle; nothing written
    outside a prompt's share of the packed outputs."""
    import torch
    import paper_2603_02631_amd as sp
    from gpu_util import DEV, gpu_select, workspace
    name, lens, pool_w, chunk, keep = case
    say(f"[select/project batch] {name} lengths={lens} pool={pool_w} chunk={chunk} keep={keep}")
    B = len(lens)
    rng = np.random.default_rng(500 + BATCHES.index(case))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(off[-1])
    scores = rng.random(max(T, 1)).astype(np.float32) ** 4
    ks = [int(sp.sp_keep_count((L + chunk - 1) // chunk, *keep)) if L > 0 else 0 for L in lens]
    kept = np.concatenate([[0], np.cumsum(ks)]).astype(np.int64)
    K = int(kept[-1])
    doffs, toffs = [], []
    for L in lens:
        d = offsets_from_lengths(rng.integers(1, 9, size=L)) if L > 0 else np.zeros(1, np.int64)
        t = split_same_text(rng, int(d[-1]), 7) if L > 0 else np.zeros(1, np.int64)
        doffs.append(d)
        toffs.append(t)
    Ms = [t.size - 1 for t in toffs]
    moff = np.concatenate([[0], np.cumsum(Ms)]).astype(np.int64)
    MT = int(moff[-1])

    def dev(a, dt):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(DEV)
    sd, off_d, kept_d, moff_d = dev(scores, np.float32), dev(off, np.int64), dev(kept, np.int64), dev(moff, np.int64)
    dd, td = dev(np.concatenate(doffs), np.int64), dev(np.concatenate(toffs), np.int64)
    sel = torch.full((max(K, 1),), -1, dtype=torch.int32, device=DEV)
    spans = torch.full((max(K, 1), 2), -1, dtype=torch.int64, device=DEV)
    n_spans = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    n_cs = T // chunk + B + 1
    cs = torch.full((n_cs,), float("nan"), dtype=torch.float32, device=DEV)
    ws = workspace(sp.sp_select_batch_workspace(T, B, chunk))
    sp.sp_select_batch(sd, [int(v) for v in off], off_d, pool_w, chunk, [int(v) for v in kept], kept_d, sel, spans,
                       n_spans, cs, ws)
    tsp = torch.full((max(K, 1), 2), -1, dtype=torch.int64, device=DEV)
    n_t = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    n_kept = torch.full((B,), -1, dtype=torch.int64, device=DEV)
    mask = torch.full((max(MT, 1),), 7, dtype=torch.uint8, device=DEV)
    sp.sp_project_batch(dd, [int(v) for v in off], off_d, td, [int(v) for v in moff], moff_d, spans, n_spans,
                        [int(v) for v in kept], kept_d, tsp, n_t, mask, n_kept)
    torch.cuda.synchronize()
    sel, spans, n_spans, cs = sel.cpu().numpy(), spans.cpu().numpy(), n_spans.cpu().numpy(), cs.cpu().numpy()
    tsp, n_t, n_kept, mask = tsp.cpu().numpy(), n_t.cpu().numpy(), n_kept.cpu().numpy(), mask.cpu().numpy()
    for b, L in enumerate(lens):
        k0, k1 = int(kept[b]), int(kept[b + 1])
        if L == 0:
            assert n_spans[b] == 0 and n_t[b] == 0 and n_kept[b] == 0
            continue
        s_sel, s_spans, s_cs = gpu_select(scores[off[b]:off[b + 1]], pool_w, chunk, ks[b])
        C = (L + chunk - 1) // chunk
        slot = int(off[b]) // chunk + b
        assert cs[slot:slot + C].tobytes() == s_cs.tobytes()
        np.testing.assert_array_equal(sel[k0:k1], s_sel)
        ns = int(n_spans[b])
        np.testing.assert_array_equal(spans[k0:k0 + ns], s_spans)
        assert (spans[k0 + ns:k1] == -1).all()
        exact = oracle.topk(s_cs.astype(np.float64), ks[b])
        np.testing.assert_array_equal(sel[k0:k1].astype(np.int64), exact)
        np.testing.assert_array_equal(spans[k0:k0 + ns], oracle.merge(exact, chunk, L))
        o_ts, o_mask, o_n = oracle.project(doffs[b], toffs[b], spans[k0:k0 + ns])
        nt = int(n_t[b])
        np.testing.assert_array_equal(tsp[k0:k0 + nt], o_ts)
        assert (tsp[k0 + nt:k1] == -1).all()
        np.testing.assert_array_equal(mask[moff[b]:moff[b + 1]], o_mask)
        assert n_kept[b] == o_n
    if K:
        assert (sel[K:] == -1).all()
    # without the optional outputs: same selections
    sel2 = torch.full((max(K, 1),), -1, dtype=torch.int32, device=DEV)
    spans2 = torch.full((max(K, 1), 2), -1, dtype=torch.int64, device=DEV)
    n_spans2 = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    sp.sp_select_batch(sd, [int(v) for v in off], off_d, pool_w, chunk, [int(v) for v in kept], kept_d, sel2, spans2,
                       n_spans2, None, ws)
    n_kept2 = torch.full((B,), -1, dtype=torch.int64, device=DEV)
    tsp2 = torch.full((max(K, 1), 2), -1, dtype=torch.int64, device=DEV)
    n_t2 = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    sp.sp_project_batch(dd, [int(v) for v in off], off_d, td, [int(v) for v in moff], moff_d, spans2, n_spans2,
                        [int(v) for v in kept], kept_d, tsp2, n_t2, None, n_kept2)
    torch.cuda.synchronize()
    assert sel2.cpu().numpy().tobytes() == sel.tobytes() and spans2.cpu().numpy().tobytes() == spans.tobytes()
    assert tsp2.cpu().numpy().tobytes() == tsp.tobytes() and n_kept2.cpu().numpy().tobytes() == n_kept.tobytes()
