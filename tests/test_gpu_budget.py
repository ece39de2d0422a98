"""GPU parity of sp_select_budget (chunk selection for a fixed target-side
length, Section 3.1) against the CPU oracle. Everything after the fp32 chunk
scores is integer work, so the comparison is exact: the oracle's plain search
(every k tried with top-k, merge and projection) runs on the GPU's own chunk
scores, the same precision on both sides of every decision."""
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


def offsets_from_lengths(lens):
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)


def split_same_text(rng, total, max_len, allow_zero=False):
    cuts = [0]
    while cuts[-1] < total:
        cuts.append(min(total, cuts[-1] + int(rng.integers(0 if allow_zero else 1, max_len + 1))))
    return np.array(cuts, dtype=np.int64)


def check_budget(scores32, pool_w, chunk, doff, toff, budget):
    from gpu_util import gpu_project, gpu_select_budget
    L = scores32.size
    k, n_kept, sel, spans, cs = gpu_select_budget(scores32, pool_w, chunk, doff, toff, budget)
    o_cs = oracle.chunk_mean(oracle.pool(scores32.astype(np.float64), pool_w), chunk)
    np.testing.assert_allclose(cs.astype(np.float64), o_cs, rtol=1e-3, atol=1e-30)
    want_k, want_kept = oracle.budget_keep(cs.astype(np.float64), chunk, doff, toff, budget)
    assert (k, n_kept) == (want_k, want_kept), (budget, k, n_kept, want_k, want_kept)
    exact = oracle.topk(cs.astype(np.float64), k)
    np.testing.assert_array_equal(sel.astype(np.int64), exact)
    np.testing.assert_array_equal(spans, oracle.merge(exact, chunk, L))
    # the reported count is what the projection of the written spans keeps, on both sides
    assert oracle.project(doff, toff, spans)[2] == n_kept
    assert gpu_project(doff, toff, spans)[2] == n_kept
    return k, n_kept


def test_budget_small_random_cases_with_exact_ties():
    say("[budget] small random cases")
    rng = np.random.default_rng(51)
    for trial in range(25):
        L = int(rng.integers(3, 300))
        chunk = int(rng.integers(1, 9))
        doff = offsets_from_lengths(rng.integers(1, 7, size=L))
        toff = split_same_text(rng, int(doff[-1]), 9)
        M = toff.size - 1
        scores = rng.integers(0, 5, size=L).astype(np.float32)        # many equal chunk scores
        for budget in (0, 1, M // 4, M // 2, M - 1, M, M + 7):
            check_budget(scores, 1, chunk, doff, toff, budget)


def test_budget_tokens_and_chunks_without_characters():
    """Offsets that are only non-decreasing: target tokens without characters (kept only strictly
    inside a merged span) and whole chunks without characters."""
    say("[budget] zero-length tokens and chunks")
    rng = np.random.default_rng(52)
    for trial in range(40):
        L = int(rng.integers(2, 120))
        chunk = int(rng.integers(1, 5))
        lens = rng.integers(0, 4, size=L)
        if trial % 3 == 0:                                            # runs of empty draft tokens: empty chunks
            lens[rng.integers(0, L):][: 3 * chunk] = 0
        doff = offsets_from_lengths(lens)
        if doff[-1] == 0:
            doff[-1] = 1
        toff = split_same_text(rng, int(doff[-1]), 3, allow_zero=True)
        M = toff.size - 1
        scores = rng.integers(0, 4, size=L).astype(np.float32)
        for budget in (0, M // 3, (2 * M) // 3, M):
            check_budget(scores, 3, chunk, doff, toff, budget)


@pytest.mark.parametrize("name", ["tiny", "llama1b-8k"])
def test_budget_workload_char_models(name):
    w = synth.get_config(name)
    doff, toff = synth.gen_char_offsets(w, w.L)
    M = toff.size - 1
    rng = np.random.default_rng(w.cfg_id)
    scores = rng.random(w.L).astype(np.float32)
    for budget in (M // 8, M // 4, M // 2):
        k, kept = check_budget(scores, w.pool, w.chunk, doff, toff, budget)
        say(f"[budget] {name}: budget {budget} of {M} -> k = {k}, kept {kept}")
        assert budget - 3 * w.chunk <= kept <= budget                  # lands just under the budget


@pytest.mark.timeout(300)
def test_budget_full_size_benchmark_workload():
    """The 128K-token workload with 8k / 16k target-token budgets. The plain search would take C
    full projections; instead the two facts that define the answer are checked with the oracle:
    the chosen k keeps at most the budget and k + 1 keeps more (more chunks never keep fewer)."""
    from gpu_util import gpu_select_budget
    w = synth.get_config("long-128k")
    doff, toff = synth.gen_char_offsets(w, w.L)
    M = toff.size - 1
    rng = np.random.default_rng(w.cfg_id)
    scores = rng.random(w.L).astype(np.float32)
    C = (w.L + w.chunk - 1) // w.chunk
    for budget in (8192, 16384):
        k, n_kept, sel, spans, cs = gpu_select_budget(scores, w.pool, w.chunk, doff, toff, budget)
        cs64 = cs.astype(np.float64)
        exact = oracle.topk(cs64, k)
        np.testing.assert_array_equal(sel.astype(np.int64), exact)
        np.testing.assert_array_equal(spans, oracle.merge(exact, w.chunk, w.L))
        assert oracle.project(doff, toff, spans)[2] == n_kept <= budget
        assert k < C
        more = oracle.project(doff, toff, oracle.merge(oracle.topk(cs64, k + 1), w.chunk, w.L))[2]
        assert more > budget
        say(f"[budget] {w.name}: budget {budget} of {M} -> k = {k} of {C}, kept {n_kept}; k + 1 keeps {more}")
