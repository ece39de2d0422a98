"""Pins of the CPU oracle against what the paper and the mathematics fix.

The paper prints no worked numerical example for the token-importance pass
(Appendix A.1 describes it in words; Appendix A.3 gives only the
hyper-parameters), so every function of the oracle is pinned here by closed
forms, invariants, library routines (numpy / scipy) on special cases, and brute
force on tiny inputs. Each test names the mistake it is meant to catch.
"""
from __future__ import annotations

import itertools
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle
import synth
from synth import bf16_bits_to_f32, f32_to_bf16_bits


def bits(x):
    return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def rand_small_ints(rng, shape, lo=-3, hi=3):
    """Small integers: exactly representable in bf16, sums exact in float64."""
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)


def make_qk(rng, Lyr, H, Hkv, n_q, d, L, q_scale=0.25):
    q = rand_small_ints(rng, (Lyr, H, n_q, d)) * np.float32(q_scale)
    k = [rand_small_ints(rng, (Hkv, L, d)) for _ in range(Lyr)]
    return q, k


# --------------------------------------------------------------------------
# softmax / logits  (Appendix A.1.1)
# --------------------------------------------------------------------------

def test_softmax_rows_sum_to_one_and_stats():
    """O1: every probability row sums to 1; returned (max, sum) are the row's own."""
    rng = np.random.default_rng(1)
    s = rng.normal(size=(5, 7, 301)) * 6.0
    p, m, l = oracle.softmax_rows(s, return_stats=True)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(m, s.max(-1))
    np.testing.assert_allclose(l, np.exp(s - m[..., None]).sum(-1), rtol=1e-13)
    assert (p > 0).all()


def test_single_row_equals_library_softmax_of_matmul():
    """O8: with one layer, one head, one lookahead row the importance vector is a
    softmax row; it must equal scipy's float64 softmax of numpy's matmul.
    Catches a wrong scale, a transposed operand, a wrong stride."""
    rng = np.random.default_rng(2)
    d, L = 64, 257
    qf = rng.standard_normal((1, 1, 1, d)).astype(np.float32)
    kf = rng.standard_normal((1, L, d)).astype(np.float32)
    qb, kb = bits(qf), bits(kf)
    scale = 0.125
    I = oracle.score(qb, [kb], scale, oracle.LAYER_MAX)
    ref = scipy.special.softmax(scale * (bf16_bits_to_f32(kb[0]).astype(np.float64)
                                         @ bf16_bits_to_f32(qb[0, 0, 0]).astype(np.float64)))
    np.testing.assert_allclose(I, ref, rtol=1e-12, atol=0)
    I2 = oracle.score(qb, [kb], scale, oracle.LAYER_MEAN)
    np.testing.assert_allclose(I2, ref, rtol=1e-12, atol=0)
    # token-major layout of the same keys gives the same result (stride handling)
    k_nhd = np.ascontiguousarray(kb.transpose(1, 0, 2))
    np.testing.assert_allclose(oracle.score(qb, [k_nhd], scale, 0, layout="NHD"), ref, rtol=1e-12)


def test_logits_match_library_contraction_with_gqa_groups():
    """Logits of a multi-head GQA layer against numpy einsum per kv group.
    Catches a wrong head -> kv-head mapping and index mix-ups."""
    rng = np.random.default_rng(3)
    H, Hkv, n_q, d, L = 6, 3, 4, 32, 50
    qf, kf = make_qk(rng, 1, H, Hkv, n_q, d, L)
    s = oracle.logits_layer(bits(qf[0]), bits(kf[0]), 0.3)
    G = H // Hkv
    q64 = bf16_bits_to_f32(bits(qf[0])).astype(np.float64)
    k64 = bf16_bits_to_f32(bits(kf[0])).astype(np.float64)
    ref = np.stack([0.3 * np.einsum("ne,je->nj", q64[h], k64[h // G]) for h in range(H)])
    np.testing.assert_allclose(s, ref, rtol=1e-13, atol=1e-13)


def test_uniform_keys_give_uniform_scores_and_lowest_index_selection():
    """O2: identical keys (or all-zero K) give I[j] = 1/L in both modes; the pooled
    interior equals 1/L; tied chunk scores select the lowest indices."""
    rng = np.random.default_rng(4)
    Lyr, H, Hkv, n_q, d, L = 3, 4, 2, 5, 16, 416
    qf, _ = make_qk(rng, Lyr, H, Hkv, n_q, d, L)
    krow = rand_small_ints(rng, (Hkv, 1, d))
    for kf in ([np.repeat(krow, L, axis=1)] * Lyr, [np.zeros((Hkv, L, d), np.float32)] * Lyr):
        for mode in (oracle.LAYER_MEAN, oracle.LAYER_MAX):
            I = oracle.score(bits(qf), [bits(k) for k in kf], 0.25, mode)
            np.testing.assert_allclose(I, 1.0 / L, rtol=1e-12)
    I = np.full(L, 1.0 / L)
    P = oracle.pool(I, 13)
    np.testing.assert_allclose(P[6:L - 6], 1.0 / L, rtol=1e-13)
    # interior chunks (those not touching the 6-token edges) tie exactly when
    # the input is a constant whose window sum is exact: use a power of two.
    I2 = np.full(L, 2.0 ** -9)
    sel, spans, cs = oracle.select(I2, 13, 32, 4)
    C = L // 32
    assert np.all(cs[1:C - 1] == cs[1])
    assert cs[0] < cs[1] and cs[C - 1] < cs[1]
    np.testing.assert_array_equal(sel, [1, 2, 3, 4])
    np.testing.assert_array_equal(spans, [[32, 160]])


def test_single_dominant_key_closed_form():
    """O3: K = 0 except one position j*: p(j*) = e^a / (e^a + L - 1), others
    1 / (e^a + L - 1), a = scale * q.k*. A large a lets the key capture the score."""
    d, L, jstar = 16, 100, 37
    q = np.zeros((1, 1, 1, d), np.float32)
    q[..., :4] = [1.0, -2.0, 0.5, 3.0]
    k = np.zeros((1, L, d), np.float32)
    k[0, jstar, :4] = [2.0, -1.0, 4.0, 1.0]
    scale = 0.5
    a = scale * (2.0 + 2.0 + 2.0 + 3.0)
    I = oracle.score(bits(q), [bits(k)], scale, oracle.LAYER_MAX)
    den = np.exp(a) + L - 1
    expect = np.full(L, 1.0 / den)
    expect[jstar] = np.exp(a) / den
    np.testing.assert_allclose(I, expect, rtol=1e-13)
    k[0, jstar, :4] *= 16.0      # a -> 72: the key takes all the mass
    I = oracle.score(bits(q), [bits(k)], scale, oracle.LAYER_MAX)
    assert 1.0 - 1e-15 <= I[jstar] <= 1.0
    assert np.delete(I, jstar).max() < 1e-29


def test_two_level_keys_closed_form_with_head_max():
    """O4: keys take two values; with two heads attending oppositely the max over
    heads has a closed form. Catches a max taken before the normalisation."""
    d, L, n1 = 8, 60, 20
    q = np.zeros((1, 2, 1, d), np.float32)
    q[0, 0, 0, 0] = 2.0       # head 0 likes key type A
    q[0, 1, 0, 1] = 1.0       # head 1 likes key type B
    k = np.zeros((1, L, d), np.float32)
    k[0, :n1, 0] = 1.5        # type A: first n1 keys
    k[0, n1:, 1] = 2.0        # type B
    I = oracle.score(bits(q), [bits(k)], 1.0, oracle.LAYER_MAX)   # H=2, Hkv=1
    a, b = 3.0, 2.0
    pA0 = np.exp(a) / (n1 * np.exp(a) + (L - n1))      # head 0 on type A
    pB0 = 1.0 / (n1 * np.exp(a) + (L - n1))
    pA1 = 1.0 / (n1 + (L - n1) * np.exp(b))            # head 1 on type A
    pB1 = np.exp(b) / (n1 + (L - n1) * np.exp(b))
    expect = np.concatenate([np.full(n1, max(pA0, pA1)), np.full(L - n1, max(pB0, pB1))])
    np.testing.assert_allclose(I, expect, rtol=1e-13)
    assert pA0 > pA1 and pB1 > pB0      # the max really switches head


def test_shift_invariance_large_offset():
    """O5: adding one vector to every key shifts each row's logits by a constant
    and must not change the scores, even when the shift is huge (max-subtraction)."""
    rng = np.random.default_rng(5)
    Lyr, H, Hkv, n_q, d, L = 2, 4, 2, 3, 16, 90
    qf, kf = make_qk(rng, Lyr, H, Hkv, n_q, d, L, q_scale=1.0)
    v = rng.choice([-64.0, 64.0], size=(1, 1, d)).astype(np.float32)   # |k+v| <= 67: exact in bf16
    base = oracle.score(bits(qf), [bits(k) for k in kf], 1.0, oracle.LAYER_MEAN)
    shifted = oracle.score(bits(qf), [bits(k + v) for k in kf], 1.0, oracle.LAYER_MEAN)
    assert np.isfinite(shifted).all()
    np.testing.assert_allclose(shifted, base, rtol=1e-10)


def test_key_permutation_permutes_scores():
    """O6."""
    rng = np.random.default_rng(6)
    Lyr, H, Hkv, n_q, d, L = 2, 4, 2, 3, 16, 77
    qf, kf = make_qk(rng, Lyr, H, Hkv, n_q, d, L)
    perm = rng.permutation(L)
    for mode in (0, 1):
        a = oracle.score(bits(qf), [bits(k) for k in kf], 0.25, mode)
        b = oracle.score(bits(qf), [bits(k[:, perm]) for k in kf], 0.25, mode)
        np.testing.assert_allclose(b, a[perm], rtol=1e-12)


def test_gqa_equals_replicated_kv_heads():
    """O7: query head h reads kv head h // G. Replicating each kv head G times and
    running as multi-head attention gives the same scores."""
    rng = np.random.default_rng(7)
    Lyr, H, Hkv, n_q, d, L = 2, 8, 2, 3, 16, 64
    G = H // Hkv
    qf, kf = make_qk(rng, Lyr, H, Hkv, n_q, d, L)
    rep = [np.repeat(k, G, axis=0) for k in kf]
    for mode in (0, 1):
        a = oracle.score(bits(qf), [bits(k) for k in kf], 0.25, mode)
        b = oracle.score(bits(qf), [bits(k) for k in rep], 0.25, mode)
        np.testing.assert_allclose(a, b, rtol=1e-13)
    # and the mapping is not h % Hkv: interleaving the replicas must change it
    wrong = [np.tile(k, (G, 1, 1)) for k in kf]
    c = oracle.score(bits(qf), [bits(k) for k in wrong], 0.25, 0)
    assert np.abs(c - a).max() > 1e-6


def test_head_max_identity_via_logsumexp():
    """O9: max_h softmax_h(s)[j] = exp(max_h (s_h[j] - lse_h)); checked through the
    oracle's own logits and row statistics against its aggregated score."""
    rng = np.random.default_rng(8)
    H, Hkv, n_q, d, L = 4, 2, 3, 16, 120
    qf, kf = make_qk(rng, 1, H, Hkv, n_q, d, L)
    s = oracle.logits_layer(bits(qf[0]), bits(kf[0]), 0.25)
    lse = scipy.special.logsumexp(s, axis=-1)
    via_lse = np.exp((s - lse[..., None]).max(axis=0)).mean(axis=0)
    I = oracle.score(bits(qf), [bits(kf[0])], 0.25, oracle.LAYER_MAX)
    np.testing.assert_allclose(I, via_lse, rtol=1e-12)


def test_aggregation_modes_definition_and_bounds():
    """O10 and the two aggregation modes written out with numpy on the oracle's
    probabilities: mean mode averages the per-layer head-max over layers and
    lookahead rows; max mode takes the max over layers too. Bounds: 0 < I <= 1,
    1 <= sum I <= H (mean) or H*Lyr (max), I_max >= I_mean, and duplicating a
    layer changes neither mode."""
    rng = np.random.default_rng(9)
    Lyr, H, Hkv, n_q, d, L = 3, 4, 2, 5, 16, 150
    qf, kf = make_qk(rng, Lyr, H, Hkv, n_q, d, L)
    qb, kb = bits(qf), [bits(k) for k in kf]
    p = np.stack([oracle.softmax_rows(oracle.logits_layer(qb[l], kb[l], 0.25)) for l in range(Lyr)])
    head_max = p.max(axis=1)                     # p is [Lyr][H][n_q][L] -> [Lyr][n_q][L]
    mean_ref = head_max.mean(axis=(0, 1))
    max_ref = head_max.max(axis=0).mean(axis=0)
    I_mean = oracle.score(qb, kb, 0.25, oracle.LAYER_MEAN)
    I_max = oracle.score(qb, kb, 0.25, oracle.LAYER_MAX)
    np.testing.assert_allclose(I_mean, mean_ref, rtol=1e-13)
    np.testing.assert_allclose(I_max, max_ref, rtol=1e-13)
    assert (I_mean > 0).all() and (I_max <= 1).all()
    assert 1 - 1e-12 <= I_mean.sum() <= H + 1e-12
    assert 1 - 1e-12 <= I_max.sum() <= H * Lyr + 1e-12
    assert (I_max >= I_mean - 1e-15).all()
    q2 = np.concatenate([qb, qb[-1:]], axis=0)
    k2 = kb + [kb[-1]]
    np.testing.assert_allclose(oracle.score(q2, k2, 0.25, 1), I_max, rtol=1e-13)
    # duplicating a layer leaves the max mode alone and re-weights the mean mode
    dup_mean = (head_max.sum(axis=0) + head_max[-1]).mean(axis=0) / (Lyr + 1)
    np.testing.assert_allclose(oracle.score(q2, k2, 0.25, 0), dup_mean, rtol=1e-13)
    # duplicating every layer changes neither mode
    q3, k3 = np.concatenate([qb, qb], axis=0), kb + kb
    np.testing.assert_allclose(oracle.score(q3, k3, 0.25, 0), I_mean, rtol=1e-13)
    np.testing.assert_allclose(oracle.score(q3, k3, 0.25, 1), I_max, rtol=1e-13)


def test_split_row_statistics_merge_by_logsumexp():
    """O11: statistics (m, l) of two halves of a row merged by log-sum-exp equal
    those of the whole row: the identity a split-L streaming pass relies on."""
    rng = np.random.default_rng(10)
    s = rng.normal(size=(6, 400)) * 8
    _, m, l = oracle.softmax_rows(s, return_stats=True)
    _, m1, l1 = oracle.softmax_rows(s[:, :123], return_stats=True)
    _, m2, l2 = oracle.softmax_rows(s[:, 123:], return_stats=True)
    M = np.maximum(m1, m2)
    np.testing.assert_array_equal(M, m)
    np.testing.assert_allclose(l1 * np.exp(m1 - M) + l2 * np.exp(m2 - M), l, rtol=1e-13)


def test_scale_is_applied_inside_the_exponent():
    """Doubling the scale equals doubling the queries (a power of two is exact in
    bf16). Catches a scale applied after the softmax or dropped."""
    rng = np.random.default_rng(11)
    qf, kf = make_qk(rng, 2, 4, 2, 3, 16, 70)
    a = oracle.score(bits(qf * 2), [bits(k) for k in kf], 0.125, 0)
    b = oracle.score(bits(qf), [bits(k) for k in kf], 0.25, 0)
    np.testing.assert_allclose(a, b, rtol=1e-13)
    c = oracle.score(bits(qf), [bits(k) for k in kf], 0.125, 0)
    assert np.abs(c - b).max() > 1e-6



def test_gather_pages_against_explicit_loops():
    """Paged keys (Section 3.1, KV blocks): token j is row j % P of page table[j // P]. The gather is
    checked element by element with plain loops, in both page layouts, with a ragged last page."""
    rng = np.random.default_rng(35)
    Hkv, P, d, L = 2, 4, 3, 10
    pool_hnd = rng.integers(0, 60000, size=(5, Hkv, P, d)).astype(np.uint16)
    table = np.array([3, 0, 4])
    got = oracle.gather_pages(pool_hnd, table, L, "HND")
    assert got.shape == (Hkv, L, d)
    for kv in range(Hkv):
        for j in range(L):
            for e in range(d):
                assert got[kv, j, e] == pool_hnd[table[j // P], kv, j % P, e]
    pool_nhd = np.ascontiguousarray(pool_hnd.transpose(0, 2, 1, 3))
    got2 = oracle.gather_pages(pool_nhd, table, L, "NHD")
    np.testing.assert_array_equal(got2, got.transpose(1, 0, 2))


# --------------------------------------------------------------------------
# lookahead keys in the normaliser  (Algorithm 1, ForwardWithAttn with lookahead = i)
# --------------------------------------------------------------------------

def test_look_zero_queries_closed_form_counts_visible_keys():
    """All logits 0: row n is uniform over L + (n + look_self) keys, so
    I[j] = mean_n 1 / (L + n + look_self) in both modes. Catches an off-by-one in
    the visible count and a look_self flag that does nothing."""
    Lyr, H, Hkv, n_q, d, L = 2, 4, 2, 5, 16, 37
    qb = bits(np.zeros((Lyr, H, n_q, d), np.float32))
    rng = np.random.default_rng(31)
    kb = [bits(rand_small_ints(rng, (Hkv, L, d))) for _ in range(Lyr)]
    kl = bits(rand_small_ints(rng, (Lyr, Hkv, n_q, d)))
    for look_self in (0, 1):
        want = float(np.mean([Fraction(1, L + n + look_self) for n in range(n_q)]))
        for mode in (oracle.LAYER_MEAN, oracle.LAYER_MAX):
            I = oracle.score_look(qb, kb, kl, look_self, 0.25, mode)
            np.testing.assert_allclose(I, want, rtol=1e-14)


def test_look_equals_plain_score_on_concatenated_keys_row_by_row():
    """Row n normalised over prompt + visible lookahead keys is the plain softmax of
    the prompt with those keys appended as extra tokens. Per lookahead row the
    pinned plain path scores that row alone (n_q = 1) against the concatenation;
    the mean over rows must equal the lookahead variant. Catches a wrong kv head,
    a transposed lookahead operand, a causal mask off by one, a dropped term."""
    rng = np.random.default_rng(32)
    Lyr, H, Hkv, n_q, d, L = 3, 4, 2, 4, 16, 83
    qf, kf = make_qk(rng, Lyr, H, Hkv, n_q, d, L)
    klf = rand_small_ints(rng, (Lyr, Hkv, n_q, d))
    qb, kb, kl = bits(qf), [bits(k) for k in kf], bits(klf)
    for look_self in (0, 1):
        for mode in (oracle.LAYER_MEAN, oracle.LAYER_MAX):
            rows = []
            for n in range(n_q):
                vis = min(n + look_self, n_q)
                cat = [np.concatenate([kb[l], kl[l][:, :vis, :]], axis=1) for l in range(Lyr)]
                rows.append(oracle.score(qb[:, :, n:n + 1, :], cat, 0.25, mode)[:L])
            got = oracle.score_look(qb, kb, kl, look_self, 0.25, mode)
            np.testing.assert_allclose(got, np.mean(rows, axis=0), rtol=1e-12)
            # the lookahead keys take probability mass: strictly below the prompt-only scores
            # (row 0 without look_self sees none, so compare the sum)
            assert got.sum() < oracle.score(qb, kb, 0.25, mode).sum()


def test_look_single_row_library_softmax_and_token_major_layout():
    """One layer, one head, two lookahead rows, look_self = 1: each row is scipy's
    softmax of [prompt logits, visible lookahead logits]; also through the
    token-major K layout."""
    rng = np.random.default_rng(33)
    d, L = 32, 61
    qf = rng.standard_normal((1, 1, 2, d)).astype(np.float32)
    kf = rng.standard_normal((1, L, d)).astype(np.float32)
    klf = rng.standard_normal((1, 1, 2, d)).astype(np.float32)
    qb, kb, kl = bits(qf), bits(kf), bits(klf)
    Q = bf16_bits_to_f32(qb[0, 0]).astype(np.float64)
    K = bf16_bits_to_f32(kb[0]).astype(np.float64)
    KL = bf16_bits_to_f32(kl[0, 0]).astype(np.float64)
    scale = 0.2
    ref = np.zeros(L)
    for n in range(2):
        row = np.concatenate([K @ Q[n], KL[:n + 1] @ Q[n]]) * scale
        ref += scipy.special.softmax(row)[:L] / 2
    np.testing.assert_allclose(oracle.score_look(qb, [kb], kl, 1, scale, oracle.LAYER_MAX), ref, rtol=1e-12)
    k_nhd = np.ascontiguousarray(kb.transpose(1, 0, 2))
    np.testing.assert_allclose(oracle.score_look(qb, [k_nhd], kl, 1, scale, 0, layout="NHD"), ref, rtol=1e-12)


# --------------------------------------------------------------------------
# pooling and chunk means  (Algorithm 1, Appendix A.1.2, Appendix A.3)
# --------------------------------------------------------------------------

def test_pool_impulse_and_textbook_convolution():
    """O12: an interior unit impulse spreads to w entries of 1/w; near the edge it
    is truncated; the pool equals numpy's 'same' convolution with ones(w)/w."""
    L, w = 50, 13
    x = np.zeros(L)
    x[20] = 1.0
    P = oracle.pool(x, w)
    expect = np.zeros(L)
    expect[14:27] = 1.0 / 13
    np.testing.assert_allclose(P, expect, rtol=1e-15, atol=0)
    x = np.zeros(L)
    x[2] = 1.0
    P = oracle.pool(x, w)
    expect = np.zeros(L)
    expect[0:9] = 1.0 / 13
    np.testing.assert_allclose(P, expect, rtol=1e-15, atol=0)
    rng = np.random.default_rng(12)
    for L, w in ((50, 13), (7, 13), (1, 13), (33, 1), (40, 5)):
        x = rng.random(L)
        np.testing.assert_allclose(oracle.pool(x, w), np.convolve(x, np.ones(w) / w, mode="same")[:L]
                                   if L >= w else
                                   np.array([x[max(0, j - w // 2): j + w // 2 + 1].sum() / w for j in range(L)]),
                                   rtol=1e-13)
    a, b = rng.random(64), rng.random(64)
    np.testing.assert_allclose(oracle.pool(2 * a - 3 * b, 13), 2 * oracle.pool(a, 13) - 3 * oracle.pool(b, 13),
                               rtol=1e-12, atol=1e-15)
    with pytest.raises(ValueError):
        oracle.pool(a, 12)


def test_pool_mass_closed_form():
    """O13: the divisor is always w, so sum(pool) = (1/w) sum_j cnt(j) I[j] with
    cnt(j) the number of windows covering j; the mean is preserved exactly when
    the outer (w-1)/2 entries on each side are zero."""
    rng = np.random.default_rng(13)
    L, w = 200, 13
    h = (w - 1) // 2
    x = rng.random(L)
    j = np.arange(L)
    cnt = np.minimum(j + h, L - 1) - np.maximum(j - h, 0) + 1
    np.testing.assert_allclose(oracle.pool(x, w).sum(), (cnt * x).sum() / w, rtol=1e-13)
    x[:h] = 0
    x[L - h:] = 0
    np.testing.assert_allclose(oracle.pool(x, w).mean(), x.mean(), rtol=1e-13)
    c = np.full(L, 0.37)
    np.testing.assert_allclose(oracle.pool(c, w)[h:L - h], 0.37, rtol=1e-14)


def test_chunk_mean_mass_and_short_last_chunk():
    """O14: sum_i size_i * cs[i] = sum_j P[j]; the short last chunk divides by its
    own size; matches numpy's reshape-mean when c divides L."""
    rng = np.random.default_rng(14)
    P = rng.random(100)
    cs = oracle.chunk_mean(P, 32)
    assert cs.size == 4
    sizes = np.array([32, 32, 32, 4])
    np.testing.assert_allclose((sizes * cs).sum(), P.sum(), rtol=1e-13)
    np.testing.assert_allclose(cs[3], P[96:].mean(), rtol=1e-14)
    np.testing.assert_allclose(oracle.chunk_mean(P[:96], 32), P[:96].reshape(3, 32).mean(1), rtol=1e-14)
    np.testing.assert_allclose(oracle.chunk_mean(P, 1), P, rtol=0)
    np.testing.assert_allclose(oracle.chunk_mean(P, 1000), [P.mean()], rtol=1e-14)


def test_pool_then_chunk_exact_rationals():
    """A hand-checkable case in exact rational arithmetic: I = 0..11, w = 3, c = 5."""
    I = [Fraction(v) for v in range(12)]
    pooled = []
    for j in range(12):
        lo, hi = max(0, j - 1), min(11, j + 1)
        pooled.append(sum(I[lo:hi + 1]) / 3)
    cs = [sum(pooled[0:5]) / 5, sum(pooled[5:10]) / 5, sum(pooled[10:12]) / 2]
    got_p = oracle.pool(np.arange(12.0), 3)
    got_c = oracle.chunk_mean(got_p, 5)
    np.testing.assert_allclose(got_p, [float(v) for v in pooled], rtol=1e-15)
    np.testing.assert_allclose(got_c, [float(v) for v in cs], rtol=1e-15)
    assert pooled[0] == Fraction(1, 3) and pooled[11] == Fraction(21, 3) and pooled[5] == 5


# --------------------------------------------------------------------------
# top-k, merge, keep count  (Algorithm 1; Sections 3.1, 3.2)
# --------------------------------------------------------------------------

def brute_force_topk(cs, k):
    """The k-subset with the largest total; among equal totals the one whose sorted
    index tuple is lexicographically smallest (lower index wins a tie)."""
    best, best_sum = None, None
    for comb in itertools.combinations(range(len(cs)), k):
        tot = sum(Fraction(float(cs[i])) for i in comb)
        if best is None or tot > best_sum:          # combinations come in lexicographic order
            best, best_sum = comb, tot
    return np.array(best, dtype=np.int64)


def test_topk_equals_brute_force_on_tiny_inputs():
    """O15, O16."""
    rng = np.random.default_rng(15)
    for trial in range(40):
        C = int(rng.integers(1, 11))
        if trial % 2:
            cs = rng.integers(0, 4, size=C).astype(np.float64)      # many exact ties
        else:
            cs = rng.random(C)
        for k in range(1, C + 1):
            np.testing.assert_array_equal(oracle.topk(cs, k), brute_force_topk(cs, k))
    cs = np.array([1.0, 5.0, 5.0, 2.0, 5.0])
    np.testing.assert_array_equal(oracle.topk(cs, 1), [1])
    np.testing.assert_array_equal(oracle.topk(cs, 2), [1, 2])
    np.testing.assert_array_equal(oracle.topk(cs, 5), [0, 1, 2, 3, 4])
    with pytest.raises(ValueError):
        oracle.topk(cs, 0)
    with pytest.raises(ValueError):
        oracle.topk(cs, 6)


def test_merge_spans_invariants():
    """O17: spans sorted, disjoint, non-adjacent, total length = kept chunk sizes,
    boundaries multiples of c or L."""
    rng = np.random.default_rng(16)
    for _ in range(50):
        L = int(rng.integers(1, 400))
        c = int(rng.integers(1, 40))
        C = (L + c - 1) // c
        k = int(rng.integers(1, C + 1))
        sel = np.sort(rng.choice(C, size=k, replace=False)).astype(np.int64)
        spans = oracle.merge(sel, c, L)
        assert (spans[:, 0] < spans[:, 1]).all()
        assert (spans[1:, 0] > spans[:-1, 1]).all()
        sizes = np.minimum((sel + 1) * c, L) - sel * c
        assert (spans[:, 1] - spans[:, 0]).sum() == sizes.sum()
        assert all(b % c == 0 for b in spans[:, 0])
        assert all(e % c == 0 or e == L for e in spans[:, 1])
        covered = np.zeros(L, bool)
        for b, e in spans:
            covered[b:e] = True
        expect = np.zeros(L, bool)
        for i in sel:
            expect[i * c:min((i + 1) * c, L)] = True
        np.testing.assert_array_equal(covered, expect)
    np.testing.assert_array_equal(oracle.merge(np.array([0, 1, 3, 4, 5, 9]), 4, 38),
                                  [[0, 8], [12, 24], [36, 38]])


def test_keep_count_table():
    """O22: K = clamp(ceil(C * rho), 1, C) at the five workloads' (C, rho)."""
    table = [(32, 25, 100, 8), (256, 20, 100, 52), (1024, 15, 100, 154), (2048, 10, 100, 205),
             (10, 0, 100, 1), (10, 100, 100, 10), (10, 250, 100, 10), (3, 1, 3, 1), (1, 1, 2, 1)]
    for C, num, den, k in table:
        assert oracle.keep_count(C, num, den) == k


# --------------------------------------------------------------------------
# projection onto the target tokenisation  (Algorithm 1; Section 3.1)
# --------------------------------------------------------------------------

def random_offsets(rng, n, max_len):
    return np.concatenate([[0], np.cumsum(rng.integers(1, max_len + 1, size=n))]).astype(np.int64)


def split_same_text(rng, total, max_len):
    cuts = [0]
    while cuts[-1] < total:
        cuts.append(min(total, cuts[-1] + int(rng.integers(1, max_len + 1))))
    return np.array(cuts, dtype=np.int64)


def random_spans(rng, L):
    n_cut = int(rng.integers(1, 6)) * 2
    pts = np.sort(rng.choice(L + 1, size=min(n_cut, L + 1) // 2 * 2, replace=False))
    return pts.reshape(-1, 2).astype(np.int64)


def test_projection_identity_tokenisation():
    """O18: target tokenisation = draft tokenisation gives target spans = draft spans."""
    rng = np.random.default_rng(17)
    doff = random_offsets(rng, 120, 8)
    spans = np.array([[0, 5], [9, 10], [50, 120]], dtype=np.int64)
    ts, mask, n = oracle.project(doff, doff, spans)
    np.testing.assert_array_equal(ts, spans)
    assert n == 5 + 1 + 70 == mask.sum()


def test_projection_char_level_and_single_token_targets():
    """O19: all-length-1 target tokens keep exactly the kept characters; a single
    target token is kept iff any span exists."""
    rng = np.random.default_rng(18)
    doff = random_offsets(rng, 60, 8)
    total = int(doff[-1])
    chars = np.arange(total + 1, dtype=np.int64)
    spans = np.array([[3, 7], [20, 33]], dtype=np.int64)
    ts, mask, n = oracle.project(doff, chars, spans)
    kept_chars = (doff[7] - doff[3]) + (doff[33] - doff[20])
    assert n == kept_chars
    np.testing.assert_array_equal(ts, [[doff[3], doff[7]], [doff[20], doff[33]]])
    one = np.array([0, total], dtype=np.int64)
    ts, mask, n = oracle.project(doff, one, spans)
    assert n == 1 and ts.tolist() == [[0, 1]]
    ts, mask, n = oracle.project(doff, one, np.zeros((0, 2), np.int64))
    assert n == 0 and ts.shape == (0, 2)


def test_projection_keep_all_and_monotone():
    """O20."""
    rng = np.random.default_rng(19)
    doff = random_offsets(rng, 90, 8)
    toff = split_same_text(rng, int(doff[-1]), 7)
    M = toff.size - 1
    ts, mask, n = oracle.project(doff, toff, np.array([[0, 90]]))
    assert ts.tolist() == [[0, M]] and n == M
    few = np.array([[10, 20]], dtype=np.int64)
    more = np.array([[10, 20], [40, 45]], dtype=np.int64)
    _, m1, _ = oracle.project(doff, toff, few)
    _, m2, _ = oracle.project(doff, toff, more)
    assert ((m2 >= m1).all()) and m2.sum() > m1.sum()


def test_projection_covers_exactly_the_overlapping_tokens():
    """O21: on tiny random splits, the kept set equals the set of target tokens that
    share at least one character with a kept draft token (computed through an
    explicit per-character ownership table, a different route than interval tests),
    and target spans are sorted, disjoint, non-adjacent with total = n_kept."""
    rng = np.random.default_rng(20)
    for _ in range(60):
        L = int(rng.integers(1, 40))
        doff = random_offsets(rng, L, 8)
        total = int(doff[-1])
        toff = split_same_text(rng, total, 7)
        M = toff.size - 1
        spans = random_spans(rng, L)
        spans = spans[spans[:, 0] < spans[:, 1]]
        char_kept = np.zeros(total, bool)
        for a, b in spans:
            char_kept[doff[a]:doff[b]] = True
        owner = np.repeat(np.arange(M), np.diff(toff))        # target token of each char
        expect = np.zeros(M, np.uint8)
        expect[np.unique(owner[char_kept])] = 1
        ts, mask, n = oracle.project(doff, toff, spans)
        np.testing.assert_array_equal(mask, expect)
        assert n == expect.sum() == (ts[:, 1] - ts[:, 0]).sum()
        assert (ts[1:, 0] > ts[:-1, 1]).all()
        rebuilt = np.zeros(M, np.uint8)
        for a, b in ts:
            rebuilt[a:b] = 1
        np.testing.assert_array_equal(rebuilt, expect)


def test_projection_boundary_token_is_kept_once():
    """A target token straddling the gap between two kept spans is kept and bridges
    the two target ranges into one span."""
    doff = np.array([0, 2, 4, 6, 8, 10], dtype=np.int64)
    toff = np.array([0, 3, 7, 10], dtype=np.int64)
    ts, mask, n = oracle.project(doff, toff, np.array([[0, 2], [3, 5]]))  # chars [0,4) and [6,10)
    assert mask.tolist() == [1, 1, 1] and ts.tolist() == [[0, 3]] and n == 3
    ts, mask, n = oracle.project(doff, toff, np.array([[0, 1], [4, 5]]))  # chars [0,2) and [8,10)
    assert mask.tolist() == [1, 0, 1] and ts.tolist() == [[0, 1], [2, 3]] and n == 2
    # touching but not overlapping: span ends exactly at a target boundary
    toff2 = np.array([0, 4, 10], dtype=np.int64)
    ts, mask, n = oracle.project(doff, toff2, np.array([[0, 2]]))         # chars [0,4)
    assert mask.tolist() == [1, 0] and n == 1


# --------------------------------------------------------------------------
# keep rate from a target-side budget (Section 3.1: rho = L_hat_target / L_target, per sample)
# --------------------------------------------------------------------------

def test_keep_rate_from_target_budget_lands_near_the_budget():
    """With rho = L_hat / M applied to the draft chunks, the projected target-side length comes out
    close to L_hat (slightly above: chunk rounding up, and tokens straddling a span boundary)."""
    w = synth.get_config("llama1b-8k")
    doff, toff = synth.gen_char_offsets(w, w.L)
    M = toff.size - 1
    rng = np.random.default_rng(5)
    I = rng.random(w.L)
    C = (w.L + w.chunk - 1) // w.chunk
    for budget in (1024, 2048, 4096):
        k = oracle.keep_count(C, budget, M)
        assert k == -(-C * budget // M)                              # ceil(rho * C) in integers
        _, spans, _ = oracle.select(I, w.pool, w.chunk, k)
        _, _, n_kept = oracle.project(doff, toff, spans)
        assert budget <= n_kept <= budget * 1.08 + 2 * len(spans), (budget, n_kept)
    assert oracle.keep_count(C, 2 * M, M) == C and oracle.keep_count(C, 0, M) == 1   # clamped to [1, C]


def test_budget_keep_worked_example_and_identity_tokenisation():
    """Budget-targeted keep. Hand-worked: 4 one-token chunks of 2 characters, target tokens
    [0,3) [3,5) [5,8), chunk scores .1 .9 .5 .2. Top-1 (chunk 1, chars [2,4)) touches tokens 0 and 1;
    from top-2 on all three tokens are kept. With one-character tokens in both tokenisations and full
    chunks, k chunks keep exactly k*c tokens, so k = floor(budget / c), clamped to [1, C]."""
    doff = np.array([0, 2, 4, 6, 8])
    toff = np.array([0, 3, 5, 8])
    cs = np.array([0.1, 0.9, 0.5, 0.2])
    assert oracle.budget_keep(cs, 1, doff, toff, 2) == (1, 2)
    assert oracle.budget_keep(cs, 1, doff, toff, 3) == (4, 3)      # every k >= 2 keeps 3: the largest wins
    assert oracle.budget_keep(cs, 1, doff, toff, 1) == (1, 2)      # even one chunk exceeds the budget: k = 1
    rng = np.random.default_rng(41)
    c, C = 8, 12
    off = np.arange(c * C + 1)
    cs = rng.random(C)
    for budget in (0, 7, 8, 9, 31, 32, 95, 96, 1000):
        k, kept = oracle.budget_keep(cs, c, off, off, budget)
        assert k == min(C, max(1, budget // c)) and kept == k * c


def test_budget_keep_against_character_coverage_brute_force():
    """Tiny random tokenisations: per k, the chunks are ranked with Python's sort (score descending,
    index ascending), the characters of the first k chunks are put in a set, and a target token counts
    as kept iff one of its characters is in it; the answer is the largest k within the budget.
    Independent of the oracle's own top-k, merge and projection."""
    rng = np.random.default_rng(42)
    for trial in range(30):
        L = int(rng.integers(5, 40))
        c = int(rng.integers(1, 6))
        dlen = rng.integers(1, 6, size=L)
        doff = np.concatenate([[0], np.cumsum(dlen)])
        total = int(doff[-1])
        cuts = np.sort(rng.choice(np.arange(1, total), size=int(rng.integers(1, max(2, total // 3))), replace=False))
        toff = np.concatenate([[0], cuts, [total]])
        C = -(-L // c)
        cs = rng.integers(0, 4, size=C).astype(np.float64)          # many exact ties
        order = sorted(range(C), key=lambda j: (-cs[j], j))
        kept_at = []
        for k in range(1, C + 1):
            chars = set()
            for j in order[:k]:
                chars.update(range(int(doff[j * c]), int(doff[min((j + 1) * c, L)])))
            kept_at.append(sum(1 for t in range(toff.size - 1)
                               if any(x in chars for x in range(int(toff[t]), int(toff[t + 1])))))
        assert kept_at == sorted(kept_at)                           # more chunks never keep fewer tokens
        for budget in (0, kept_at[0], kept_at[C // 2], kept_at[C // 2] - 1, kept_at[-1], kept_at[-1] + 5):
            within = [k for k in range(1, C + 1) if kept_at[k - 1] <= budget]
            want_k = max(within) if within else 1
            assert oracle.budget_keep(cs, c, doff, toff, budget) == (want_k, kept_at[want_k - 1]), (trial, budget)


# --------------------------------------------------------------------------
# compressed-prompt assembly (Algorithm 1: ConcatWithDelim, new position ids; Section 3.2)
# --------------------------------------------------------------------------

def test_assemble_worked_example_and_special_cases():
    ids = np.arange(100, 120, dtype=np.int32)
    out, pos, src = oracle.assemble(ids, np.array([[2, 5], [9, 11], [19, 20]]), np.array([7, 8]))
    assert out.tolist() == [102, 103, 104, 7, 8, 109, 110, 7, 8, 119]          # written out by hand
    assert pos.tolist() == list(range(10))                                      # contiguous position ids
    assert src.tolist() == [2, 3, 4, -1, -1, 9, 10, -1, -1, 19]
    # keep-all: the prompt itself, no delimiter anywhere
    out, pos, src = oracle.assemble(ids, np.array([[0, 20]]), np.array([7, 8]))
    assert out.tolist() == ids.tolist() and src.tolist() == list(range(20))
    # nothing kept; empty delimiter = plain concatenation
    assert oracle.assemble(ids, np.zeros((0, 2)), np.array([7]))[0].size == 0
    out, _, _ = oracle.assemble(ids, np.array([[0, 2], [4, 6]]), np.zeros(0))
    assert out.tolist() == [100, 101, 104, 105]


def test_assemble_against_list_concatenation_and_projection_mask():
    """Brute force on small random inputs; without its delimiters the output is exactly the target
    tokens the projection keeps (its mask), and the length is n_kept + (ranges - 1) * |delim|."""
    rng = np.random.default_rng(11)
    w = synth.get_config("tiny")
    for trial in range(20):
        L = int(rng.integers(40, 200))
        doff, toff = synth.gen_char_offsets(w, L, prompt=trial)
        M = toff.size - 1
        kept = np.sort(rng.choice(L // 8, size=int(rng.integers(1, L // 8)), replace=False))
        spans = oracle.merge(kept, 8, L)
        ts, mask, n_kept = oracle.project(doff, toff, spans)
        ids = rng.integers(0, 50000, size=M).astype(np.int32)
        delim = rng.integers(50000, 50010, size=int(rng.integers(0, 4))).astype(np.int32)
        out, pos, src = oracle.assemble(ids, ts, delim)
        want = []
        for r, (b, e) in enumerate(ts.tolist()):
            if r > 0:
                want += delim.tolist()
            want += ids[b:e].tolist()
        assert out.tolist() == want
        assert out.size == n_kept + max(len(ts) - 1, 0) * delim.size
        assert out[src >= 0].tolist() == ids[mask.astype(bool)].tolist()
        assert (ids[src[src >= 0]] == out[src >= 0]).all() and (np.diff(src[src >= 0]) > 0).all()
        assert pos.tolist() == list(range(out.size))


# --------------------------------------------------------------------------
# generator sanity (no arithmetic of the method involved)
# --------------------------------------------------------------------------

def test_generator_shapes_and_heavy_hitters_show_up():
    w = synth.get_config("tiny")
    inp = synth.make_score_inputs(w)
    assert inp["q"].shape == (1, 2, 4, 8, 64) and inp["k"][0].shape == (2, 1024, 64)
    assert inp["hh_pos"][0].size == 11
    I = oracle.score(inp["q"][0], inp["k"], w.scale, oracle.LAYER_MEAN)
    top = np.argsort(-I)[:11]
    assert set(top.tolist()) == set(inp["hh_pos"][0].tolist())
    doff, toff = synth.gen_char_offsets(w, w.L)
    assert doff.size == w.L + 1 and doff[-1] == toff[-1] and (np.diff(toff) >= 1).all()
    assert (np.diff(doff) >= 1).all() and np.diff(doff).max() <= 8 and np.diff(toff).max() <= 7
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], np.float32)   # RNE ties and exact values
    assert bf16_bits_to_f32(f32_to_bf16_bits(x)).tolist() == [1.0, 1.0, 1.015625, -2.5, 0.0]


# ---------------------------------------------------------------------------
# keys kept as 8-bit floating point (E4M3) with one scale per (layer, kv head)
# ---------------------------------------------------------------------------
def test_e4m3_decode_matches_the_format_and_a_library():
    """The oracle's E4M3 decode against values that follow from the format's definition (bias 7, three
    mantissa bits, subnormals at exponent field 0, largest finite value 448, NaN only at all ones) and
    against an independent library's decode of all 256 codes."""
    import torch
    val = oracle.e4m3_to_f64
    one = lambda b: float(val(np.array([b], dtype=np.uint8))[0])
    assert one(0x38) == 1.0 and one(0xB8) == -1.0           # exponent field 7, mantissa 0
    assert one(0x3C) == 1.5 and one(0x40) == 2.0
    assert one(0x7E) == 448.0 and one(0xFE) == -448.0       # largest finite: 1.75 * 2^8
    assert one(0x08) == 2.0 ** -6                           # smallest normal
    assert one(0x01) == 2.0 ** -9 and one(0x07) == 7 * 2.0 ** -9   # subnormals m/8 * 2^-6
    assert one(0x00) == 0.0 and one(0x80) == 0.0 and np.signbit(one(0x80))
    assert np.isnan(one(0x7F)) and np.isnan(one(0xFF))
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = val(codes)
    assert np.array_equal(np.isnan(got), np.isnan(lib))
    ok = ~np.isnan(lib)
    assert np.array_equal(got[ok], lib[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(lib[ok]))


def _fp8_case(seed, Lyr=2, H=4, Hkv=2, d=16, n_q=3, L=37):
    rng = np.random.default_rng([260302631, 61, seed])
    q = synth.f32_to_bf16_bits(rng.standard_normal((Lyr, H, n_q, d)).astype(np.float32))
    finite = np.array([b for b in range(256) if (b & 0x7F) != 0x7F], dtype=np.uint8)
    k8 = [finite[rng.integers(0, finite.size, size=(Hkv, L, d))] for _ in range(Lyr)]
    return q, k8, rng


def test_fp8_scores_equal_the_bf16_path_on_exactly_representable_keys():
    """With power-of-two scales, scale * E4M3 value is exact in bf16: the quantised-key path must then
    agree with the (separately pinned) bf16 path fed those very keys, in both layouts and both modes:
    this ties its strides, kv-head mapping, softmax and aggregation to the pinned ones."""
    q, k8, rng = _fp8_case(1)
    kscale = 2.0 ** rng.integers(-6, 3, size=(2, 2)).astype(np.float64)
    kb = [synth.f32_to_bf16_bits((oracle.e4m3_to_f64(k) * kscale[l][:, None, None]).astype(np.float32))
          for l, k in enumerate(k8)]
    for l, k in enumerate(k8):      # the bf16 keys hold exactly the dequantised values
        assert np.array_equal(synth.bf16_bits_to_f32(kb[l]).astype(np.float64), oracle.e4m3_to_f64(k) * kscale[l][:, None, None])
    for mode in (oracle.LAYER_MEAN, oracle.LAYER_MAX):
        want = oracle.score(q, kb, 0.25, mode)
        got = oracle.score_fp8(q, k8, kscale, 0.25, mode)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=0)
        k8_nhd = [np.ascontiguousarray(k.transpose(1, 0, 2)) for k in k8]
        np.testing.assert_allclose(oracle.score_fp8(q, k8_nhd, kscale, 0.25, mode, layout="NHD"), want, rtol=1e-12, atol=0)


def test_fp8_logits_with_arbitrary_scales_against_numpy():
    """Scales that are not powers of two (one per layer and kv head): logits against a numpy einsum over
    the library-decoded keys, scores against scipy's softmax and numpy's max/mean written out."""
    import torch
    from scipy.special import softmax
    q, k8, rng = _fp8_case(2)
    kscale = rng.uniform(0.003, 0.07, size=(2, 2))
    qf = synth.bf16_bits_to_f32(q).astype(np.float64)
    P = []
    for l in range(2):
        kd = torch.from_numpy(k8[l]).view(torch.float8_e4m3fn).to(torch.float64).numpy() * kscale[l][:, None, None]
        s = np.stack([0.25 * np.einsum("ne,je->nj", qf[l, h], kd[h // 2]) for h in range(4)])
        np.testing.assert_allclose(oracle.logits_layer_fp8(q[l], k8[l], kscale[l], 0.25), s, rtol=1e-12, atol=1e-13)
        P.append(softmax(s, axis=-1))
    P = np.stack(P)                                   # [Lyr][H][n_q][L]
    np.testing.assert_allclose(oracle.score_fp8(q, k8, kscale, 0.25, oracle.LAYER_MEAN), P.max(axis=1).mean(axis=(0, 1)), rtol=1e-11)
    np.testing.assert_allclose(oracle.score_fp8(q, k8, kscale, 0.25, oracle.LAYER_MAX), P.max(axis=(0, 1)).mean(axis=0), rtol=1e-11)
    # a wrong scale index (layer and head swapped) must show: the scales differ in every entry
    swapped = oracle.score_fp8(q, k8, kscale.T.copy(), 0.25, oracle.LAYER_MEAN)
    assert np.max(np.abs(swapped - P.max(axis=1).mean(axis=(0, 1)))) > 1e-6


def test_quantised_keys_of_the_generator_decode_close_to_the_originals():
    """The input generator's 8-bit keys (library cast, scale = head maximum / 448): decoded with the
    oracle's table they sit within half an E4M3 step of the bf16 keys they came from."""
    w = synth.get_config("tiny")
    inp = synth.make_score_inputs(w)
    k8, ksc = synth.quantise_k_e4m3(inp["k"][0])
    x = synth.bf16_bits_to_f32(inp["k"][0]).astype(np.float64)
    back = oracle.e4m3_to_f64(k8) * ksc.astype(np.float64)[:, None, None]
    assert not np.isnan(back).any()
    step = np.maximum(np.abs(x) * 2.0 ** -3, ksc.astype(np.float64)[:, None, None] * 2.0 ** -9)   # spacing at x
    assert np.all(np.abs(back - x) <= 0.5 * step * (1 + 1e-6))
    assert np.allclose(np.abs(back).max(axis=(1, 2)), np.abs(x).max(axis=(1, 2)))
