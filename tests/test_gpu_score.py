"""GPU parity of sp_score / sp_score_batch against the CPU float64 oracle,
element by element on the same seeded inputs. Tolerance (stated target of the
build): |gpu - oracle| <= 1e-3 * |oracle| for every token, both aggregation
modes. All calls go through the C ABI."""
from __future__ import annotations

import dataclasses
import sys

import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def small_workload(name, Lyr, H, Hkv, d, n_q, L, cfg_id=100, hh=(1, 100)):
    return synth.Workload(name, cfg_id, Lyr, H, Hkv, d, n_q, L, hh_frac_num=hh[0], hh_frac_den=hh[1])


SHAPES = [
    # name, Lyr, H, Hkv, d, n_q, L   (several key tiles and a ragged tail unless noted)
    ("g4_nq16_d64", 3, 8, 2, 64, 16, 1500),
    ("g4_nq8_d64", 2, 8, 2, 64, 8, 777),
    ("g2_nq8_d128", 3, 4, 2, 128, 8, 777),
    ("g1_nq3_d64", 2, 3, 3, 64, 3, 333),
    ("g8_nq5_d128", 2, 8, 1, 128, 5, 300),
    ("g16_nq8_d64", 1, 16, 1, 64, 8, 260),
    ("g8_nq16_d64", 1, 16, 2, 64, 16, 260),
    ("g3_nq9_d64", 2, 6, 2, 64, 9, 515),
    ("one_key", 2, 4, 2, 64, 8, 1),
    ("exact_tile", 2, 4, 2, 64, 8, 256),
    ("tile_plus_one", 2, 4, 2, 64, 8, 257),
    ("sub_tile_d128", 2, 4, 2, 128, 8, 31),
    # general path with the layers of the prob pass in ranges of 2 + 1, and with enough tiles for no split
    ("uneven_split_d128", 3, 2, 1, 128, 4, 70001),
    ("unsplit_d128", 2, 2, 1, 128, 4, 131072 + 77),
]


@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
@pytest.mark.parametrize("mode", [oracle.LAYER_MEAN, oracle.LAYER_MAX], ids=["mean", "max"])
def test_score_matches_oracle(shape, mode):
    from gpu_util import assert_scores_close, gpu_score
    name, Lyr, H, Hkv, d, n_q, L = shape
    say(f"[score] {name} mode={mode} Lyr={Lyr} H={H} Hkv={Hkv} d={d} n_q={n_q} L={L}")
    w = small_workload(name, Lyr, H, Hkv, d, n_q, L, cfg_id=100 + SHAPES.index(shape))
    inp = synth.make_score_inputs(w)
    want = oracle.score(inp["q"][0], inp["k"], w.scale, mode)
    got = gpu_score(inp["q"][0], inp["k"], w.scale, mode)
    assert_scores_close(got, want)


@pytest.mark.parametrize("cfg", ["tiny"])
@pytest.mark.parametrize("layout", ["HND", "NHD"])
@pytest.mark.parametrize("mode", [0, 1], ids=["mean", "max"])
def test_score_tiny_config_both_layouts(cfg, layout, mode):
    from gpu_util import assert_scores_close, gpu_score
    say(f"[score] cfg={cfg} layout={layout} mode={mode}")
    w = synth.get_config(cfg)
    inp = synth.make_score_inputs(w, layout=layout)
    want = oracle.score(inp["q"][0], inp["k"], w.scale, mode, layout=layout)
    got = gpu_score(inp["q"][0], inp["k"], w.scale, mode, layout=layout)
    assert_scores_close(got, want)


def test_score_closed_forms_on_gpu():
    """Uniform keys give 1/L; a single dominant key captures the score; a huge
    common shift of all keys does not change the result (max-subtraction)."""
    from gpu_util import gpu_score
    say("[score] closed forms")
    rng = np.random.default_rng(5)
    Lyr, H, Hkv, n_q, d, L = 2, 8, 2, 8, 64, 700
    q = synth.f32_to_bf16_bits(rng.integers(-3, 4, size=(Lyr, H, n_q, d)).astype(np.float32) * 0.25)
    krow = rng.integers(-3, 4, size=(Hkv, 1, d)).astype(np.float32)
    k = [synth.f32_to_bf16_bits(np.repeat(krow, L, axis=1)) for _ in range(Lyr)]
    for mode in (0, 1):
        got = gpu_score(q, k, 0.125, mode)
        np.testing.assert_allclose(got, 1.0 / L, rtol=1e-5)
    # dominant key
    kz = np.zeros((Hkv, L, d), np.float32)
    kz[:, 123, :] = 8.0 * synth.bf16_bits_to_f32(q[0, 0, 0])[None, :]
    kd = [synth.f32_to_bf16_bits(kz) for _ in range(Lyr)]
    want = oracle.score(q, kd, 0.125, 1)
    got = gpu_score(q, kd, 0.125, 1)
    np.testing.assert_allclose(got, want, rtol=1e-3)
    assert got.argmax() == 123
    # shift invariance with a large shift (exact in bf16: |k + v| <= 67)
    kf = rng.integers(-3, 4, size=(Hkv, L, d)).astype(np.float32)
    v = rng.choice([-64.0, 64.0], size=(1, 1, d)).astype(np.float32)
    base = gpu_score(q, [synth.f32_to_bf16_bits(kf)] * Lyr, 0.125, 0)
    shifted = gpu_score(q, [synth.f32_to_bf16_bits(kf + v)] * Lyr, 0.125, 0)
    assert np.isfinite(shifted).all()
    np.testing.assert_allclose(shifted, base, rtol=2e-4)


def test_score_is_deterministic():
    from gpu_util import gpu_score
    say("[score] determinism")
    w = small_workload("det", 3, 8, 2, 64, 16, 2100, cfg_id=150)
    inp = synth.make_score_inputs(w)
    a = gpu_score(inp["q"][0], inp["k"], w.scale, 0)
    b = gpu_score(inp["q"][0], inp["k"], w.scale, 0)
    assert a.tobytes() == b.tobytes()


@pytest.mark.parametrize("layout", ["HND", "NHD"])
def test_score_batch_matches_oracle_per_prompt(layout):
    """Ragged batch with an empty prompt, a one-token prompt and lengths around
    the tile size; each prompt is softmaxed over its own keys only."""
    from gpu_util import assert_scores_close, gpu_score, gpu_score_batch
    say(f"[score_batch] layout={layout}")
    lengths = np.array([300, 1, 0, 513, 256, 77], dtype=np.int64)
    w = dataclasses.replace(small_workload("rag", 2, 8, 2, 64, 8, 0, cfg_id=160), batch=len(lengths))
    hh = synth.heavy_hitter_positions(w, lengths)
    q = synth.gen_q(w, len(lengths))
    ks = [synth.gen_k_layer(w, l, q, lengths, hh) for l in range(w.n_layers)]      # [Hkv][T][d]
    offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    packed = ks if layout == "HND" else [np.ascontiguousarray(k.transpose(1, 0, 2)) for k in ks]
    for mode in (0, 1):
        got = gpu_score_batch(q, packed, offsets, w.scale, mode, layout=layout)
        for b, Lb in enumerate(lengths):
            if Lb == 0:
                continue
            sl = slice(int(offsets[b]), int(offsets[b + 1]))
            kb = [np.ascontiguousarray(k[:, sl, :]) for k in ks]
            want = oracle.score(q[b], kb, w.scale, mode)
            assert_scores_close(got[sl], want)
            if layout == "HND":
                single = gpu_score(q[b], kb, w.scale, mode)
                np.testing.assert_allclose(got[sl], single, rtol=1e-6)


FUSED_BATCHES = [
    # name, Lyr, H, Hkv, d, n_q, prompt lengths  (every prompt empty or >= 512 tokens: one launch or several)
    ("batch_one_launch", 2, 8, 2, 64, 8, [20000, 512, 700, 0, 15000, 9001]),
    ("batch_nq16_two_row_blocks", 1, 8, 2, 64, 16, [12000, 24000, 513]),
    ("batch_g8_two_gblocks", 1, 16, 2, 64, 8, [33000, 1024, 2047]),
    ("batch_several_launches", 1, 4, 1, 64, 8, [70000, 65000, 60000, 3000, 1500]),
    ("batch_single_prompt", 2, 8, 2, 64, 5, [40000]),
    ("batch_d128_one_launch", 2, 4, 2, 128, 8, [9000, 256, 300, 0, 7000, 4001]),
    # the kernel instantiations with a fixed model shape (16 layers, 32 / 8 heads) for several prompts a launch
    ("batch_draft_model_nq16", 16, 32, 8, 64, 16, [20000, 13000, 600]),
    ("batch_draft_model_nq8", 16, 32, 8, 64, 8, [15000, 18000, 512, 0, 1000]),
    ("batch_d128_several_launches", 1, 4, 2, 128, 8, [40000, 33000, 30000, 1500]),
]


@pytest.mark.parametrize("case", FUSED_BATCHES, ids=[c[0] for c in FUSED_BATCHES])
def test_score_batch_on_the_single_launch_kernel(case):
    """Ragged batches whose prompts are all at least one tile (512 keys; 256 at head_dim 128) long take the single-launch
    kernel, several prompts to a launch: every prompt against the oracle run on that prompt alone, both
    modes, both layouts, deterministic."""
    import paper_2603_02631_amd as sp
    from gpu_util import assert_scores_close, gpu_score_batch, make_desc
    name, Lyr, H, Hkv, d, n_q, lens = case
    lengths = np.array(lens, dtype=np.int64)
    say(f"[score_batch-fused] {name} Lyr={Lyr} H={H} Hkv={Hkv} n_q={n_q} lengths={lens}")
    w = dataclasses.replace(small_workload(name, Lyr, H, Hkv, d, n_q, 0, cfg_id=170 + FUSED_BATCHES.index(case), hh=(1, 1000)),
                            batch=len(lengths))
    hh = synth.heavy_hitter_positions(w, lengths)
    q = synth.gen_q(w, len(lengths))
    ks = [synth.gen_k_layer(w, l, q, lengths, hh) for l in range(w.n_layers)]
    offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    T = int(offsets[-1])
    n_launch = sp.sp_score_batch_is_fused(make_desc(Lyr, H, Hkv, d, n_q, w.scale, 0, "HND", T), [int(v) for v in offsets])
    assert n_launch >= (2 if "several" in name else 1)
    got = None
    for mode in (0, 1):
        got = gpu_score_batch(q, ks, offsets, w.scale, mode)
        for b, Lb in enumerate(lengths):
            if Lb == 0:
                continue
            sl = slice(int(offsets[b]), int(offsets[b + 1]))
            want = oracle.score(q[b], [np.ascontiguousarray(k[:, sl, :]) for k in ks], w.scale, mode)
            assert_scores_close(got[sl], want)
        say(f"  mode {mode}: ok")
    again = gpu_score_batch(q, ks, offsets, w.scale, 1)
    assert again.tobytes() == got.tobytes()
    nhd = [np.ascontiguousarray(k.transpose(1, 0, 2)) for k in ks]
    assert gpu_score_batch(q, nhd, offsets, w.scale, 1, layout="NHD").tobytes() == got.tobytes()


def test_score_mid_size_config():
    """The 16-layer, 32/8-head, head_dim-64 shape at L = 8192 (second workload), full element-wise parity."""
    from gpu_util import assert_scores_close, gpu_score
    say("[score] llama1b-8k full")
    w = synth.get_config("llama1b-8k")
    inp = synth.make_score_inputs(w)
    for mode in (0, 1):
        want = oracle.score(inp["q"][0], inp["k"], w.scale, mode)
        got = gpu_score(inp["q"][0], inp["k"], w.scale, mode)
        assert_scores_close(got, want)
        say(f"  mode {mode}: max rel err {np.max(np.abs(got - want) / want):.2e}")


# Long single prompts take the single-launch kernel that keeps K on chip (head_dim 64: up to 64 padded
# query rows and 128K tokens; head_dim 128: up to 32 rows and 64K tokens).
FUSED_SHAPES = [
    # name, Lyr, H, Hkv, d, n_q, L
    ("fused_g4_nq16_tail", 2, 8, 2, 64, 16, 40000),       # 79 workgroups, 64-key tail
    ("fused_g4_nq8", 2, 8, 2, 64, 8, 33000),
    ("fused_g2_nq8_rows32", 3, 4, 2, 64, 8, 36001),
    ("fused_g8_nq8_two_gblocks", 1, 16, 2, 64, 8, 34000),
    ("fused_g3_nq5_padding", 2, 6, 2, 64, 5, 35000),
    ("fused_single_phase_full_grid", 1, 4, 1, 64, 16, 131072),
    ("fused_20_phases", 5, 8, 4, 64, 16, 40000),
    # the two kernel instantiations with a fixed model shape (16 layers, 32 / 8 heads): 8 and 16 lookahead rows
    ("fused_draft_model_nq8", 16, 32, 8, 64, 8, 33000),
    ("fused_draft_model_nq16", 16, 32, 8, 64, 16, 32768 + 513),
    ("fused_draft_model_nq8_full_grid", 16, 32, 8, 64, 8, 131072 - 100),     # 256 workgroups, ragged last tile
    # head_dim 128 (up to 32 padded query rows): 256 keys per workgroup, from 96 workgroups up
    ("fused_d128_g2_nq8", 3, 4, 2, 128, 8, 25000),                           # 98 workgroups, 168-key tail
    ("fused_d128_g4_nq8_rows32", 2, 8, 2, 128, 8, 24576 + 1),                # 1-key tail
    ("fused_d128_g2_nq5_padding", 2, 4, 2, 128, 5, 26000),
    ("fused_d128_g3_nq8_padding", 2, 6, 2, 128, 8, 25500),
    ("fused_d128_full_grid", 2, 4, 2, 128, 8, 65536 - 100),                  # 256 workgroups, ragged last tile
    ("fused_d128_28_phases", 7, 8, 4, 128, 8, 24576),
    ("fused_d128_40k", 2, 4, 2, 128, 8, 40000),
]


def test_which_prompts_take_the_single_launch_kernel():
    """The lengths at which sp_score changes kernels (sp_score_is_fused): head_dim 64 from 64 workgroups of
    512 keys up to 256; head_dim 128 from 96 workgroups of 256 keys up to 256, and only with at most 32
    padded query rows."""
    import paper_2603_02631_amd as sp
    from gpu_util import make_desc
    def fused(d, G, n_q, L):
        return sp.sp_score_is_fused(make_desc(2, 2 * G, 2, d, n_q, 0.1, 0, "HND", L), L)
    assert [fused(64, 4, 16, L) for L in (63 * 512, 63 * 512 + 1, 131072, 131073)] == [0, 1, 1, 0]
    assert [fused(128, 2, 8, L) for L in (95 * 256, 95 * 256 + 1, 65536, 65537)] == [0, 1, 1, 0]
    assert fused(128, 4, 8, 40000) == 1 and fused(128, 4, 16, 40000) == 0 and fused(128, 8, 8, 40000) == 0
    assert fused(64, 8, 16, 40000) == 0          # 128 padded rows


@pytest.mark.parametrize("shape", FUSED_SHAPES, ids=[s[0] for s in FUSED_SHAPES])
def test_fused_score_matches_oracle(shape):
    import paper_2603_02631_amd as sp
    from gpu_util import assert_scores_close, gpu_score, make_desc
    name, Lyr, H, Hkv, d, n_q, L = shape
    say(f"[score-fused] {name} Lyr={Lyr} H={H} Hkv={Hkv} d={d} n_q={n_q} L={L}")
    w = small_workload(name, Lyr, H, Hkv, d, n_q, L, cfg_id=200 + FUSED_SHAPES.index(shape), hh=(1, 1000))
    assert sp.sp_score_is_fused(make_desc(Lyr, H, Hkv, d, n_q, w.scale, 0, "HND", L), L) == 1
    inp = synth.make_score_inputs(w)
    for mode in (0, 1):
        want = oracle.score(inp["q"][0], inp["k"], w.scale, mode)
        got = gpu_score(inp["q"][0], inp["k"], w.scale, mode)
        assert_scores_close(got, want)
        say(f"  mode {mode}: max rel err {np.max(np.abs(got - want) / want):.2e}")
    again = gpu_score(inp["q"][0], inp["k"], w.scale, 1)
    assert again.tobytes() == got.tobytes()          # deterministic
    nhd = [np.ascontiguousarray(k.transpose(1, 0, 2)) for k in inp["k"]]
    got_nhd = gpu_score(inp["q"][0], nhd, w.scale, 1, layout="NHD")
    assert got_nhd.tobytes() == got.tobytes()        # same keys through token-major strides


def test_fused_score_gives_up_as_a_whole():
    """The bounded waits of the single-launch kernel, driven to give up from the host (the test hook
    makes the combining waves treat their partial results as never arriving, with a spin limit of a few
    polls, so every kernel still runs to its end): all scores NaN, status word 1; the next ordinary
    call on the same workspace is valid again."""
    import torch
    import paper_2603_02631_amd as sp
    from gpu_util import DEV, dev_bits, make_desc, status_word, workspace
    Lyr, H, Hkv, d, n_q, L = 2, 8, 2, 64, 16, 40000
    w = small_workload("fused_give_up", Lyr, H, Hkv, d, n_q, L, cfg_id=290, hh=(1, 1000))
    inp = synth.make_score_inputs(w)
    desc = make_desc(Lyr, H, Hkv, d, n_q, w.scale, 0, "HND", L)
    assert sp.sp_score_is_fused(desc, L) == 1
    qd = dev_bits(inp["q"][0])
    kd = [dev_bits(k) for k in inp["k"]]
    ws = workspace(sp.sp_score_workspace(desc, L, 1))
    scores = torch.zeros(L, dtype=torch.float32, device=DEV)
    say("[score-fused] give-up path: spin limit 4, partials treated as missing")
    try:
        sp.sp_debug_fused_giveup(4, 1)
        sp.sp_score(desc, qd, kd, L, scores, ws)
        torch.cuda.synchronize()
    finally:
        sp.sp_debug_fused_giveup(1 << 20, 0)
    assert status_word(ws) == 1
    assert bool(torch.isnan(scores).all())
    say("[score-fused] ordinary call on the same workspace")
    sp.sp_score(desc, qd, kd, L, scores, ws)
    torch.cuda.synchronize()
    assert status_word(ws) == 0
    from gpu_util import assert_scores_close
    assert_scores_close(scores.cpu().numpy(), oracle.score(inp["q"][0], inp["k"], w.scale, 0))


LOOK_SHAPES = [
    # name, Lyr, H, Hkv, d, n_q, L   (general path: short prompts, head_dim 128; fused path: long prompts)
    ("look_g4_nq16_d64", 3, 8, 2, 64, 16, 1500),
    ("look_g2_nq8_d128", 2, 4, 2, 128, 8, 777),
    ("look_g3_nq5_d64", 2, 6, 2, 64, 5, 333),
    ("look_nq1_d64", 2, 4, 2, 64, 1, 300),
    ("look_fused_g4_nq16", 3, 8, 2, 64, 16, 33000),
    ("look_fused_g3_nq5_padding", 2, 6, 2, 64, 5, 35000),
    ("look_fused_d128_g2_nq8", 2, 4, 2, 128, 8, 25000),
]


@pytest.mark.parametrize("shape", LOOK_SHAPES, ids=[s[0] for s in LOOK_SHAPES])
def test_score_with_lookahead_keys_matches_oracle(shape):
    """sp_score_look: the rows' normalisers include their visible lookahead keys
    (Algorithm 1, ForwardWithAttn at lookahead = i); both visibility settings and
    both aggregation modes, on both kernels."""
    import paper_2603_02631_amd as sp
    from gpu_util import assert_scores_close, gpu_score, gpu_score_look, make_desc
    name, Lyr, H, Hkv, d, n_q, L = shape
    say(f"[score-look] {name} Lyr={Lyr} H={H} Hkv={Hkv} d={d} n_q={n_q} L={L}")
    w = small_workload(name, Lyr, H, Hkv, d, n_q, L, cfg_id=300 + LOOK_SHAPES.index(shape), hh=(1, 1000))
    fused = sp.sp_score_is_fused(make_desc(Lyr, H, Hkv, d, n_q, w.scale, 0, "HND", L), L)
    assert fused == (1 if "fused" in name else 0)
    inp = synth.make_score_inputs(w)
    q = inp["q"][0]
    kl = synth.gen_look_keys(w, inp["q"])
    plain = oracle.score(q, inp["k"], w.scale, 0)
    for look_self in (0, 1):
        for mode in (0, 1):
            want = oracle.score_look(q, inp["k"], kl, look_self, w.scale, mode)
            got = gpu_score_look(q, inp["k"], kl, look_self, w.scale, mode)
            assert_scores_close(got, want)
            say(f"  self {look_self} mode {mode}: max rel err {np.max(np.abs(got - want) / want):.2e}")
    # the term matters on these inputs, well above the tolerance (a test that passes without it would prove nothing)
    assert np.max(np.abs(oracle.score_look(q, inp["k"], kl, 1, w.scale, 0) - plain) / plain) > 5e-3
    # and a call without lookahead keys afterwards is the plain result again (no state left behind)
    assert_scores_close(gpu_score(q, inp["k"], w.scale, 0), plain)


PAGED_SHAPES = [
    # name, Lyr, H, Hkv, d, n_q, L, page_tokens, layout
    ("paged_general_d64", 3, 8, 2, 64, 16, 1500, 512, "HND"),
    ("paged_general_d128_nhd", 2, 4, 2, 128, 8, 777, 512, "NHD"),
    ("paged_general_one_page", 2, 4, 2, 64, 8, 300, 1024, "HND"),
    ("paged_fused_4k_ragged_tail", 3, 8, 2, 64, 16, 33000 + 77, 4096, "HND"),
    ("paged_fused_4k_whole_pages", 2, 8, 2, 64, 8, 8 * 4096, 4096, "HND"),
    ("paged_fused_512_nhd", 2, 6, 2, 64, 5, 35000, 512, "NHD"),
    ("paged_fused_d128_2k_ragged_tail", 2, 4, 2, 128, 8, 25000 + 77, 2048, "HND"),
    ("paged_fused_d128_512_nhd", 2, 4, 2, 128, 5, 24600, 512, "NHD"),
    ("paged_fused_d128_40k_4k_pages", 1, 4, 2, 128, 8, 40000 + 5, 4096, "HND"),
]


@pytest.mark.parametrize("shape", PAGED_SHAPES, ids=[s[0] for s in PAGED_SHAPES])
def test_score_over_paged_keys_matches_oracle(shape):
    """sp_score_paged: the keys sit in shuffled pages of per-layer pools (Section 3.1: KV caches in
    fixed-size blocks); rows that hold no token are NaN. Oracle: the plain score of the keys gathered
    through the block table."""
    import paper_2603_02631_amd as sp
    from gpu_util import assert_scores_close, gpu_score_paged, make_desc, make_paged
    name, Lyr, H, Hkv, d, n_q, L, P, layout = shape
    say(f"[score-paged] {name} Lyr={Lyr} H={H} Hkv={Hkv} d={d} n_q={n_q} L={L} page={P} {layout}")
    w = small_workload(name, Lyr, H, Hkv, d, n_q, L, cfg_id=400 + PAGED_SHAPES.index(shape), hh=(1, 1000))
    fused = sp.sp_score_is_fused(make_desc(Lyr, H, Hkv, d, n_q, w.scale, 0, layout, P), L)
    assert fused == (1 if "fused" in name else 0)
    inp = synth.make_score_inputs(w)
    q = inp["q"][0]
    pools, table = make_paged(inp["k"], P, layout, seed=w.cfg_id)
    gathered = [oracle.gather_pages(pool, table, L, layout) for pool in pools]
    for l in range(Lyr):                      # the scatter of the test and the oracle's gather are inverse
        ref = inp["k"][l] if layout == "HND" else inp["k"][l].transpose(1, 0, 2)
        np.testing.assert_array_equal(gathered[l], ref)
    for mode in (0, 1):
        want = oracle.score(q, gathered, w.scale, mode, layout=layout)
        got = gpu_score_paged(q, pools, table, P, L, w.scale, mode, layout)
        assert_scores_close(got, want)
        say(f"  mode {mode}: max rel err {np.max(np.abs(got - want) / want):.2e}")
