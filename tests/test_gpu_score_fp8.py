"""GPU parity of sp_score_fp8 (keys stored as E4M3 codes with one scale per layer and kv head)
against the oracle on exactly the same dequantised keys: |gpu - oracle| <= 1e-3 * |oracle| for every
token, both aggregation modes, both key layouts. The keys are the generator's bf16 keys (N(0,1) plus
planted heavy hitters) quantised with the head's maximum mapped to 448."""
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


FP8_SHAPES = [
    # name, Lyr, H, Hkv, d, n_q, L
    ("fp8_g4_nq16_d64", 3, 8, 2, 64, 16, 1500),
    ("fp8_g2_nq8_d128", 3, 4, 2, 128, 8, 777),
    ("fp8_g3_nq5_d64_one_tile_plus_one", 2, 6, 2, 64, 5, 257),
    ("fp8_one_key", 2, 4, 2, 64, 8, 1),
    ("fp8_g4_nq8_d64_long", 2, 8, 2, 64, 8, 40000),          # past the length where bf16 keys take the single-launch kernel
    ("fp8_layer_split_d128", 3, 2, 1, 128, 4, 70001),
    # head_dim 64 at the lengths of the single-launch kernel: its variant for 8-bit keys
    ("fp8_fused_g4_nq16_tail", 2, 8, 2, 64, 16, 40000 + 64),
    ("fp8_fused_g8_nq8_two_gblocks", 1, 16, 2, 64, 8, 34000),
    ("fp8_fused_g3_nq5_padding", 2, 6, 2, 64, 5, 35000),
    ("fp8_fused_20_phases", 5, 8, 4, 64, 16, 33000),
    ("fp8_fused_full_grid", 1, 4, 1, 64, 8, 131072 - 100),
    # head_dim 128 on the single-launch kernel
    ("fp8_fused_d128_g2_nq8", 3, 4, 2, 128, 8, 25000),
    ("fp8_fused_d128_g4_nq5_tail", 2, 8, 2, 128, 5, 24576 + 1),
    ("fp8_fused_d128_full_grid", 1, 4, 2, 128, 8, 65536 - 100),
    # the instantiations with a fixed model shape (16 layers, 32 / 8 heads)
    ("fp8_fused_draft_model_nq8", 16, 32, 8, 64, 8, 33000),
    ("fp8_fused_draft_model_nq16", 16, 32, 8, 64, 16, 32768 + 513),
    ("fp8_fused_draft_model_nq16_full_grid", 16, 32, 8, 64, 16, 131072 - 100),
]


@pytest.mark.parametrize("shape", FP8_SHAPES, ids=[s[0] for s in FP8_SHAPES])
def test_score_fp8_matches_oracle(shape):
    import paper_2603_02631_amd as sp
    from gpu_util import assert_scores_close, gpu_score_fp8, make_desc
    name, Lyr, H, Hkv, d, n_q, L = shape
    fused = sp.sp_score_fp8_is_fused(make_desc(Lyr, H, Hkv, d, n_q, 0.125, 0, "HND", L), L)
    assert fused == (1 if ("fused" in name or name == "fp8_g4_nq8_d64_long") else 0)
    say(f"[score-fp8] {name} Lyr={Lyr} H={H} Hkv={Hkv} d={d} n_q={n_q} L={L}")
    w = synth.Workload(name, 300 + FP8_SHAPES.index(shape), Lyr, H, Hkv, d, n_q, L, hh_frac_num=1, hh_frac_den=100)
    inp = synth.make_score_inputs(w)
    # every layer gets its own headroom on top of the heads' own maxima: scales differ, so a mixed-up index shows
    k8, ksc = zip(*[synth.quantise_k_e4m3(k, headroom=1.0 + 0.07 * l) for l, k in enumerate(inp["k"])])
    ksc = np.stack(ksc)
    for mode in (oracle.LAYER_MEAN, oracle.LAYER_MAX):
        want = oracle.score_fp8(inp["q"][0], k8, ksc.astype(np.float64), w.scale, mode)
        got = gpu_score_fp8(inp["q"][0], k8, ksc, w.scale, mode)
        assert_scores_close(got, want)
        say(f"  mode {mode}: max rel err {np.max(np.abs(got - want) / want):.2e}")
    nhd = [np.ascontiguousarray(k.transpose(1, 0, 2)) for k in k8]
    got_nhd = gpu_score_fp8(inp["q"][0], nhd, ksc, w.scale, oracle.LAYER_MAX, layout="NHD")
    assert got_nhd.tobytes() == got.tobytes()        # same keys through token-major strides


def test_score_fp8_differs_from_bf16_scores_by_the_quantisation_only():
    """Sanity of the stand-in data: the quantised keys change the scores visibly (so the test above is
    not vacuous) but not wildly."""
    w = synth.Workload("fp8_vs_bf16", 320, 2, 8, 2, 64, 8, 1024)
    inp = synth.make_score_inputs(w)
    k8, ksc = zip(*[synth.quantise_k_e4m3(k) for k in inp["k"]])
    a = oracle.score(inp["q"][0], inp["k"], w.scale, 0)
    b = oracle.score_fp8(inp["q"][0], k8, np.stack(ksc).astype(np.float64), w.scale, 0)
    rel = np.abs(a - b) / a
    assert 1e-3 < rel.max() < 1.0
