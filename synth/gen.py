"""Seeded generators: bf16 Q/K tensors with planted heavy-hitter keys, prompt
lengths of a ragged batch, and character-offset arrays of two tokenizations of
one text.

Everything is drawn with numpy's counter-based ``default_rng`` seeded by
``[SEED, cfg_id, stream...]`` so that any single layer (or prompt) can be
regenerated on its own without holding the whole K cache in host memory.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .configs import Workload

SEED = 260302631

_STREAM_Q = 0
_STREAM_HH = 1
_STREAM_LEN = 2
_STREAM_CHARS = 3
_STREAM_LOOK = 4
_STREAM_K0 = 16        # layer l draws from stream _STREAM_K0 + l


def _rng(cfg_id: int, *stream: int) -> np.random.Generator:
    return np.random.default_rng([SEED, cfg_id, *stream])


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def gen_prompt_lengths(w: Workload) -> np.ndarray:
    """Prompt lengths: one entry for a single prompt, ``w.batch`` log-uniform
    draws in ``w.batch_len_range`` for the ragged batch."""
    if w.batch <= 0:
        return np.array([w.L], dtype=np.int64)
    lo, hi = w.batch_len_range
    u = _rng(w.cfg_id, _STREAM_LEN).uniform(math.log(lo), math.log(hi), size=w.batch)
    return np.clip(np.rint(np.exp(u)), lo, hi).astype(np.int64)


def heavy_hitter_positions(w: Workload, lengths: Sequence[int]) -> List[np.ndarray]:
    """Per prompt, the sorted key positions (prompt-local) that carry a planted
    heavy-hitter key. The same set is used in every layer and kv head."""
    out = []
    for b, L in enumerate(lengths):
        L = int(L)
        rng = _rng(w.cfg_id, _STREAM_HH, b)
        n_hh = -(-L * w.hh_frac_num // w.hh_frac_den) if w.hh_frac_num > 0 else 0
        n_hh = min(n_hh, L)
        if n_hh == 0:
            out.append(np.zeros(0, dtype=np.int64))
            continue
        if w.hh_bands > 0 and L >= w.hh_bands * w.hh_band_len * 2:
            # non-overlapping bands with uniform random starts: place the bands
            # by drawing sorted offsets in the slack and spacing them out.
            slack = L - w.hh_bands * w.hh_band_len
            gaps = np.sort(rng.integers(0, slack + 1, size=w.hh_bands))
            starts = gaps + np.arange(w.hh_bands) * w.hh_band_len
            pool = (starts[:, None] + np.arange(w.hh_band_len)[None, :]).reshape(-1)
            pos = rng.choice(pool, size=min(n_hh, pool.size), replace=False)
        else:
            pos = rng.choice(L, size=n_hh, replace=False)
        out.append(np.sort(pos.astype(np.int64)))
    return out


def gen_q(w: Workload, n_prompts: int = 1) -> np.ndarray:
    """Lookahead queries as bf16 bits, shape [B][n_layers][n_q_heads][n_q][head_dim]."""
    rng = _rng(w.cfg_id, _STREAM_Q)
    x = rng.standard_normal((n_prompts, w.n_layers, w.n_q_heads, w.n_q, w.head_dim), dtype=np.float32)
    return f32_to_bf16_bits(x)


def gen_look_keys(w: Workload, q_bits: np.ndarray, self_gain: float = 1.0) -> np.ndarray:
    """Keys of the lookahead tokens of prompt 0 as bf16 bits, [n_layers][n_kv_heads][n_q][head_dim]:
    N(0,1) plus ``self_gain`` times the query vector of the same lookahead row (first head of the kv
    head's group), so that a row attends to its own token's key about as strongly as decoders do."""
    rng = _rng(w.cfg_id, _STREAM_LOOK)
    x = rng.standard_normal((w.n_layers, w.n_kv_heads, w.n_q, w.head_dim), dtype=np.float32)
    qv = bf16_bits_to_f32(q_bits[0][:, ::w.group, :, :])
    return f32_to_bf16_bits(x + np.float32(self_gain) * qv)


def gen_k_layer(w: Workload, layer: int, q_bits: np.ndarray, lengths: Sequence[int],
                hh_pos: Sequence[np.ndarray], hh_gain: float = 3.0) -> np.ndarray:
    """K of one layer as bf16 bits, head-major packed layout [n_kv_heads][T][head_dim]
    with T = sum(lengths) and prompts back to back along T.

    Background keys are N(0,1). At each heavy-hitter position, per kv head, the
    key is replaced by ``hh_gain`` times one lookahead query vector of that kv
    head's query group (random head in the group, random lookahead row), so that
    query row attends to it with a logit of about ``hh_gain * |q|^2 * scale``.
    """
    T = int(np.sum(lengths))
    rng = _rng(w.cfg_id, _STREAM_K0 + layer)
    k = f32_to_bf16_bits(rng.standard_normal((w.n_kv_heads, T, w.head_dim), dtype=np.float32))
    G = w.group
    off = 0
    for b, L in enumerate(lengths):
        pos = hh_pos[b]
        if pos.size:
            g_idx = rng.integers(0, G, size=(w.n_kv_heads, pos.size))
            n_idx = rng.integers(0, w.n_q, size=(w.n_kv_heads, pos.size))
            for kv in range(w.n_kv_heads):
                qv = bf16_bits_to_f32(q_bits[b, layer, kv * G + g_idx[kv], n_idx[kv], :])
                k[kv, off + pos, :] = f32_to_bf16_bits(np.float32(hh_gain) * qv)
        off += int(L)
    return k


def quantise_k_e4m3(k_bits: np.ndarray, headroom: float = 1.0) -> Tuple[np.ndarray, np.ndarray]:
    """8-bit keys for one layer: bf16 keys ``[Hkv][T][d]`` -> (E4M3 codes uint8 of the same shape,
    float32 scale per kv head), scale = largest magnitude of the head / 448 (the format's largest
    finite value) times ``headroom`` (>= 1), codes = the library's round-to-nearest cast of key / scale. This is input
    preparation, like the rounding to bf16: what the codes and scales mean is for the consumers."""
    import torch
    x = torch.from_numpy(bf16_bits_to_f32(k_bits))
    amax = x.abs().amax(dim=(1, 2)).clamp_min(1e-30)
    scale = (amax / 448.0 * float(headroom)).to(torch.float32)
    codes = (x / scale[:, None, None]).to(torch.float8_e4m3fn).view(torch.uint8)
    return codes.numpy().copy(), scale.numpy().copy()


def _draw_lengths(rng: np.random.Generator, model: str, params: Tuple[int, float], n: int) -> np.ndarray:
    if model == "uniform":
        return rng.integers(1, params[0] + 1, size=n).astype(np.int64)
    return rng.geometric(1.0 / params[1], size=n).astype(np.int64)


def gen_char_offsets(w: Workload, L: int, prompt: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Character offsets of two tokenizations of one text.

    Returns ``(draft_off[L+1], target_off[M+1])``, both int64, starting at 0,
    strictly increasing, and ending at the same total character count. The
    draft side has exactly ``L`` tokens; the target side is an independent split
    of the same character string whose last token is truncated to fit.
    """
    rng = _rng(w.cfg_id, _STREAM_CHARS, prompt)
    dl = _draw_lengths(rng, w.char_model, w.draft_chars, L)
    doff = np.concatenate([[0], np.cumsum(dl)]).astype(np.int64)
    total = int(doff[-1])
    mean = (w.target_chars[0] + 1) / 2.0 if w.char_model == "uniform" else w.target_chars[1]
    pieces = []
    have = 0
    while have < total:
        n = int((total - have) / mean * 1.1) + 64
        tl = _draw_lengths(rng, w.char_model, w.target_chars, n)
        pieces.append(tl)
        have += int(tl.sum())
    tl = np.concatenate(pieces)
    cs = np.cumsum(tl)
    m = int(np.searchsorted(cs, total, side="left")) + 1   # first prefix reaching total
    toff = np.concatenate([[0], cs[:m]]).astype(np.int64)
    toff[-1] = total
    return doff, toff


def make_score_inputs(w: Workload, layout: str = "HND"):
    """All score-pass inputs of a (small) workload held in host memory.

    Returns a dict with ``q`` (uint16 [B][Lyr][H][n_q][d]), ``k`` (list over
    layers of uint16 arrays, [Hkv][T][d] for "HND" or [T][Hkv][d] for "NHD"),
    ``lengths`` (int64 [B]), ``offsets`` (int64 [B+1]) and ``hh_pos``.
    """
    lengths = gen_prompt_lengths(w)
    hh = heavy_hitter_positions(w, lengths)
    q = gen_q(w, len(lengths))
    ks = []
    for l in range(w.n_layers):
        k = gen_k_layer(w, l, q, lengths, hh)
        if layout == "NHD":
            k = np.ascontiguousarray(k.transpose(1, 0, 2))
        elif layout != "HND":
            raise ValueError("layout must be 'HND' or 'NHD'")
        ks.append(k)
    offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    return {"q": q, "k": ks, "lengths": lengths, "offsets": offsets, "hh_pos": hh, "layout": layout}
