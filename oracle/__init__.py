"""CPU float64 oracle of the token-importance pass (test infrastructure).

Thin ctypes wrapper over ``sp_oracle.c``: the arithmetic lives in the C file,
this module only marshals numpy arrays. Only tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the GPU library never does, and
this module imports nothing from the GPU package.

Citations (paper sections) are given per function in ``sp_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "sp_oracle.c")
_LIB = os.path.join(_DIR, "libsp_oracle.so")

LAYER_MEAN = 0
LAYER_MAX = 1


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (``-O2``, OpenMP over rows, no hand vectorisation)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        build(force=True)
    lib = ctypes.CDLL(_LIB)
    c = ctypes
    P = c.c_void_p
    lib.sp_oracle_max_threads.restype = c.c_int
    lib.sp_oracle_set_threads.argtypes = [c.c_int]
    lib.sp_oracle_logits_layer.argtypes = [P, P, c.c_int64, c.c_int64, c.c_int, c.c_int, c.c_int,
                                           c.c_int, c.c_int64, c.c_double, P]
    lib.sp_oracle_softmax_rows.argtypes = [P, c.c_int64, c.c_int64, P, P]
    lib.sp_oracle_score.argtypes = [P, P, c.c_int64, c.c_int64, c.c_int, c.c_int, c.c_int, c.c_int,
                                    c.c_int, c.c_int64, c.c_double, c.c_int, P]
    lib.sp_oracle_score_look.argtypes = [P, P, c.c_int64, c.c_int64, c.c_int, c.c_int, c.c_int, c.c_int,
                                         c.c_int, c.c_int64, c.c_double, c.c_int, P, c.c_int, P]
    lib.sp_oracle_e4m3_to_f64.argtypes = [c.c_uint8]
    lib.sp_oracle_e4m3_to_f64.restype = c.c_double
    lib.sp_oracle_logits_layer_fp8.argtypes = [P, P, c.c_int64, c.c_int64, c.c_int, c.c_int, c.c_int,
                                               c.c_int, c.c_int64, P, c.c_double, P]
    lib.sp_oracle_score_fp8.argtypes = [P, P, c.c_int64, c.c_int64, c.c_int, c.c_int, c.c_int, c.c_int,
                                        c.c_int, c.c_int64, P, c.c_double, c.c_int, P]
    lib.sp_oracle_pool.argtypes = [P, c.c_int64, c.c_int, P]
    lib.sp_oracle_chunk_mean.argtypes = [P, c.c_int64, c.c_int, P]
    lib.sp_oracle_keep_count.argtypes = [c.c_int64, c.c_int64, c.c_int64]
    lib.sp_oracle_keep_count.restype = c.c_int64
    lib.sp_oracle_topk.argtypes = [P, c.c_int64, c.c_int64, P]
    lib.sp_oracle_merge.argtypes = [P, c.c_int64, c.c_int, c.c_int64, P]
    lib.sp_oracle_merge.restype = c.c_int64
    lib.sp_oracle_assemble.argtypes = [P, c.c_int64, P, c.c_int64, P, c.c_int64, P, P, P, P]
    lib.sp_oracle_project.argtypes = [P, c.c_int64, P, c.c_int64, P, c.c_int64, P, P, P, P]
    _lib = lib
    return lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid arguments (code {rc})")


def max_threads() -> int:
    return int(_load().sp_oracle_max_threads())


def set_threads(n: int) -> None:
    _load().sp_oracle_set_threads(int(n))


def _k_strides(k_layer: np.ndarray, layout: str) -> Tuple[int, int, int, int, int]:
    """(stride_token, stride_head, Hkv, L, d) in elements for a contiguous layer array."""
    if layout == "HND":
        hkv, L, d = k_layer.shape
        return d, L * d, hkv, L, d
    if layout == "NHD":
        L, hkv, d = k_layer.shape
        return hkv * d, d, hkv, L, d
    raise ValueError("layout must be 'HND' or 'NHD'")


def logits_layer(q_layer: np.ndarray, k_layer: np.ndarray, scale: float, layout: str = "HND") -> np.ndarray:
    """Scaled logits of one layer, float64 [H][n_q][L]. q_layer: uint16 [H][n_q][d]."""
    q_layer = np.ascontiguousarray(q_layer, dtype=np.uint16)
    k_layer = np.ascontiguousarray(k_layer, dtype=np.uint16)
    H, n_q, d = q_layer.shape
    st, sh, hkv, L, dk = _k_strides(k_layer, layout)
    if dk != d:
        raise ValueError("head_dim mismatch")
    s = np.empty((H, n_q, L), dtype=np.float64)
    _check(_load().sp_oracle_logits_layer(_ptr(q_layer), _ptr(k_layer), st, sh, H, hkv, n_q, d, L,
                                          float(scale), _ptr(s)), "logits_layer")
    return s


def softmax_rows(s: np.ndarray, return_stats: bool = False):
    """Row softmax over the last axis (copy). Optionally also (row_max, row_sum)."""
    p = np.array(s, dtype=np.float64, order="C", copy=True)
    L = p.shape[-1]
    rows = p.size // L
    m = np.empty(rows, dtype=np.float64)
    l = np.empty(rows, dtype=np.float64)
    _check(_load().sp_oracle_softmax_rows(_ptr(p), rows, L, _ptr(m), _ptr(l)), "softmax_rows")
    if return_stats:
        return p, m.reshape(p.shape[:-1]), l.reshape(p.shape[:-1])
    return p


def score(q: np.ndarray, k_layers: Sequence[np.ndarray], scale: float, layer_agg: int = LAYER_MEAN,
          layout: str = "HND") -> np.ndarray:
    """Token importance I[L] (float64). q: uint16 [Lyr][H][n_q][d]; k_layers: list of uint16 layer arrays."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    Lyr, H, n_q, d = q.shape
    if len(k_layers) != Lyr:
        raise ValueError("need one K array per layer")
    ks = [np.ascontiguousarray(k, dtype=np.uint16) for k in k_layers]
    st, sh, hkv, L, dk = _k_strides(ks[0], layout)
    for k in ks:
        if k.shape != ks[0].shape:
            raise ValueError("K layers must share a shape")
    if dk != d:
        raise ValueError("head_dim mismatch")
    ptrs = (ctypes.c_void_p * Lyr)(*[k.ctypes.data for k in ks])
    out = np.empty(L, dtype=np.float64)
    _check(_load().sp_oracle_score(_ptr(q), ctypes.cast(ptrs, ctypes.c_void_p), st, sh, Lyr, H, hkv, n_q,
                                   d, L, float(scale), int(layer_agg), _ptr(out)), "score")
    return out


def e4m3_to_f64(codes: np.ndarray) -> np.ndarray:
    """Values of E4M3 codes (uint8, any shape) as float64; the all-ones codes are NaN."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    lib = _load()
    table = np.array([lib.sp_oracle_e4m3_to_f64(b) for b in range(256)], dtype=np.float64)
    return table[codes]


def logits_layer_fp8(q_layer: np.ndarray, k8_layer: np.ndarray, kscale: np.ndarray, scale: float,
                     layout: str = "HND") -> np.ndarray:
    """Scaled logits of one layer over quantised keys, float64 [H][n_q][L]. k8_layer: uint8 E4M3 codes,
    kscale: [Hkv] scales."""
    q_layer = np.ascontiguousarray(q_layer, dtype=np.uint16)
    k8_layer = np.ascontiguousarray(k8_layer, dtype=np.uint8)
    H, n_q, d = q_layer.shape
    st, sh, hkv, L, dk = _k_strides(k8_layer, layout)
    ksc = np.ascontiguousarray(kscale, dtype=np.float64)
    if dk != d or ksc.shape != (hkv,):
        raise ValueError("shape mismatch")
    s = np.empty((H, n_q, L), dtype=np.float64)
    _check(_load().sp_oracle_logits_layer_fp8(_ptr(q_layer), _ptr(k8_layer), st, sh, H, hkv, n_q, d, L, _ptr(ksc),
                                              float(scale), _ptr(s)), "logits_layer_fp8")
    return s


def score_fp8(q: np.ndarray, k8_layers: Sequence[np.ndarray], kscale: np.ndarray, scale: float,
              layer_agg: int = LAYER_MEAN, layout: str = "HND") -> np.ndarray:
    """Token importance over quantised keys. k8_layers: uint8 E4M3 codes per layer; kscale: [Lyr][Hkv]."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    Lyr, H, n_q, d = q.shape
    if len(k8_layers) != Lyr:
        raise ValueError("need one K array per layer")
    ks = [np.ascontiguousarray(k, dtype=np.uint8) for k in k8_layers]
    st, sh, hkv, L, dk = _k_strides(ks[0], layout)
    ksc = np.ascontiguousarray(kscale, dtype=np.float64)
    if dk != d or ksc.shape != (Lyr, hkv) or any(k.shape != ks[0].shape for k in ks):
        raise ValueError("shape mismatch")
    ptrs = (ctypes.c_void_p * Lyr)(*[k.ctypes.data for k in ks])
    out = np.empty(L, dtype=np.float64)
    _check(_load().sp_oracle_score_fp8(_ptr(q), ctypes.cast(ptrs, ctypes.c_void_p), st, sh, Lyr, H, hkv, n_q, d, L,
                                       _ptr(ksc), float(scale), int(layer_agg), _ptr(out)), "score_fp8")
    return out


def score_look(q: np.ndarray, k_layers: Sequence[np.ndarray], k_look: np.ndarray, look_self: int, scale: float,
               layer_agg: int = LAYER_MEAN, layout: str = "HND") -> np.ndarray:
    """Token importance with the lookahead keys in every row's normaliser. k_look: uint16 [Lyr][Hkv][n_q][d];
    row n sees lookahead keys 0..n-1, and key n too when look_self is 1."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    Lyr, H, n_q, d = q.shape
    if len(k_layers) != Lyr:
        raise ValueError("need one K array per layer")
    ks = [np.ascontiguousarray(k, dtype=np.uint16) for k in k_layers]
    st, sh, hkv, L, dk = _k_strides(ks[0], layout)
    for k in ks:
        if k.shape != ks[0].shape:
            raise ValueError("K layers must share a shape")
    k_look = np.ascontiguousarray(k_look, dtype=np.uint16)
    if dk != d or k_look.shape != (Lyr, hkv, n_q, d):
        raise ValueError("head_dim or k_look shape mismatch")
    ptrs = (ctypes.c_void_p * Lyr)(*[k.ctypes.data for k in ks])
    out = np.empty(L, dtype=np.float64)
    _check(_load().sp_oracle_score_look(_ptr(q), ctypes.cast(ptrs, ctypes.c_void_p), st, sh, Lyr, H, hkv, n_q,
                                        d, L, float(scale), int(layer_agg), _ptr(k_look), int(look_self),
                                        _ptr(out)), "score_look")
    return out


def gather_pages(pool_l: np.ndarray, block_table: np.ndarray, L: int, layout: str = "HND") -> np.ndarray:
    """Contiguous keys of one layer from a paged cache (Section 3.1: KV caches kept in fixed-size
    blocks): token j is row j % P of page block_table[j // P]. pool_l: [pages][Hkv][P][d] ("HND") or
    [pages][P][Hkv][d] ("NHD"); returns [Hkv][L][d] or [L][Hkv][d]. Paging is addressing only: the
    paged score is the plain score of the gathered keys."""
    P = pool_l.shape[2] if layout == "HND" else pool_l.shape[1]
    j = np.arange(L)
    page, row = np.asarray(block_table)[j // P], j % P
    if layout == "HND":
        return np.ascontiguousarray(pool_l[page, :, row, :].transpose(1, 0, 2))
    return np.ascontiguousarray(pool_l[page, row, :, :])


def pool(I: np.ndarray, w: int) -> np.ndarray:
    I = np.ascontiguousarray(I, dtype=np.float64)
    out = np.empty_like(I)
    _check(_load().sp_oracle_pool(_ptr(I), I.size, int(w), _ptr(out)), "pool")
    return out


def chunk_mean(P: np.ndarray, c: int) -> np.ndarray:
    P = np.ascontiguousarray(P, dtype=np.float64)
    if int(c) < 1:
        raise ValueError("oracle chunk_mean: chunk must be >= 1")
    C = (P.size + c - 1) // c
    out = np.empty(C, dtype=np.float64)
    _check(_load().sp_oracle_chunk_mean(_ptr(P), P.size, int(c), _ptr(out)), "chunk_mean")
    return out


def keep_count(C: int, num: int, den: int) -> int:
    k = int(_load().sp_oracle_keep_count(int(C), int(num), int(den)))
    if k < 0:
        raise ValueError("oracle keep_count: invalid arguments")
    return k


def topk(cs: np.ndarray, k: int) -> np.ndarray:
    cs = np.ascontiguousarray(cs, dtype=np.float64)
    if not (1 <= int(k) <= cs.size):
        raise ValueError("oracle topk: k out of range")
    sel = np.empty(int(k), dtype=np.int64)
    _check(_load().sp_oracle_topk(_ptr(cs), cs.size, int(k), _ptr(sel)), "topk")
    return sel


def merge(sel: np.ndarray, c: int, L: int) -> np.ndarray:
    sel = np.ascontiguousarray(sel, dtype=np.int64)
    spans = np.empty((max(sel.size, 1), 2), dtype=np.int64)
    n = int(_load().sp_oracle_merge(_ptr(sel), sel.size, int(c), int(L), _ptr(spans)))
    if n < 0:
        raise ValueError("oracle merge: invalid arguments")
    return spans[:n].copy()


def project(draft_off: np.ndarray, target_off: np.ndarray, spans: np.ndarray):
    """Returns (target_spans [n][2] int64, keep_mask [M] uint8, n_kept)."""
    draft_off = np.ascontiguousarray(draft_off, dtype=np.int64)
    target_off = np.ascontiguousarray(target_off, dtype=np.int64)
    spans = np.ascontiguousarray(spans, dtype=np.int64).reshape(-1, 2)
    L, M = draft_off.size - 1, target_off.size - 1
    mask = np.zeros(max(M, 1), dtype=np.uint8)
    tspans = np.empty((max(M, 1), 2), dtype=np.int64)
    n_t = np.zeros(1, dtype=np.int64)
    n_k = np.zeros(1, dtype=np.int64)
    _check(_load().sp_oracle_project(_ptr(draft_off), L, _ptr(target_off), M, _ptr(spans), spans.shape[0],
                                     _ptr(mask), _ptr(tspans), _ptr(n_t), _ptr(n_k)), "project")
    return tspans[: int(n_t[0])].copy(), mask[:M], int(n_k[0])


def assemble(target_ids: np.ndarray, tspans: np.ndarray, delim_ids: np.ndarray):
    """Returns (out_ids int32[n], out_pos int32[n], out_src int64[n]) of the compressed target prompt."""
    target_ids = np.ascontiguousarray(target_ids, dtype=np.int32)
    tspans = np.ascontiguousarray(tspans, dtype=np.int64).reshape(-1, 2)
    delim_ids = np.ascontiguousarray(delim_ids, dtype=np.int32)
    cap = int(np.sum(tspans[:, 1] - tspans[:, 0])) + max(tspans.shape[0] - 1, 0) * delim_ids.size if tspans.size else 0
    cap = max(cap, 1)
    ids = np.empty(cap, dtype=np.int32)
    pos = np.empty(cap, dtype=np.int32)
    src = np.empty(cap, dtype=np.int64)
    n = np.zeros(1, dtype=np.int64)
    _check(_load().sp_oracle_assemble(_ptr(target_ids), target_ids.size, _ptr(tspans) if tspans.size else None,
                                      tspans.shape[0], _ptr(delim_ids) if delim_ids.size else None, delim_ids.size,
                                      _ptr(ids), _ptr(pos), _ptr(src), _ptr(n)), "assemble")
    k = int(n[0])
    return ids[:k].copy(), pos[:k].copy(), src[:k].copy()


def select(I: np.ndarray, w: int, c: int, k: int):
    """Pool -> chunk means -> top-k -> merge. Returns (sel, spans, chunk_scores)."""
    cs = chunk_mean(pool(I, w), c)
    sel = topk(cs, k)
    return sel, merge(sel, c, I.size), cs


def budget_keep(cs: np.ndarray, c: int, draft_off: np.ndarray, target_off: np.ndarray, budget: int):
    """Budget-targeted keep (Section 3.1: the compressed prompt is to have a fixed target-side length,
    a multiple of the KV block size): the largest k in 1..C for which the top-k chunks, merged and
    projected onto the target tokenisation, keep at most `budget` target tokens; 1 if even one chunk
    keeps more. Plain search: every k is tried with the same steps the pipeline uses (topk, merge,
    project). Returns (k, n_kept at that k). For small inputs: the cost is C full projections."""
    cs = np.ascontiguousarray(cs, dtype=np.float64)
    L = int(np.asarray(draft_off).size) - 1
    best_k, best_kept = 1, None
    for k in range(1, cs.size + 1):
        _, _, n_kept = project(draft_off, target_off, merge(topk(cs, k), c, L))
        if k == 1:
            best_kept = n_kept
        if n_kept <= int(budget):
            best_k, best_kept = k, n_kept
    return best_k, best_kept

