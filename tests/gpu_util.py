"""Helpers that drive the C-ABI library from numpy inputs (GPU tests only).

torch is used for device memory and nothing else: every tensor here is a raw
buffer whose address is handed to the library.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

import paper_2603_02631_amd as sp

DEV = "cuda:0"


def dev_bits(a: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> device buffer (int16 view, same bytes)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint16).view(np.int16)).to(DEV)


def make_desc(n_layers, H, Hkv, d, n_q, scale, layer_agg, layout, T) -> sp.ScoreDesc:
    if layout == "HND":
        st, sh = d, T * d
    else:
        st, sh = Hkv * d, d
    return sp.ScoreDesc(n_layers, H, Hkv, d, n_q, float(scale), int(layer_agg), st, sh)


def workspace(nbytes: int) -> torch.Tensor:
    # filled with ones so that a status word nobody cleared reads as non-zero
    return torch.full((max(nbytes, 256),), 0xFF, dtype=torch.uint8, device=DEV)


def status_word(ws: torch.Tensor) -> int:
    """The 32-bit status word that leads a score workspace (0 = the scores are valid)."""
    return int(ws[:4].cpu().numpy().view(np.uint32)[0])


def gpu_score(q_bits: np.ndarray, k_layers: Sequence[np.ndarray], scale: float, layer_agg: int = 0,
              layout: str = "HND", k_dev: Optional[List[torch.Tensor]] = None) -> np.ndarray:
    """q_bits: uint16 [Lyr][H][n_q][d]; k_layers: uint16 [Hkv][L][d] (HND) or [L][Hkv][d] (NHD)."""
    Lyr, H, n_q, d = q_bits.shape
    if layout == "HND":
        Hkv, L, _ = k_layers[0].shape
    else:
        L, Hkv, _ = k_layers[0].shape
    desc = make_desc(Lyr, H, Hkv, d, n_q, scale, layer_agg, layout, L)
    qd = dev_bits(q_bits)
    kd = k_dev if k_dev is not None else [dev_bits(k) for k in k_layers]
    ws = workspace(sp.sp_score_workspace(desc, L, 1))
    scores = torch.full((max(L, 1),), float("nan"), dtype=torch.float32, device=DEV)
    sp.sp_score(desc, qd, kd, L, scores, ws)
    torch.cuda.synchronize()
    assert status_word(ws) == 0 or L == 0
    return scores[:L].cpu().numpy()


def gpu_score_look(q_bits: np.ndarray, k_layers: Sequence[np.ndarray], k_look: np.ndarray, look_self: int,
                   scale: float, layer_agg: int = 0, layout: str = "HND",
                   k_dev: Optional[List[torch.Tensor]] = None) -> np.ndarray:
    """gpu_score with the lookahead keys k_look (uint16 [Lyr][Hkv][n_q][d]) in the normaliser."""
    Lyr, H, n_q, d = q_bits.shape
    if layout == "HND":
        Hkv, L, _ = k_layers[0].shape
    else:
        L, Hkv, _ = k_layers[0].shape
    desc = make_desc(Lyr, H, Hkv, d, n_q, scale, layer_agg, layout, L)
    qd = dev_bits(q_bits)
    kd = k_dev if k_dev is not None else [dev_bits(k) for k in k_layers]
    kl = dev_bits(k_look)
    ws = workspace(sp.sp_score_workspace(desc, L, 1))
    scores = torch.full((max(L, 1),), float("nan"), dtype=torch.float32, device=DEV)
    sp.sp_score_look(desc, qd, kd, L, kl, look_self, scores, ws)
    torch.cuda.synchronize()
    assert status_word(ws) == 0
    return scores[:L].cpu().numpy()


def gpu_score_fp8(q_bits: np.ndarray, k8_layers: Sequence[np.ndarray], kscale: np.ndarray, scale: float,
                  layer_agg: int = 0, layout: str = "HND") -> np.ndarray:
    """q_bits: uint16 [Lyr][H][n_q][d]; k8_layers: uint8 E4M3 codes [Hkv][L][d] (HND) or [L][Hkv][d] (NHD);
    kscale: float32 [Lyr][Hkv]."""
    Lyr, H, n_q, d = q_bits.shape
    if layout == "HND":
        Hkv, L, _ = k8_layers[0].shape
    else:
        L, Hkv, _ = k8_layers[0].shape
    desc = make_desc(Lyr, H, Hkv, d, n_q, scale, layer_agg, layout, L)
    qd = dev_bits(q_bits)
    kd = [torch.from_numpy(np.ascontiguousarray(k, dtype=np.uint8)).to(DEV) for k in k8_layers]
    sc = torch.from_numpy(np.ascontiguousarray(kscale, dtype=np.float32)).to(DEV)
    ws = workspace(sp.sp_score_workspace(desc, L, 1))
    scores = torch.full((max(L, 1),), float("nan"), dtype=torch.float32, device=DEV)
    sp.sp_score_fp8(desc, qd, kd, sc, L, scores, ws)
    torch.cuda.synchronize()
    assert status_word(ws) == 0
    return scores[:L].cpu().numpy()


def make_paged(k_layers: Sequence[np.ndarray], page_tokens: int, layout: str, seed: int, spare_pages: int = 3):
    """Scatters contiguous head-major keys ([Hkv][L][d] per layer) into per-layer page pools in a random
    page order. Rows that hold no token (the tail of the last page, spare pages) are bf16 NaN: a kernel
    that lets them into a result is caught. Returns (pools list of uint16 arrays, block_table int32)."""
    Hkv, L, d = k_layers[0].shape
    n_pages = (L + page_tokens - 1) // page_tokens
    rng = np.random.default_rng(seed)
    table = rng.permutation(n_pages + spare_pages)[:n_pages].astype(np.int32)
    pools = []
    for k in k_layers:
        shape = (n_pages + spare_pages, Hkv, page_tokens, d) if layout == "HND" else (n_pages + spare_pages, page_tokens, Hkv, d)
        pool = np.full(shape, 0x7FC0, dtype=np.uint16)
        for p in range(n_pages):
            rows = k[:, p * page_tokens:(p + 1) * page_tokens, :]
            if layout == "HND":
                pool[table[p], :, :rows.shape[1], :] = rows
            else:
                pool[table[p], :rows.shape[1], :, :] = rows.transpose(1, 0, 2)
        pools.append(pool)
    return pools, table


def gpu_score_paged(q_bits: np.ndarray, pools: Sequence[np.ndarray], table: np.ndarray, page_tokens: int, L: int,
                    scale: float, layer_agg: int = 0, layout: str = "HND") -> np.ndarray:
    Lyr, H, n_q, d = q_bits.shape
    Hkv = pools[0].shape[1] if layout == "HND" else pools[0].shape[2]
    desc = make_desc(Lyr, H, Hkv, d, n_q, scale, layer_agg, layout, page_tokens)     # strides of one page
    qd = dev_bits(q_bits)
    pd = [dev_bits(p) for p in pools]
    td = torch.from_numpy(np.ascontiguousarray(table, dtype=np.int32)).to(DEV)
    ws = workspace(sp.sp_score_workspace(desc, L, 1))
    scores = torch.full((max(L, 1),), float("nan"), dtype=torch.float32, device=DEV)
    sp.sp_score_paged(desc, qd, pd, td, page_tokens, Hkv * page_tokens * d, L, scores, ws)
    torch.cuda.synchronize()
    assert status_word(ws) == 0
    return scores[:L].cpu().numpy()


def gpu_score_batch(q_bits: np.ndarray, k_layers: Sequence[np.ndarray], offsets: np.ndarray, scale: float,
                    layer_agg: int = 0, layout: str = "HND") -> np.ndarray:
    """q_bits: uint16 [B][Lyr][H][n_q][d]; k_layers packed along tokens."""
    B, Lyr, H, n_q, d = q_bits.shape
    T = int(offsets[-1])
    Hkv = k_layers[0].shape[0] if layout == "HND" else k_layers[0].shape[1]
    desc = make_desc(Lyr, H, Hkv, d, n_q, scale, layer_agg, layout, T)
    qd = dev_bits(q_bits)
    kd = [dev_bits(k) for k in k_layers]
    off_d = torch.from_numpy(np.ascontiguousarray(offsets, dtype=np.int64)).to(DEV)
    ws = workspace(sp.sp_score_workspace(desc, T, B))
    scores = torch.full((max(T, 1),), float("nan"), dtype=torch.float32, device=DEV)
    sp.sp_score_batch(desc, qd, kd, [int(v) for v in offsets], off_d, scores, ws)
    torch.cuda.synchronize()
    assert status_word(ws) == 0 or T == 0
    return scores[:T].cpu().numpy()


def gpu_select(scores: np.ndarray, pool_w: int, chunk: int, k: int, want_chunk_scores: bool = True):
    """Returns (sel int32[k], spans int64[n][2], chunk_scores float32[C] or None)."""
    L = scores.size
    C = (L + chunk - 1) // chunk
    sd = torch.from_numpy(np.ascontiguousarray(scores, dtype=np.float32)).to(DEV)
    sel = torch.full((k,), -1, dtype=torch.int32, device=DEV)
    spans = torch.full((k, 2), -1, dtype=torch.int64, device=DEV)
    n_spans = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    cs = torch.full((C,), float("nan"), dtype=torch.float32, device=DEV) if want_chunk_scores else None
    ws = workspace(sp.sp_select_workspace(L, chunk))
    sp.sp_select(sd, L, pool_w, chunk, k, sel, spans, n_spans, cs, ws)
    torch.cuda.synchronize()
    n = int(n_spans.item())
    return sel.cpu().numpy(), spans[:n].cpu().numpy(), (cs.cpu().numpy() if cs is not None else None)


def gpu_select_budget(scores: np.ndarray, pool_w: int, chunk: int, draft_off: np.ndarray, target_off: np.ndarray,
                      budget: int):
    """Returns (k, n_kept, sel int32[k], spans int64[n][2], chunk_scores float32[C])."""
    L, M = scores.size, target_off.size - 1
    C = (L + chunk - 1) // chunk
    sd = torch.from_numpy(np.ascontiguousarray(scores, dtype=np.float32)).to(DEV)
    dd = torch.from_numpy(np.ascontiguousarray(draft_off, dtype=np.int64)).to(DEV)
    td = torch.from_numpy(np.ascontiguousarray(target_off, dtype=np.int64)).to(DEV)
    sel = torch.full((C,), -1, dtype=torch.int32, device=DEV)
    spans = torch.full((C, 2), -1, dtype=torch.int64, device=DEV)
    n_spans = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    k_out = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    n_kept = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    cs = torch.full((C,), float("nan"), dtype=torch.float32, device=DEV)
    ws = workspace(sp.sp_select_budget_workspace(L, chunk))
    sp.sp_select_budget(sd, L, pool_w, chunk, dd, td, M, int(budget), sel, spans, n_spans, k_out, n_kept, cs, ws)
    torch.cuda.synchronize()
    k, n = int(k_out.item()), int(n_spans.item())
    assert 1 <= k <= C and 1 <= n <= k
    assert (sel[k:] == -1).all() and (spans[n:] == -1).all()      # nothing written beyond the k chosen
    return k, int(n_kept.item()), sel[:k].cpu().numpy(), spans[:n].cpu().numpy(), cs.cpu().numpy()


def gpu_project(draft_off: np.ndarray, target_off: np.ndarray, spans: np.ndarray, want_mask: bool = True,
                max_spans: Optional[int] = None):
    """Returns (tspans int64[n][2], mask uint8[M] or None, n_kept)."""
    L, M = draft_off.size - 1, target_off.size - 1
    spans = np.ascontiguousarray(spans, dtype=np.int64).reshape(-1, 2)
    ns = spans.shape[0]
    cap = max_spans if max_spans is not None else max(ns, 1)
    dd = torch.from_numpy(np.ascontiguousarray(draft_off, dtype=np.int64)).to(DEV)
    td = torch.from_numpy(np.ascontiguousarray(target_off, dtype=np.int64)).to(DEV)
    sp_buf = torch.zeros((cap, 2), dtype=torch.int64, device=DEV)
    if ns:
        sp_buf[:ns] = torch.from_numpy(spans).to(DEV)
    n_sp = torch.tensor([ns], dtype=torch.int32, device=DEV)
    tsp = torch.full((cap, 2), -1, dtype=torch.int64, device=DEV)
    n_t = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    mask = torch.full((M,), 7, dtype=torch.uint8, device=DEV) if want_mask else None
    n_kept = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    sp.sp_project(dd, L, td, M, sp_buf, n_sp, cap, tsp, n_t, mask, n_kept)
    torch.cuda.synchronize()
    n = int(n_t.item())
    return tsp[:n].cpu().numpy(), (mask.cpu().numpy() if mask is not None else None), int(n_kept.item())


def assert_scores_close(got: np.ndarray, want: np.ndarray, rel: float = 1e-3):
    """|g - o| <= rel * |o| + 1e-30 element by element."""
    got = got.astype(np.float64)
    assert got.shape == want.shape
    assert np.isfinite(got).all(), "non-finite GPU scores"
    err = np.abs(got - want)
    bound = rel * np.abs(want) + 1e-30
    bad = np.nonzero(err > bound)[0]
    assert bad.size == 0, (f"{bad.size} of {got.size} scores off; worst rel err "
                           f"{(err / np.maximum(np.abs(want), 1e-300)).max():.3e} at {int(np.argmax(err / np.maximum(np.abs(want), 1e-300)))}")
