"""ctypes binding of the C ABI in ``include/sp.h``.

Argument marshalling only: every function takes torch tensors (device memory
owned by the caller) and plain integers, passes raw pointers to the library and
turns a non-zero status into :class:`SpError`. Nothing is computed here and
there is no fallback: if ``libsp_amd.so`` is missing the call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

SP_LAYER_MEAN = 0
SP_LAYER_MAX = 1

_STATUS = {1: "SP_ERR_INVALID_ARG", 2: "SP_ERR_UNSUPPORTED", 3: "SP_ERR_WORKSPACE", 4: "SP_ERR_DEVICE"}

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG_DIR, "libsp_amd.so")

EXPORTS = (
    "sp_score_workspace", "sp_score", "sp_score_look", "sp_score_paged", "sp_score_is_fused", "sp_score_batch", "sp_keep_count", "sp_select_workspace",
    "sp_select", "sp_select_static", "sp_select_budget_workspace", "sp_select_budget", "sp_project", "sp_assemble_workspace", "sp_assemble", "sp_last_error", "sp_version",
    "sp_debug_fused_giveup",
)


class SpError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status
        self.message = message


class ScoreDesc(ctypes.Structure):
    """Mirror of ``sp_score_desc``."""
    _fields_ = [
        ("n_layers", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("n_q", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("layer_agg", ctypes.c_int32),
        ("k_stride_token", ctypes.c_int64),
        ("k_stride_head", ctypes.c_int64),
    ]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads ``libsp_amd.so`` (built in-tree by ``paper_2603_02631_amd/build.py``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2603_02631_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    P = c.c_void_p
    D = c.POINTER(ScoreDesc)
    lib.sp_score_workspace.argtypes = [D, c.c_int64, c.c_int32, c.POINTER(c.c_size_t)]
    lib.sp_score.argtypes = [D, P, c.POINTER(P), c.c_int64, P, P, c.c_size_t, P]
    lib.sp_score_look.argtypes = [D, P, c.POINTER(P), c.c_int64, P, c.c_int32, P, P, c.c_size_t, P]
    lib.sp_score_paged.argtypes = [D, P, c.POINTER(P), P, c.c_int64, c.c_int64, c.c_int64, P, P, c.c_size_t, P]
    lib.sp_score_batch.argtypes = [D, P, c.POINTER(P), c.POINTER(c.c_int64), P, c.c_int32, P, P, c.c_size_t, P]
    lib.sp_score_is_fused.argtypes = [D, c.c_int64]
    lib.sp_score_is_fused.restype = c.c_int32
    lib.sp_keep_count.argtypes = [c.c_int64, c.c_int64, c.c_int64]
    lib.sp_keep_count.restype = c.c_int64
    lib.sp_select_workspace.argtypes = [c.c_int64, c.c_int32, c.POINTER(c.c_size_t)]
    lib.sp_select.argtypes = [P, c.c_int64, c.c_int32, c.c_int32, c.c_int64, P, P, P, P, P, c.c_size_t, P]
    lib.sp_select_static.argtypes = [P, c.c_int64, c.c_int32, c.c_int32, c.c_int64, P, P, P, P, P]
    lib.sp_select_budget_workspace.argtypes = [c.c_int64, c.c_int32, c.POINTER(c.c_size_t)]
    lib.sp_select_budget.argtypes = [P, c.c_int64, c.c_int32, c.c_int32, P, P, c.c_int64, c.c_int64, P, P, P, P, P, P,
                                     P, c.c_size_t, P]
    lib.sp_project.argtypes = [P, c.c_int64, P, c.c_int64, P, P, c.c_int32, P, P, P, P, P]
    lib.sp_assemble_workspace.argtypes = [c.c_int32, c.POINTER(c.c_size_t)]
    lib.sp_assemble.argtypes = [P, c.c_int64, P, P, c.c_int32, P, c.c_int32, c.c_int64, P, P, P, P, P, c.c_size_t, P]
    lib.sp_debug_fused_giveup.argtypes = [c.c_uint32, c.c_int32]
    lib.sp_debug_fused_giveup.restype = None
    lib.sp_last_error.restype = c.c_char_p
    lib.sp_version.restype = c.c_char_p
    for name in ("sp_score_workspace", "sp_score", "sp_score_look", "sp_score_paged", "sp_score_is_fused", "sp_score_batch", "sp_select_workspace", "sp_select",
                 "sp_select_static", "sp_select_budget_workspace", "sp_select_budget", "sp_project", "sp_assemble_workspace", "sp_assemble"):
        getattr(lib, name).restype = c.c_int
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        raise SpError(status, sp_last_error())


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a tensor; None passes NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def sp_last_error() -> str:
    return load_library().sp_last_error().decode()


def sp_version() -> str:
    return load_library().sp_version().decode()


def sp_debug_fused_giveup(spin_limit: int = 1 << 20, force_miss: int = 0) -> None:
    """Test hook: see ``sp_debug_fused_giveup`` in ``include/sp.h``."""
    load_library().sp_debug_fused_giveup(int(spin_limit), int(force_miss))


def sp_keep_count(n_chunks: int, keep_num: int, keep_den: int) -> int:
    return int(load_library().sp_keep_count(n_chunks, keep_num, keep_den))


def sp_score_workspace(desc: ScoreDesc, total_tokens: int, n_prompts: int = 1) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().sp_score_workspace(ctypes.byref(desc), total_tokens, n_prompts, ctypes.byref(n)))
    return int(n.value)


def sp_score_is_fused(desc: ScoreDesc, L: int) -> int:
    return int(load_library().sp_score_is_fused(ctypes.byref(desc), L))


def _layer_array(k_layers: Sequence):
    return (ctypes.c_void_p * len(k_layers))(*[_ptr(k) for k in k_layers])


def sp_score(desc: ScoreDesc, q, k_layers: Sequence, L: int, scores, ws, ws_bytes: Optional[int] = None,
             stream=None) -> None:
    if len(k_layers) != desc.n_layers:
        raise SpError(1, f"k_layers has {len(k_layers)} entries, desc.n_layers is {desc.n_layers}")
    nbytes = ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)
    _check(load_library().sp_score(ctypes.byref(desc), _ptr(q), _layer_array(k_layers), L, _ptr(scores), _ptr(ws),
                                   nbytes, _stream(stream)))


def sp_score_look(desc: ScoreDesc, q, k_layers: Sequence, L: int, k_look, look_self: int, scores, ws,
                  ws_bytes: Optional[int] = None, stream=None) -> None:
    if len(k_layers) != desc.n_layers:
        raise SpError(1, f"k_layers has {len(k_layers)} entries, desc.n_layers is {desc.n_layers}")
    nbytes = ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)
    _check(load_library().sp_score_look(ctypes.byref(desc), _ptr(q), _layer_array(k_layers), L, _ptr(k_look),
                                        int(look_self), _ptr(scores), _ptr(ws), nbytes, _stream(stream)))


def sp_score_paged(desc: ScoreDesc, q, k_pools: Sequence, block_table, page_tokens: int, page_stride: int, L: int,
                   scores, ws, ws_bytes: Optional[int] = None, stream=None) -> None:
    if len(k_pools) != desc.n_layers:
        raise SpError(1, f"k_pools has {len(k_pools)} entries, desc.n_layers is {desc.n_layers}")
    nbytes = ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)
    _check(load_library().sp_score_paged(ctypes.byref(desc), _ptr(q), _layer_array(k_pools), _ptr(block_table),
                                         int(page_tokens), int(page_stride), L, _ptr(scores), _ptr(ws), nbytes,
                                         _stream(stream)))


def sp_score_batch(desc: ScoreDesc, q, k_layers: Sequence, offsets_host: Sequence[int], offsets_dev, scores, ws,
                   ws_bytes: Optional[int] = None, stream=None) -> None:
    if len(k_layers) != desc.n_layers:
        raise SpError(1, f"k_layers has {len(k_layers)} entries, desc.n_layers is {desc.n_layers}")
    B = len(offsets_host) - 1
    off = (ctypes.c_int64 * (B + 1))(*[int(v) for v in offsets_host])
    nbytes = ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)
    _check(load_library().sp_score_batch(ctypes.byref(desc), _ptr(q), _layer_array(k_layers), off, _ptr(offsets_dev),
                                         B, _ptr(scores), _ptr(ws), nbytes, _stream(stream)))


def sp_select_workspace(L: int, chunk: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().sp_select_workspace(L, chunk, ctypes.byref(n)))
    return int(n.value)


def sp_select(scores, L: int, pool_w: int, chunk: int, k: int, sel_chunks, spans, n_spans, chunk_scores, ws,
              ws_bytes: Optional[int] = None, stream=None) -> None:
    nbytes = ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)
    _check(load_library().sp_select(_ptr(scores), L, pool_w, chunk, k, _ptr(sel_chunks), _ptr(spans), _ptr(n_spans),
                                    _ptr(chunk_scores), _ptr(ws), nbytes, _stream(stream)))


def sp_select_static(scores, L: int, pool_w: int, chunk: int, k: int, sel_chunks, spans, n_spans, chunk_scores,
                     stream=None) -> None:
    _check(load_library().sp_select_static(_ptr(scores), L, pool_w, chunk, k, _ptr(sel_chunks), _ptr(spans),
                                           _ptr(n_spans), _ptr(chunk_scores), _stream(stream)))


def sp_select_budget_workspace(L: int, chunk: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().sp_select_budget_workspace(L, chunk, ctypes.byref(n)))
    return int(n.value)


def sp_select_budget(scores, L: int, pool_w: int, chunk: int, draft_off, target_off, M: int, budget: int, sel_chunks,
                     spans, n_spans, k_out, n_kept, chunk_scores, ws, ws_bytes: Optional[int] = None,
                     stream=None) -> None:
    nbytes = ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)
    _check(load_library().sp_select_budget(_ptr(scores), L, pool_w, chunk, _ptr(draft_off), _ptr(target_off), M,
                                           budget, _ptr(sel_chunks), _ptr(spans), _ptr(n_spans), _ptr(k_out),
                                           _ptr(n_kept), _ptr(chunk_scores), _ptr(ws), nbytes, _stream(stream)))


def sp_project(draft_off, L: int, target_off, M: int, spans, n_spans, max_spans: int, tspans, n_tspans, keep_mask,
               n_kept, stream=None) -> None:
    _check(load_library().sp_project(_ptr(draft_off), L, _ptr(target_off), M, _ptr(spans), _ptr(n_spans), max_spans,
                                     _ptr(tspans), _ptr(n_tspans), _ptr(keep_mask), _ptr(n_kept), _stream(stream)))


def sp_assemble_workspace(max_spans: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().sp_assemble_workspace(max_spans, ctypes.byref(n)))
    return int(n.value)


def sp_assemble(target_ids, M: int, tspans, n_tspans, max_spans: int, delim_ids, n_delim: int, out_capacity: int,
                out_ids, out_pos, out_src, out_len, ws, ws_bytes: Optional[int] = None, stream=None) -> None:
    nbytes = ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)
    _check(load_library().sp_assemble(_ptr(target_ids), M, _ptr(tspans), _ptr(n_tspans), max_spans, _ptr(delim_ids),
                                      n_delim, out_capacity, _ptr(out_ids), _ptr(out_pos), _ptr(out_src),
                                      _ptr(out_len), _ptr(ws), nbytes, _stream(stream)))
