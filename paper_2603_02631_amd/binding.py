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
    "sp_score_workspace", "sp_score", "sp_score_look", "sp_score_paged", "sp_score_fp8", "sp_score_is_fused", "sp_score_fp8_is_fused", "sp_score_batch", "sp_score_batch_is_fused", "sp_keep_count", "sp_select_workspace",
    "sp_select", "sp_select_static", "sp_select_batch_workspace", "sp_select_batch", "sp_select_budget_workspace", "sp_select_budget", "sp_project", "sp_project_batch",
    "sp_assemble_workspace", "sp_assemble", "sp_last_error", "sp_version",
    "sp_debug_fused_giveup", "sp_hbm_read_probe",
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
    lib.sp_score_fp8.argtypes = [D, P, c.POINTER(P), P, c.c_int64, P, P, c.c_size_t, P]
    lib.sp_score_batch.argtypes = [D, P, c.POINTER(P), c.POINTER(c.c_int64), P, c.c_int32, P, P, c.c_size_t, P]
    lib.sp_score_batch_is_fused.argtypes = [D, c.POINTER(c.c_int64), c.c_int32]
    lib.sp_score_batch_is_fused.restype = c.c_int32
    lib.sp_score_is_fused.argtypes = [D, c.c_int64]
    lib.sp_score_is_fused.restype = c.c_int32
    lib.sp_score_fp8_is_fused.argtypes = [D, c.c_int64]
    lib.sp_score_fp8_is_fused.restype = c.c_int32
    lib.sp_keep_count.argtypes = [c.c_int64, c.c_int64, c.c_int64]
    lib.sp_keep_count.restype = c.c_int64
    lib.sp_select_workspace.argtypes = [c.c_int64, c.c_int32, c.POINTER(c.c_size_t)]
    lib.sp_select.argtypes = [P, c.c_int64, c.c_int32, c.c_int32, c.c_int64, P, P, P, P, P, c.c_size_t, P]
    lib.sp_select_static.argtypes = [P, c.c_int64, c.c_int32, c.c_int32, c.c_int64, P, P, P, P, P]
    I64P = c.POINTER(c.c_int64)
    lib.sp_select_batch_workspace.argtypes = [c.c_int64, c.c_int32, c.c_int32, c.POINTER(c.c_size_t)]
    lib.sp_select_batch.argtypes = [P, I64P, P, c.c_int32, c.c_int32, c.c_int32, I64P, P, P, P, P, P, P, c.c_size_t, P]
    lib.sp_project_batch.argtypes = [P, I64P, P, P, I64P, P, c.c_int32, P, P, I64P, P, P, P, P, P, P]
    lib.sp_select_budget_workspace.argtypes = [c.c_int64, c.c_int32, c.POINTER(c.c_size_t)]
    lib.sp_select_budget.argtypes = [P, c.c_int64, c.c_int32, c.c_int32, P, P, c.c_int64, c.c_int64, P, P, P, P, P, P,
                                     P, c.c_size_t, P]
    lib.sp_project.argtypes = [P, c.c_int64, P, c.c_int64, P, P, c.c_int32, P, P, P, P, P]
    lib.sp_assemble_workspace.argtypes = [c.c_int32, c.POINTER(c.c_size_t)]
    lib.sp_assemble.argtypes = [P, c.c_int64, P, P, c.c_int32, P, c.c_int32, c.c_int64, P, P, P, P, P, c.c_size_t, P]
    lib.sp_hbm_read_probe.argtypes = [P, c.c_size_t, P, P]
    lib.sp_hbm_read_probe.restype = c.c_int
    lib.sp_debug_fused_giveup.argtypes = [c.c_uint32, c.c_int32]
    lib.sp_debug_fused_giveup.restype = None
    lib.sp_last_error.restype = c.c_char_p
    lib.sp_version.restype = c.c_char_p
    for name in ("sp_score_workspace", "sp_score", "sp_score_look", "sp_score_paged", "sp_score_fp8", "sp_score_is_fused", "sp_score_batch", "sp_select_workspace", "sp_select",
                 "sp_select_static", "sp_select_batch_workspace", "sp_select_batch", "sp_select_budget_workspace", "sp_select_budget", "sp_project",
                 "sp_project_batch", "sp_assemble_workspace", "sp_assemble"):
        getattr(lib, name).restype = c.c_int
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        raise SpError(status, sp_last_error())


def _ptr(t, what: str = "buffer", nbytes: int = 0) -> Optional[int]:
    """Device address of a tensor; None passes NULL, an int is taken as a raw address.

    A tensor is checked before its address leaves Python: it has to live on the GPU, be contiguous
    and hold at least ``nbytes`` bytes (what the call will read or write), so that a short or
    host-side buffer becomes an :class:`SpError` instead of an out-of-bounds device access."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not getattr(t, "is_cuda", False):
        raise SpError(1, f"{what} is not a device tensor")
    if not t.is_contiguous():
        raise SpError(1, f"{what} is not contiguous")
    have = t.numel() * t.element_size()
    if have < nbytes:
        raise SpError(1, f"{what} holds {have} bytes, the call needs {nbytes}")
    return t.data_ptr()


def _q_bytes(desc: "ScoreDesc", n_prompts: int = 1) -> int:
    return n_prompts * desc.n_layers * desc.n_q_heads * desc.n_q * desc.head_dim * 2


def _k_bytes(desc: "ScoreDesc", tokens: int) -> int:
    """Bytes a layer's K buffer must hold for `tokens` tokens under the desc's strides."""
    if tokens <= 0:
        return 0
    return ((desc.n_kv_heads - 1) * desc.k_stride_head + (tokens - 1) * desc.k_stride_token + desc.head_dim) * 2


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


def sp_hbm_read_probe(buf, nbytes: int, sink, stream=None) -> None:
    _check(load_library().sp_hbm_read_probe(_ptr(buf, "buf", nbytes), nbytes, _ptr(sink, "sink", 8), _stream(stream)))


def sp_keep_count(n_chunks: int, keep_num: int, keep_den: int) -> int:
    return int(load_library().sp_keep_count(n_chunks, keep_num, keep_den))


def sp_score_workspace(desc: ScoreDesc, total_tokens: int, n_prompts: int = 1) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().sp_score_workspace(ctypes.byref(desc), total_tokens, n_prompts, ctypes.byref(n)))
    return int(n.value)


def sp_score_is_fused(desc: ScoreDesc, L: int) -> int:
    return int(load_library().sp_score_is_fused(ctypes.byref(desc), L))


def sp_score_fp8_is_fused(desc: ScoreDesc, L: int) -> int:
    return int(load_library().sp_score_fp8_is_fused(ctypes.byref(desc), L))


def sp_score_batch_is_fused(desc: ScoreDesc, offsets_host: Sequence[int]) -> int:
    B = len(offsets_host) - 1
    off = (ctypes.c_int64 * (B + 1))(*[int(v) for v in offsets_host])
    return int(load_library().sp_score_batch_is_fused(ctypes.byref(desc), off, B))


def _layer_array(k_layers: Sequence, nbytes: int = 0):
    return (ctypes.c_void_p * len(k_layers))(*[_ptr(k, f"k_layers[{i}]", nbytes) for i, k in enumerate(k_layers)])


def _ws_bytes(ws, ws_bytes: Optional[int]) -> int:
    have = 0 if ws is None or isinstance(ws, int) else ws.numel() * ws.element_size()
    if ws_bytes is None:
        return have
    if not isinstance(ws, int) and ws is not None and ws_bytes > have:
        raise SpError(3, f"ws_bytes = {ws_bytes} exceeds the workspace tensor ({have} bytes)")
    return ws_bytes


def sp_score(desc: ScoreDesc, q, k_layers: Sequence, L: int, scores, ws, ws_bytes: Optional[int] = None,
             stream=None) -> None:
    if len(k_layers) != desc.n_layers:
        raise SpError(1, f"k_layers has {len(k_layers)} entries, desc.n_layers is {desc.n_layers}")
    nbytes = _ws_bytes(ws, ws_bytes)
    _check(load_library().sp_score(ctypes.byref(desc), _ptr(q, "q", _q_bytes(desc)),
                                   _layer_array(k_layers, _k_bytes(desc, L)), L, _ptr(scores, "scores", 4 * max(L, 0)),
                                   _ptr(ws, "ws"), nbytes, _stream(stream)))


def sp_score_look(desc: ScoreDesc, q, k_layers: Sequence, L: int, k_look, look_self: int, scores, ws,
                  ws_bytes: Optional[int] = None, stream=None) -> None:
    if len(k_layers) != desc.n_layers:
        raise SpError(1, f"k_layers has {len(k_layers)} entries, desc.n_layers is {desc.n_layers}")
    nbytes = _ws_bytes(ws, ws_bytes)
    look_bytes = desc.n_layers * desc.n_kv_heads * desc.n_q * desc.head_dim * 2
    _check(load_library().sp_score_look(ctypes.byref(desc), _ptr(q, "q", _q_bytes(desc)),
                                        _layer_array(k_layers, _k_bytes(desc, L)), L, _ptr(k_look, "k_look", look_bytes),
                                        int(look_self), _ptr(scores, "scores", 4 * max(L, 0)), _ptr(ws, "ws"), nbytes,
                                        _stream(stream)))


def sp_score_paged(desc: ScoreDesc, q, k_pools: Sequence, block_table, page_tokens: int, page_stride: int, L: int,
                   scores, ws, ws_bytes: Optional[int] = None, stream=None) -> None:
    if len(k_pools) != desc.n_layers:
        raise SpError(1, f"k_pools has {len(k_pools)} entries, desc.n_layers is {desc.n_layers}")
    nbytes = _ws_bytes(ws, ws_bytes)
    n_pages = (max(L, 0) + page_tokens - 1) // page_tokens if page_tokens > 0 else 0
    _check(load_library().sp_score_paged(ctypes.byref(desc), _ptr(q, "q", _q_bytes(desc)), _layer_array(k_pools),
                                         _ptr(block_table, "block_table", 4 * n_pages), int(page_tokens),
                                         int(page_stride), L, _ptr(scores, "scores", 4 * max(L, 0)), _ptr(ws, "ws"),
                                         nbytes, _stream(stream)))


def sp_score_fp8(desc: ScoreDesc, q, k8_layers: Sequence, kscale, L: int, scores, ws, ws_bytes: Optional[int] = None,
                 stream=None) -> None:
    if len(k8_layers) != desc.n_layers:
        raise SpError(1, f"k8_layers has {len(k8_layers)} entries, desc.n_layers is {desc.n_layers}")
    nbytes = _ws_bytes(ws, ws_bytes)
    _check(load_library().sp_score_fp8(ctypes.byref(desc), _ptr(q, "q", _q_bytes(desc)),
                                       _layer_array(k8_layers, _k_bytes(desc, L) // 2),
                                       _ptr(kscale, "kscale", 4 * desc.n_layers * desc.n_kv_heads), L,
                                       _ptr(scores, "scores", 4 * max(L, 0)), _ptr(ws, "ws"), nbytes, _stream(stream)))


def sp_score_batch(desc: ScoreDesc, q, k_layers: Sequence, offsets_host: Sequence[int], offsets_dev, scores, ws,
                   ws_bytes: Optional[int] = None, stream=None) -> None:
    if len(k_layers) != desc.n_layers:
        raise SpError(1, f"k_layers has {len(k_layers)} entries, desc.n_layers is {desc.n_layers}")
    B = len(offsets_host) - 1
    off = (ctypes.c_int64 * (B + 1))(*[int(v) for v in offsets_host])
    nbytes = _ws_bytes(ws, ws_bytes)
    total = int(offsets_host[-1]) if B >= 0 else 0
    _check(load_library().sp_score_batch(ctypes.byref(desc), _ptr(q, "q", _q_bytes(desc, max(B, 0))),
                                         _layer_array(k_layers, _k_bytes(desc, total)), off,
                                         _ptr(offsets_dev, "offsets_dev", 8 * (B + 1)), B,
                                         _ptr(scores, "scores", 4 * max(total, 0)), _ptr(ws, "ws"), nbytes,
                                         _stream(stream)))


def sp_select_workspace(L: int, chunk: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().sp_select_workspace(L, chunk, ctypes.byref(n)))
    return int(n.value)


def sp_select(scores, L: int, pool_w: int, chunk: int, k: int, sel_chunks, spans, n_spans, chunk_scores, ws,
              ws_bytes: Optional[int] = None, stream=None) -> None:
    nbytes = _ws_bytes(ws, ws_bytes)
    C = (L + chunk - 1) // chunk if chunk > 0 and L > 0 else 0
    kk = max(int(k), 0)
    _check(load_library().sp_select(_ptr(scores, "scores", 4 * max(L, 0)), L, pool_w, chunk, k,
                                    _ptr(sel_chunks, "sel_chunks", 4 * kk), _ptr(spans, "spans", 16 * kk),
                                    _ptr(n_spans, "n_spans", 4), _ptr(chunk_scores, "chunk_scores", 4 * C),
                                    _ptr(ws, "ws"), nbytes, _stream(stream)))


def sp_select_static(scores, L: int, pool_w: int, chunk: int, k: int, sel_chunks, spans, n_spans, chunk_scores,
                     stream=None) -> None:
    C = (L + chunk - 1) // chunk if chunk > 0 and L > 0 else 0
    kk = max(int(k), 0)
    _check(load_library().sp_select_static(_ptr(scores, "scores", 4 * max(L, 0)), L, pool_w, chunk, k,
                                           _ptr(sel_chunks, "sel_chunks", 4 * kk), _ptr(spans, "spans", 16 * kk),
                                           _ptr(n_spans, "n_spans", 4), _ptr(chunk_scores, "chunk_scores", 4 * C),
                                           _stream(stream)))


def _host_i64(values: Sequence[int]):
    return (ctypes.c_int64 * len(values))(*[int(v) for v in values])


def sp_select_batch_workspace(total_tokens: int, B: int, chunk: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().sp_select_batch_workspace(total_tokens, B, chunk, ctypes.byref(n)))
    return int(n.value)


def sp_select_batch(scores, offsets_host: Sequence[int], offsets_dev, pool_w: int, chunk: int,
                    kept_off_host: Sequence[int], kept_off_dev, sel_chunks, spans, n_spans, chunk_scores, ws,
                    ws_bytes: Optional[int] = None, stream=None) -> None:
    B = len(offsets_host) - 1
    if len(kept_off_host) != B + 1:
        raise SpError(1, f"kept_off_host has {len(kept_off_host)} entries, offsets_host {B + 1}")
    total, kept = max(int(offsets_host[-1]), 0), max(int(kept_off_host[-1]), 0)
    n_cs = total // chunk + B + 1 if chunk > 0 else 0
    _check(load_library().sp_select_batch(
        _ptr(scores, "scores", 4 * total), _host_i64(offsets_host), _ptr(offsets_dev, "offsets_dev", 8 * (B + 1)), B,
        pool_w, chunk, _host_i64(kept_off_host), _ptr(kept_off_dev, "kept_off_dev", 8 * (B + 1)),
        _ptr(sel_chunks, "sel_chunks", 4 * kept), _ptr(spans, "spans", 16 * kept), _ptr(n_spans, "n_spans", 4 * B),
        _ptr(chunk_scores, "chunk_scores", 4 * n_cs), _ptr(ws, "ws"), _ws_bytes(ws, ws_bytes), _stream(stream)))


def sp_project_batch(draft_off, offsets_host: Sequence[int], offsets_dev, target_off, moffsets_host: Sequence[int],
                     moffsets_dev, spans, n_spans, kept_off_host: Sequence[int], kept_off_dev, tspans, n_tspans,
                     keep_mask, n_kept, stream=None) -> None:
    B = len(offsets_host) - 1
    if len(moffsets_host) != B + 1 or len(kept_off_host) != B + 1:
        raise SpError(1, "offsets_host, moffsets_host and kept_off_host must have the same length")
    total, m_total, kept = max(int(offsets_host[-1]), 0), max(int(moffsets_host[-1]), 0), max(int(kept_off_host[-1]), 0)
    _check(load_library().sp_project_batch(
        _ptr(draft_off, "draft_off", 8 * (total + B)), _host_i64(offsets_host),
        _ptr(offsets_dev, "offsets_dev", 8 * (B + 1)), _ptr(target_off, "target_off", 8 * (m_total + B)),
        _host_i64(moffsets_host), _ptr(moffsets_dev, "moffsets_dev", 8 * (B + 1)), B, _ptr(spans, "spans", 16 * kept),
        _ptr(n_spans, "n_spans", 4 * B), _host_i64(kept_off_host), _ptr(kept_off_dev, "kept_off_dev", 8 * (B + 1)),
        _ptr(tspans, "tspans", 16 * kept), _ptr(n_tspans, "n_tspans", 4 * B), _ptr(keep_mask, "keep_mask", m_total),
        _ptr(n_kept, "n_kept", 8 * B), _stream(stream)))


def sp_select_budget_workspace(L: int, chunk: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().sp_select_budget_workspace(L, chunk, ctypes.byref(n)))
    return int(n.value)


def sp_select_budget(scores, L: int, pool_w: int, chunk: int, draft_off, target_off, M: int, budget: int, sel_chunks,
                     spans, n_spans, k_out, n_kept, chunk_scores, ws, ws_bytes: Optional[int] = None,
                     stream=None) -> None:
    nbytes = _ws_bytes(ws, ws_bytes)
    C = (L + chunk - 1) // chunk if chunk > 0 and L > 0 else 0
    _check(load_library().sp_select_budget(_ptr(scores, "scores", 4 * max(L, 0)), L, pool_w, chunk,
                                           _ptr(draft_off, "draft_off", 8 * (max(L, 0) + 1)),
                                           _ptr(target_off, "target_off", 8 * (max(M, 0) + 1)), M, budget,
                                           _ptr(sel_chunks, "sel_chunks", 4 * C), _ptr(spans, "spans", 16 * C),
                                           _ptr(n_spans, "n_spans", 4), _ptr(k_out, "k_out", 8), _ptr(n_kept, "n_kept", 8),
                                           _ptr(chunk_scores, "chunk_scores", 4 * C), _ptr(ws, "ws"), nbytes,
                                           _stream(stream)))


def sp_project(draft_off, L: int, target_off, M: int, spans, n_spans, max_spans: int, tspans, n_tspans, keep_mask,
               n_kept, stream=None) -> None:
    cap = max(int(max_spans), 0)
    _check(load_library().sp_project(_ptr(draft_off, "draft_off", 8 * (max(L, 0) + 1)), L,
                                     _ptr(target_off, "target_off", 8 * (max(M, 0) + 1)), M,
                                     _ptr(spans, "spans", 16 * cap), _ptr(n_spans, "n_spans", 4), max_spans,
                                     _ptr(tspans, "tspans", 16 * cap), _ptr(n_tspans, "n_tspans", 4),
                                     _ptr(keep_mask, "keep_mask", max(M, 0)), _ptr(n_kept, "n_kept", 8), _stream(stream)))


def sp_assemble_workspace(max_spans: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().sp_assemble_workspace(max_spans, ctypes.byref(n)))
    return int(n.value)


def sp_assemble(target_ids, M: int, tspans, n_tspans, max_spans: int, delim_ids, n_delim: int, out_capacity: int,
                out_ids, out_pos, out_src, out_len, ws, ws_bytes: Optional[int] = None, stream=None) -> None:
    nbytes = _ws_bytes(ws, ws_bytes)
    cap = max(int(max_spans), 0)
    oc = max(int(out_capacity), 0)
    _check(load_library().sp_assemble(_ptr(target_ids, "target_ids", 4 * max(M, 0)), M, _ptr(tspans, "tspans", 16 * cap),
                                      _ptr(n_tspans, "n_tspans", 4), max_spans,
                                      _ptr(delim_ids, "delim_ids", 4 * max(int(n_delim), 0)), n_delim, out_capacity,
                                      _ptr(out_ids, "out_ids", 4 * oc), _ptr(out_pos, "out_pos", 4 * oc),
                                      _ptr(out_src, "out_src", 8 * oc), _ptr(out_len, "out_len", 8), _ptr(ws, "ws"),
                                      nbytes, _stream(stream)))
