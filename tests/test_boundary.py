"""CPU-side checks of the C-ABI boundary: the library loads, exports every
symbol the header declares, and rejects bad host-visible arguments before
anything is launched (so these calls never touch a GPU)."""
from __future__ import annotations

import ctypes
import os
import re

import pytest

import paper_2603_02631_amd as sp
from paper_2603_02631_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = sp.load_library()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert "gfx950" in sp.sp_version()


def test_keep_count_host_function():
    for line in open(os.path.join(ROOT, "tests", "golden", "keep_count.txt")):
        if line.startswith("#") or not line.strip():
            continue
        C, num, den, k = map(int, line.split())
        assert sp.sp_keep_count(C, num, den) == k
    assert sp.sp_keep_count(10, 0, 100) == 1
    assert sp.sp_keep_count(10, 1000, 100) == 10
    assert sp.sp_keep_count(0, 1, 2) == -1
    assert sp.sp_keep_count(5, 1, 0) == -1
    assert sp.sp_keep_count(5, -1, 2) == -1
    assert sp.sp_keep_count(2 ** 40, 2 ** 30, 2 ** 31) == 2 ** 39


def good_desc(**kw):
    base = dict(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=64, n_q=8, scale=0.125, layer_agg=0,
                k_stride_token=64, k_stride_head=64 * 1024)
    base.update(kw)
    return sp.ScoreDesc(*[base[f[0]] for f in sp.ScoreDesc._fields_])


@pytest.mark.parametrize("kw,status", [
    (dict(n_layers=0), 1), (dict(n_q_heads=5), 1), (dict(n_q=0), 1), (dict(scale=0.0), 1),
    (dict(scale=float("nan")), 1), (dict(scale=-1.0), 1), (dict(layer_agg=2), 1),
    (dict(k_stride_token=60), 1), (dict(k_stride_token=32), 1), (dict(k_stride_head=-8), 1),
    (dict(head_dim=96), 2), (dict(n_q=17), 2), (dict(n_layers=129), 2),
    (dict(n_q_heads=34, n_kv_heads=2), 2),
    (dict(n_q_heads=32, n_kv_heads=2, n_q=16, head_dim=128, k_stride_token=128), 2),
    # query groups beyond the on-chip staging: 16 heads x 16 rows at head_dim 64, 8 heads x 16 rows at head_dim 128
    (dict(n_q_heads=32, n_kv_heads=2, n_q=16), 2),
    (dict(n_q_heads=16, n_kv_heads=2, n_q=16, head_dim=128, k_stride_token=128), 2),
    (dict(n_q_heads=16, n_kv_heads=1, n_q=8, head_dim=128, k_stride_token=128), 2),
    # more (layer, kv head) pairs than a launch dimension holds
    (dict(n_layers=128, n_q_heads=512, n_kv_heads=512), 2),
])
def test_score_desc_validation(kw, status):
    with pytest.raises(sp.SpError) as e:
        sp.sp_score_workspace(good_desc(**kw), 1024, 1)
    assert e.value.status == status
    assert sp.sp_last_error() != ""


def test_score_workspace_and_argument_errors():
    d = good_desc()
    n = sp.sp_score_workspace(d, 1024, 1)
    assert n > 0 and n % 256 == 0
    assert sp.sp_score_workspace(d, 0, 1) >= 0
    with pytest.raises(sp.SpError):
        sp.sp_score_workspace(d, -1, 1)
    with pytest.raises(sp.SpError):
        sp.sp_score_workspace(d, 10, 0)
    lib = sp.load_library()
    assert lib.sp_score_workspace(None, 10, 1, ctypes.byref(ctypes.c_size_t())) == 1
    assert lib.sp_score_workspace(ctypes.byref(d), 10, 1, None) == 1

    fake = 0x1000  # never dereferenced: validation fails first
    layers = [fake, fake]
    with pytest.raises(sp.SpError) as e:        # null q
        sp.sp_score(d, None, layers, 1024, fake, fake, n, stream=0)
    assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:        # null layer pointer
        sp.sp_score(d, fake, [fake, None], 1024, fake, fake, n, stream=0)
    assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:        # misaligned layer pointer
        sp.sp_score(d, fake, [fake, fake + 2], 1024, fake, fake, n, stream=0)
    assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:        # negative length
        sp.sp_score(d, fake, layers, -5, fake, fake, n, stream=0)
    assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:        # workspace missing
        sp.sp_score(d, fake, layers, 1024, fake, None, 0, stream=0)
    assert e.value.status == 3
    with pytest.raises(sp.SpError) as e:        # workspace too small
        sp.sp_score(d, fake, layers, 1024, fake, fake, 256, stream=0)
    assert e.value.status == 3
    with pytest.raises(sp.SpError) as e:        # workspace misaligned
        sp.sp_score(d, fake, layers, 1024, fake, fake + 16, n, stream=0)
    assert e.value.status == 3
    with pytest.raises(sp.SpError):             # wrong number of layers (caught by the binding)
        sp.sp_score(d, fake, [fake], 1024, fake, fake, n, stream=0)
    sp.sp_score(d, fake, layers, 0, fake, None, 0, stream=0)   # empty prompt: no-op, SP_OK
    with pytest.raises(sp.SpError) as e:        # lookahead variant: null lookahead keys
        sp.sp_score_look(d, fake, layers, 1024, None, 0, fake, fake, n, stream=0)
    assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:        # misaligned lookahead keys
        sp.sp_score_look(d, fake, layers, 1024, fake + 4, 0, fake, fake, n, stream=0)
    assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:        # look_self outside {0, 1}
        sp.sp_score_look(d, fake, layers, 1024, fake, 2, fake, fake, n, stream=0)
    assert e.value.status == 1
    sp.sp_score_look(d, fake, layers, 0, fake, 1, fake, None, 0, stream=0)   # empty prompt: no-op
    stride = 2 * 4096 * 64
    with pytest.raises(sp.SpError) as e:        # paged variant: null block table
        sp.sp_score_paged(d, fake, layers, None, 4096, stride, 1024, fake, fake, n, stream=0)
    assert e.value.status == 1
    for bad_page in (0, 256, 4096 + 8):          # pages hold a positive multiple of 512 tokens
        with pytest.raises(sp.SpError) as e:
            sp.sp_score_paged(d, fake, layers, fake, bad_page, stride, 1024, fake, fake, n, stream=0)
        assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:        # page stride not a multiple of 8 elements
        sp.sp_score_paged(d, fake, layers, fake, 4096, stride + 4, 1024, fake, fake, n, stream=0)
    assert e.value.status == 1
    sp.sp_score_paged(d, fake, layers, fake, 4096, stride, 0, fake, None, 0, stream=0)   # empty prompt: no-op


def test_score_batch_argument_errors():
    d = good_desc()
    fake = 0x1000
    layers = [fake, fake]
    n = sp.sp_score_workspace(d, 4096, 3)
    with pytest.raises(sp.SpError) as e:        # offsets must start at 0
        sp.sp_score_batch(d, fake, layers, [1, 5, 9], fake, fake, fake, n, stream=0)
    assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:        # decreasing offsets
        sp.sp_score_batch(d, fake, layers, [0, 9, 5], fake, fake, fake, n, stream=0)
    assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:        # device copy missing
        sp.sp_score_batch(d, fake, layers, [0, 5, 9], None, fake, fake, n, stream=0)
    assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:        # no prompts
        sp.sp_score_batch(d, fake, layers, [0], fake, fake, fake, n, stream=0)
    assert e.value.status == 1
    sp.sp_score_batch(d, fake, layers, [0, 0, 0], fake, fake, None, 0, stream=0)   # all empty: no-op


def test_select_argument_errors():
    fake = 0x1000
    n = sp.sp_select_workspace(1000, 32)
    assert n >= 32 * 4 and n % 256 == 0
    with pytest.raises(sp.SpError):
        sp.sp_select_workspace(0, 32)
    with pytest.raises(sp.SpError):
        sp.sp_select_workspace(10, 0)

    def call(L=1000, pool=13, chunk=32, k=4, scores=fake, sel=fake, spans=fake, ns=fake, ws=fake, wsb=n):
        sp.sp_select(scores, L, pool, chunk, k, sel, spans, ns, None, ws, wsb, stream=0)

    for kw, status in [(dict(scores=None), 1), (dict(sel=None), 1), (dict(spans=None), 1), (dict(ns=None), 1),
                       (dict(L=0), 1), (dict(chunk=0), 1), (dict(pool=12), 1), (dict(pool=0), 1), (dict(pool=-3), 1),
                       (dict(pool=131), 2), (dict(k=0), 1), (dict(k=33), 1), (dict(ws=None, wsb=0), 3),
                       (dict(wsb=0), 3), (dict(ws=fake + 8), 3)]:
        with pytest.raises(sp.SpError) as e:
            call(**kw)
        assert e.value.status == status, kw


def test_select_static_argument_errors():
    fake = 0x1000

    def call(L=1000, pool=13, chunk=32, k=4, scores=fake, sel=fake, spans=fake, ns=fake):
        sp.sp_select_static(scores, L, pool, chunk, k, sel, spans, ns, None, stream=0)

    for kw, status in [(dict(scores=None), 1), (dict(sel=None), 1), (dict(spans=None), 1), (dict(ns=None), 1),
                       (dict(L=0), 1), (dict(chunk=0), 1), (dict(pool=12), 1), (dict(pool=131), 2), (dict(k=0), 1),
                       (dict(k=33), 1), (dict(L=(1 << 18) + 1, chunk=1), 2)]:
        with pytest.raises(sp.SpError) as e:
            call(**kw)
        assert e.value.status == status, kw


def test_select_batch_argument_errors():
    fake = 0x1000
    n = sp.sp_select_batch_workspace(1000, 3, 32)
    assert n >= 4 * (1000 // 32 + 3 + 1) and n % 256 == 0
    for args in [(-1, 3, 32), (1000, 0, 32), (1000, 4097, 32), (1000, 3, 0)]:
        with pytest.raises(sp.SpError) as e:
            sp.sp_select_batch_workspace(*args)
        assert e.value.status == 1

    def call(off=(0, 400, 400, 1000), kept=(0, 3, 3, 7), pool=13, chunk=32, scores=fake, offd=fake, keptd=fake, sel=fake,
             spans=fake, ns=fake, ws=fake, wsb=n):
        sp.sp_select_batch(scores, list(off), offd, pool, chunk, list(kept), keptd, sel, spans, ns, None, ws, wsb, stream=0)

    for kw, status in [(dict(scores=None), 1), (dict(offd=None), 1), (dict(keptd=None), 1), (dict(sel=None), 1),
                       (dict(spans=None), 1), (dict(ns=None), 1), (dict(pool=12), 1), (dict(pool=131), 2),
                       (dict(chunk=0), 1), (dict(off=(1, 400, 400, 1000)), 1), (dict(off=(0, 400, 300, 1000)), 1),
                       (dict(kept=(1, 3, 3, 7)), 1),
                       (dict(kept=(0, 3, 4, 7)), 1),            # an empty prompt keeps nothing
                       (dict(kept=(0, 0, 0, 7)), 1),            # a prompt with tokens keeps at least one chunk
                       (dict(kept=(0, 14, 14, 18)), 1),         # more than the 13 chunks of 400 tokens
                       (dict(ws=None, wsb=0), 3), (dict(wsb=8), 3), (dict(ws=fake + 8), 3)]:
        with pytest.raises(sp.SpError) as e:
            call(**kw)
        assert e.value.status == status, (kw, e.value)
    with pytest.raises(sp.SpError):
        sp.sp_select_batch(fake, [0, 10], fake, 13, 32, [0, 1, 2], fake, fake, fake, fake, None, fake, n, stream=0)


def test_project_batch_argument_errors():
    fake = 0x1000

    def call(off=(0, 400, 400, 1000), moff=(0, 450, 450, 1100), kept=(0, 3, 3, 7), doff=fake, offd=fake, toff=fake,
             moffd=fake, spans=fake, ns=fake, keptd=fake, tsp=fake, nt=fake, nk=fake):
        sp.sp_project_batch(doff, list(off), offd, toff, list(moff), moffd, spans, ns, list(kept), keptd, tsp, nt, None, nk,
                            stream=0)

    for kw, status in [(dict(doff=None), 1), (dict(offd=None), 1), (dict(toff=None), 1), (dict(moffd=None), 1),
                       (dict(spans=None), 1), (dict(ns=None), 1), (dict(keptd=None), 1), (dict(tsp=None), 1),
                       (dict(nt=None), 1), (dict(nk=None), 1), (dict(off=(1, 400, 400, 1000)), 1),
                       (dict(moff=(0, 450, 440, 1100)), 1), (dict(kept=(0, 3, 2, 7)), 1),
                       (dict(kept=(0, 1025, 1025, 1030)), 2),                   # more spans than one launch holds
                       (dict(moff=(0, 258048, 258048, 258100)), 2)]:            # more target tokens than a wave-wide probe covers
        with pytest.raises(sp.SpError) as e:
            call(**kw)
        assert e.value.status == status, (kw, e.value)


def test_project_argument_errors():
    fake = 0x1000

    def call(doff=fake, L=10, toff=fake, M=12, spans=fake, ns=fake, cap=4, tsp=fake, nt=fake, nk=fake):
        sp.sp_project(doff, L, toff, M, spans, ns, cap, tsp, nt, None, nk, stream=0)

    for kw in [dict(doff=None), dict(toff=None), dict(spans=None), dict(ns=None), dict(tsp=None), dict(nt=None),
               dict(nk=None), dict(L=0), dict(M=0), dict(cap=0), dict(cap=(1 << 24) + 1)]:
        with pytest.raises(sp.SpError) as e:
            call(**kw)
        assert e.value.status == 1, kw


def test_assemble_argument_errors():
    fake = 0x1000
    n = sp.sp_assemble_workspace(100)
    assert n >= 101 * 8 and n % 256 == 0
    with pytest.raises(sp.SpError):
        sp.sp_assemble_workspace(0)

    def call(ids=fake, M=12, tsp=fake, nt=fake, cap=100, delim=fake, nd=2, ocap=50, oi=fake, op=fake, ol=fake, ws=fake,
             wsb=n):
        sp.sp_assemble(ids, M, tsp, nt, cap, delim, nd, ocap, oi, op, None, ol, ws, wsb, stream=0)

    for kw, status in [(dict(ids=None), 1), (dict(tsp=None), 1), (dict(nt=None), 1), (dict(oi=None), 1),
                       (dict(op=None), 1), (dict(ol=None), 1), (dict(M=0), 1), (dict(cap=0), 1), (dict(nd=-1), 1),
                       (dict(nd=2000), 1), (dict(delim=None), 1), (dict(ocap=0), 1), (dict(ocap=1 << 31), 1),
                       (dict(ws=None, wsb=0), 3), (dict(wsb=8), 3), (dict(ws=fake + 8), 3)]:
        with pytest.raises(sp.SpError) as e:
            call(**kw)
        assert e.value.status == status, kw


def test_select_budget_argument_errors():
    fake = 0x1000
    n = sp.sp_select_budget_workspace(4096, 32)
    assert n % 256 == 0 and n >= 128 * 4 * 3
    with pytest.raises(sp.SpError) as e:                   # more chunks than the rank kernel is sized for
        sp.sp_select_budget_workspace(1 << 22, 32)
    assert e.value.status == 2

    def call(sc=fake, L=4096, w=13, c=32, do=fake, to=fake, M=5000, budget=1024, sel=fake, spans=fake, ns=fake,
             k=fake, ws=fake, wsb=n):
        sp.sp_select_budget(sc, L, w, c, do, to, M, budget, sel, spans, ns, k, None, None, ws, wsb, stream=0)

    for kw, status in [(dict(sc=None), 1), (dict(do=None), 1), (dict(to=None), 1), (dict(sel=None), 1),
                       (dict(spans=None), 1), (dict(ns=None), 1), (dict(k=None), 1), (dict(L=0), 1), (dict(M=0), 1),
                       (dict(c=0), 1), (dict(w=4), 1), (dict(w=131), 2), (dict(budget=-1), 1), (dict(M=1 << 31), 2),
                       (dict(L=1 << 22), 2), (dict(ws=None, wsb=0), 3), (dict(wsb=256), 3), (dict(ws=fake + 8), 3)]:
        with pytest.raises(sp.SpError) as e:
            call(**kw)
        assert e.value.status == status, kw


def test_binding_rejects_host_tensors_before_the_call():
    """Tensors are checked in the binding: a host tensor never reaches the library as a device address."""
    import torch
    host = torch.zeros(1000, dtype=torch.float32)
    sel = torch.zeros(4, dtype=torch.int32)
    with pytest.raises(sp.SpError) as e:
        sp.sp_select(host, 1000, 13, 32, 4, sel, sel, sel, None, 0x1000, 256, stream=0)
    assert e.value.status == 1 and "scores is not a device tensor" in e.value.message
    d = good_desc()
    with pytest.raises(sp.SpError) as e:
        sp.sp_score(d, host, [0x1000, 0x1000], 1024, 0x1000, 0x1000, 1 << 20, stream=0)
    assert e.value.status == 1 and "q is not a device tensor" in e.value.message
    with pytest.raises(sp.SpError) as e:
        sp.sp_score(d, 0x1000, [0x1000, host], 1024, 0x1000, 0x1000, 1 << 20, stream=0)
    assert "k_layers[1]" in e.value.message


def test_read_probe_argument_errors():
    fake = 0x1000
    for kw in [dict(buf=None), dict(sink=None), dict(n=0), dict(n=24), dict(buf=fake + 8)]:
        args = dict(buf=fake, n=1024, sink=fake)
        args.update(kw)
        with pytest.raises(sp.SpError) as e:
            sp.sp_hbm_read_probe(args["buf"], args["n"], args["sink"], stream=0)
        assert e.value.status == 1, kw


def test_score_fp8_argument_errors():
    d = good_desc()
    fake = 0x1000
    n = sp.sp_score_workspace(d, 1024, 1)
    with pytest.raises(sp.SpError) as e:
        sp.sp_score_fp8(d, fake, [fake, fake], None, 1024, fake, fake, n, stream=0)
    assert e.value.status == 1 and "kscale" in e.value.message
    with pytest.raises(sp.SpError) as e:
        sp.sp_score_fp8(d, fake, [fake, None], fake, 1024, fake, fake, n, stream=0)
    assert e.value.status == 1
    with pytest.raises(sp.SpError) as e:
        sp.sp_score_fp8(d, fake, [fake, fake], fake, 1024, fake, fake, 256, stream=0)
    assert e.value.status == 3
