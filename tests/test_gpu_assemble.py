"""GPU parity of sp_assemble (compressed-prompt token and position ids) against the oracle:
integer work, compared bit for bit. All calls go through the C ABI."""
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


def gpu_assemble(ids, tspans, delim, max_spans=None, out_capacity=None, want_src=True, n_override=None):
    import torch
    import paper_2603_02631_amd as sp
    from gpu_util import DEV, workspace
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    tspans = np.ascontiguousarray(tspans, dtype=np.int64).reshape(-1, 2)
    delim = np.ascontiguousarray(delim, dtype=np.int32)
    n = tspans.shape[0]
    cap = max_spans if max_spans is not None else max(n, 1)
    ocap = out_capacity if out_capacity is not None else ids.size + cap * max(delim.size, 1) + 1
    idd = torch.from_numpy(ids).to(DEV)
    tsp = torch.full((cap, 2), -7, dtype=torch.int64, device=DEV)
    if n:
        tsp[:n] = torch.from_numpy(tspans).to(DEV)
    nt = torch.tensor([n if n_override is None else n_override], dtype=torch.int32, device=DEV)
    dl = torch.from_numpy(delim).to(DEV) if delim.size else None
    out_ids = torch.full((ocap,), -1, dtype=torch.int32, device=DEV)
    out_pos = torch.full((ocap,), -1, dtype=torch.int32, device=DEV)
    out_src = torch.full((ocap,), -9, dtype=torch.int64, device=DEV) if want_src else None
    out_len = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    ws = workspace(sp.sp_assemble_workspace(cap))
    sp.sp_assemble(idd, ids.size, tsp, nt, cap, dl, delim.size, ocap, out_ids, out_pos, out_src, out_len, ws)
    torch.cuda.synchronize()
    return (out_ids.cpu().numpy(), out_pos.cpu().numpy(), out_src.cpu().numpy() if want_src else None,
            int(out_len.item()))


def check(ids, tspans, delim, **kw):
    want_ids, want_pos, want_src = oracle.assemble(ids, tspans, delim)
    got_ids, got_pos, got_src, n = gpu_assemble(ids, tspans, delim, **kw)
    assert n == want_ids.size
    np.testing.assert_array_equal(got_ids[:n], want_ids)
    np.testing.assert_array_equal(got_pos[:n], want_pos)
    if got_src is not None:
        np.testing.assert_array_equal(got_src[:n], want_src)
        assert (got_src[n:] == -9).all()
    assert (got_ids[n:] == -1).all() and (got_pos[n:] == -1).all()        # nothing written past the end
    return n


def test_assemble_small_cases_and_edges():
    say("[assemble] small cases")
    ids = np.arange(1000, 1400, dtype=np.int32)
    check(ids, [[2, 5], [9, 11], [399, 400]], [7, 8])
    check(ids, [[0, 400]], [7, 8])                      # keep-all: no delimiter
    check(ids, np.zeros((0, 2)), [7])                   # nothing kept: length 0
    check(ids, [[0, 2], [4, 6]], [])                    # empty delimiter
    check(ids, [[5, 5], [7, 9]], [1, 2, 3])             # an empty range still separates
    check(ids, [[3, 4]], [9], want_src=False)           # optional output absent
    check(ids, [[i, i + 1] for i in range(0, 400, 2)], [5], max_spans=300)     # 200 one-token ranges
    # more ranges on the device than max_spans: the count is clamped
    want = oracle.assemble(ids, [[0, 2], [4, 6]], [7])[0]
    got_ids, _, _, n = gpu_assemble(ids, [[0, 2], [4, 6], [8, 9]], [7], max_spans=3, n_override=2)
    assert n == want.size and got_ids[:n].tolist() == want.tolist()


def test_assemble_many_ranges_span_several_scan_segments():
    say("[assemble] 1000 ranges")
    rng = np.random.default_rng(3)
    M = 60000
    ids = rng.integers(0, 150000, size=M).astype(np.int32)
    cuts = np.sort(rng.choice(np.arange(1, M), size=1999, replace=False))
    bounds = np.concatenate([[0], cuts, [M]])
    tspans = np.stack([bounds[0:-1:2], bounds[1::2]], axis=1)       # every other piece: 1000 ranges
    assert tspans.shape[0] == 1000
    check(ids, tspans, rng.integers(150000, 150010, size=3))


def test_assemble_truncates_at_capacity_and_reports_full_length():
    say("[assemble] capacity")
    ids = np.arange(50, dtype=np.int32)
    want = oracle.assemble(ids, [[0, 10], [20, 30]], [99, 98])[0]
    got_ids, got_pos, _, n = gpu_assemble(ids, [[0, 10], [20, 30]], [99, 98], out_capacity=15)
    assert n == 22 and got_ids.tolist() == want[:15].tolist() and got_pos.tolist() == list(range(15))


@pytest.mark.parametrize("name", ["tiny", "llama1b-8k"])
def test_assemble_after_projection_on_workloads(name):
    """Chained on the device after sp_select and sp_project, the way a caller would run it."""
    import torch
    import paper_2603_02631_amd as sp
    from gpu_util import DEV, workspace
    w = synth.get_config(name)
    say(f"[assemble] {name}: chained after select + project")
    rng = np.random.default_rng(w.cfg_id)
    L = w.L
    I = rng.random(L)
    doff, toff = synth.gen_char_offsets(w, L)
    M = toff.size - 1
    C = (L + w.chunk - 1) // w.chunk
    k = sp.sp_keep_count(C, w.keep_num, w.keep_den)
    sel, spans, _ = oracle.select(I, w.pool, w.chunk, k)
    ts, mask, n_kept = oracle.project(doff, toff, spans)
    ids = rng.integers(0, 128000, size=M).astype(np.int32)
    delim = np.array([58, 1131, 60], dtype=np.int32)
    want_ids, want_pos, want_src = oracle.assemble(ids, ts, delim)

    sd = torch.from_numpy(I.astype(np.float32)).to(DEV)
    seld = torch.empty(k, dtype=torch.int32, device=DEV)
    spd = torch.empty((k, 2), dtype=torch.int64, device=DEV)
    nsd = torch.zeros(1, dtype=torch.int32, device=DEV)
    sp.sp_select(sd, L, w.pool, w.chunk, k, seld, spd, nsd, None, workspace(sp.sp_select_workspace(L, w.chunk)))
    tsd = torch.empty((k, 2), dtype=torch.int64, device=DEV)
    ntd = torch.zeros(1, dtype=torch.int32, device=DEV)
    nkd = torch.zeros(1, dtype=torch.int64, device=DEV)
    sp.sp_project(torch.from_numpy(doff).to(DEV), L, torch.from_numpy(toff).to(DEV), M, spd, nsd, k, tsd, ntd, None, nkd)
    ocap = M + k * delim.size
    oi = torch.full((ocap,), -1, dtype=torch.int32, device=DEV)
    op = torch.full((ocap,), -1, dtype=torch.int32, device=DEV)
    os_ = torch.full((ocap,), -9, dtype=torch.int64, device=DEV)
    ol = torch.zeros(1, dtype=torch.int64, device=DEV)
    sp.sp_assemble(torch.from_numpy(ids).to(DEV), M, tsd, ntd, k, torch.from_numpy(delim).to(DEV), delim.size, ocap,
                   oi, op, os_, ol, workspace(sp.sp_assemble_workspace(k)))
    torch.cuda.synchronize()
    n = int(ol.item())
    # the float32 scores on the device may order near-ties differently from the float64 oracle only
    # if two chunk means coincide to ~1e-7: with random scores they do not, so the chain is exact
    assert n == want_ids.size == n_kept + (ts.shape[0] - 1) * delim.size
    np.testing.assert_array_equal(oi.cpu().numpy()[:n], want_ids)
    np.testing.assert_array_equal(op.cpu().numpy()[:n], want_pos)
    np.testing.assert_array_equal(os_.cpu().numpy()[:n], want_src)
    say(f"[assemble] {name}: ok, {n} ids ({ts.shape[0]} ranges) from {M} target tokens")
