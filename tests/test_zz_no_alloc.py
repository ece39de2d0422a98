"""sp_select_static (the selection entry point that takes no workspace and allocates nothing)
against sp_select, through the C ABI: two calls in a row, the second on a smaller input, so that
what the first call left in the library's own scratch array cannot leak into the second result."""
import numpy as np
import pytest
import torch

import paper_2603_02631_amd as sp

from gpu_util import DEV, workspace

pytestmark = pytest.mark.gpu


def _run(entry, scores: np.ndarray, pool_w: int, chunk: int, k: int):
    L = scores.size
    C = (L + chunk - 1) // chunk
    sd = torch.from_numpy(np.ascontiguousarray(scores, dtype=np.float32)).to(DEV)
    sel = torch.full((k,), -1, dtype=torch.int32, device=DEV)
    spans = torch.full((k, 2), -1, dtype=torch.int64, device=DEV)
    n_spans = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    cs = torch.full((C,), float("nan"), dtype=torch.float32, device=DEV)
    if entry == "static":
        sp.sp_select_static(sd, L, pool_w, chunk, k, sel, spans, n_spans, cs)
    else:
        ws = workspace(sp.sp_select_workspace(L, chunk))
        sp.sp_select(sd, L, pool_w, chunk, k, sel, spans, n_spans, cs, ws)
    torch.cuda.synchronize()
    return sel.cpu().numpy(), spans.cpu().numpy(), int(n_spans.item()), cs.cpu().numpy()


def _scores(seed: int, L: int) -> np.ndarray:
    rng = np.random.default_rng([260302631, 77, seed])
    s = rng.random(L).astype(np.float32) * 1e-4
    hot = rng.choice(L, size=max(1, L // 50), replace=False)
    s[hot] += rng.random(hot.size).astype(np.float32)
    return s


def test_static_scratch_entry_point_matches_sp_select_twice():
    # first call: 131072 tokens in chunks of 32 (4096 chunks, several key tiles of the top-k kernel);
    # second call: a smaller, ragged input (L not a multiple of the chunk) that overwrites only the
    # head of the scratch array
    for seed, L, pool_w, chunk, keep in ((1, 131072, 13, 32, 0.1), (2, 5003, 13, 64, 0.25)):
        s = _scores(seed, L)
        C = (L + chunk - 1) // chunk
        k = sp.sp_keep_count(C, int(keep * 100), 100)
        want = _run("workspace", s, pool_w, chunk, k)
        got = _run("static", s, pool_w, chunk, k)
        np.testing.assert_array_equal(got[3].view(np.uint32), want[3].view(np.uint32))     # chunk scores, bit for bit
        np.testing.assert_array_equal(got[0], want[0])
        assert got[2] == want[2]
        np.testing.assert_array_equal(got[1], want[1])
        assert (got[0] >= 0).all() and got[2] >= 1


def test_static_scratch_entry_point_rejects_sizes_beyond_its_array():
    L = (1 << 18) + 1          # chunk 1: one chunk more than the array holds
    sd = torch.zeros(L, dtype=torch.float32, device=DEV)
    sel = torch.zeros(1, dtype=torch.int32, device=DEV)
    spans = torch.zeros((1, 2), dtype=torch.int64, device=DEV)
    n_spans = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(sp.SpError) as e:
        sp.sp_select_static(sd, L, 1, 1, 1, sel, spans, n_spans, None)
    assert e.value.status == 2 and "scratch" in e.value.message
