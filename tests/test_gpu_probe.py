"""The streaming-read probe reads every byte it is given: its XOR checksum against numpy, on sizes
that end inside a block's span and with a non-zero starting value in the sink. A short buffer is
refused by the binding before the call."""
import numpy as np
import pytest
import torch

import paper_2603_02631_amd as sp

from gpu_util import DEV

pytestmark = pytest.mark.gpu


def _fold(a: np.ndarray) -> int:
    w = a.view(np.uint32).reshape(-1, 4)
    x = np.bitwise_xor.reduce(w, axis=0)
    return (int(x[0] ^ x[2]) << 32) | int(x[1] ^ x[3])


@pytest.mark.parametrize("nbytes", [16, 4096, 16 * (256 * 8 + 3), 16 * 1234567])
def test_probe_checksum_matches_numpy(nbytes):
    rng = np.random.default_rng([260302631, 88, nbytes])
    a = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
    buf = torch.from_numpy(a).to(DEV)
    start = 0x0123456789ABCDEF
    sink = torch.tensor([start], dtype=torch.int64, device=DEV)
    sp.sp_hbm_read_probe(buf, nbytes, sink)
    torch.cuda.synchronize()
    got = int(sink.cpu().numpy().view(np.uint64)[0])
    assert got == start ^ _fold(a)
    with pytest.raises(sp.SpError):
        sp.sp_hbm_read_probe(buf, nbytes + 16, sink)
