"""The read-probe calibration kernel: its per-workgroup checksums combine to the exclusive-or of the
buffer's 32-bit words (numpy), for sizes from one 16-byte word to a layer."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from gpu_util import ctx

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_words", [4, 4 * 255, 4 * 256 * 2048, 4 * (256 * 2048 * 3 + 77), 4096 * 11008 // 2])
def test_checksum(n_words):
    import torch
    rng = np.random.default_rng(n_words)
    x = rng.integers(0, 1 << 32, size=n_words, dtype=np.uint64).astype(np.uint32)
    xt = torch.from_numpy(x.view(np.int32)).cuda()
    out = ctx().read_probe(xt)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(out.cpu().numpy().view(np.uint32))
    assert got == np.bitwise_xor.reduce(x)


def test_argument_errors():
    import torch
    x = torch.zeros(6, dtype=torch.int32, device="cuda")              # 24 bytes: not a multiple of 16
    with pytest.raises(sop.SopError) as e:
        ctx().read_probe(x)
    assert e.value.status == 1
    y = torch.zeros(12, dtype=torch.int32, device="cuda")[1:9]        # 32 bytes at a 4-byte offset
    with pytest.raises(sop.SopError):
        ctx().read_probe(y)
