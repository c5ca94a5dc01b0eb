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


def _issue_expected(kind, iters, a, b):
    """The chain values of the issue probe by a plain loop (operands chosen so that every step is exact)."""
    f = np.float32
    out = np.zeros(8, dtype=np.float64)
    lanes = []
    for t in range(8):
        xs = [f(t * 0.125 + j) for j in range(8)]
        for _ in range(iters * 4):                      # four statements of two instructions per chain and iteration
            for j in range(8):
                x = xs[j]
                if kind == 0: x = f(x + f(a) * f(b)); x = f(x + f(a) * f(b))
                elif kind == 1: x = max(x, f(a)); x = max(x, f(b))
                elif kind == 2: x = f(x * f(a) + f(b)); x = f(x * f(a) + f(b))
                elif kind == 3: x = f(b) if x < f(a) else x
                elif kind == 4: x = f(x * f(a)); x = f(x * f(a))
                else: x = f(x * f(a) + f(b)); x = max(x, f(b))
                xs[j] = x
        lanes.append(f(f(f(xs[0] + xs[1]) + f(xs[2] + xs[3])) + f(f(xs[4] + xs[5]) + f(xs[6] + xs[7]))))
    return np.array(lanes, dtype=np.float32)


@pytest.mark.parametrize("kind,a,b", [(0, 0.5, 0.25), (1, 3.5, 5.25), (2, 1.0, 0.125), (3, 4.0, 9.0), (4, 0.5, 0.0), (6, 1.0, 0.125)])
def test_issue_probe_values(kind, a, b):
    # dyadic operands: every fma, product and sum below is exact in binary32, so the plain loop is the definition
    import torch
    iters = 5
    out = ctx().issue_probe(kind, 2, iters, a, b)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(-1, 256)
    want = np.tile(_issue_expected(kind, iters, a, b), 32)
    assert got.shape[0] == 2 * torch.cuda.get_device_properties(0).multi_processor_count
    assert np.array_equal(got, np.broadcast_to(want, got.shape))


def test_issue_probe_argument_errors():
    for bad in ((19, 1, 1), (-1, 1, 1), (0, 0, 1), (0, 9, 1), (0, 1, 0)):
        with pytest.raises(sop.SopError) as e:
            ctx().issue_probe(*bad)
        assert e.value.status == 1


@pytest.mark.parametrize("kind", [15, 16, 17, 18])
def test_element_pass_probe_runs_and_repeats(kind):
    # the element-pass kinds hold a pattern, not a codebook: their sums are finite and the same on every run
    import torch
    a = ctx().issue_probe(kind, 3, 3, 0.3, 1.25).clone()
    b = ctx().issue_probe(kind, 3, 3, 0.3, 1.25)
    torch.cuda.synchronize()
    assert torch.isfinite(a).all() and torch.equal(a, b)
