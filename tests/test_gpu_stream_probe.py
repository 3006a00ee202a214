"""The bare streaming kernels behind bench.py's `ceilings` do what lioncub.h says (plumbing,
not a step of the method: the reference here is the same arithmetic in torch on the host)."""
import numpy as np
import pytest
import torch

import paper_2411_16462_amd as lc

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [1, 3, 255, 256, 1027, 300001])
def test_stream_probe_kernels(n):
    gen = torch.Generator().manual_seed(n)
    a0 = torch.randn(n + 8, generator=gen)
    b0 = torch.randn(n + 8, generator=gen)
    s = 0.99

    def run(kind, with_b=True):
        a, b = a0.cuda(), b0.cuda()
        lc.lc_stream_probe(kind, a, b if with_b else None, n, s)
        torch.cuda.synchronize()
        assert torch.equal(b.cpu(), b0) and torch.equal(a.cpu()[n:], a0[n:])     # b is only read, nothing beyond n is written
        return a.cpu()[:n]

    assert torch.equal(run(lc.LC_PROBE_READ), a0[:n]) and torch.equal(run(lc.LC_PROBE_READ, False), a0[:n])
    assert torch.equal(run(lc.LC_PROBE_WRITE, False), torch.full((n,), s, dtype=torch.float32))
    assert torch.equal(run(lc.LC_PROBE_COPY), b0[:n])
    assert torch.equal(run(lc.LC_PROBE_SCALE, False), a0[:n] * np.float32(s))
    t = np.float32(1.0) - np.float32(s)
    want = a0[:n].double() * float(np.float32(s)) + (b0[:n] * t).double()
    assert torch.allclose(run(lc.LC_PROBE_RMW2).double(), want, rtol=1e-6, atol=1e-7)
