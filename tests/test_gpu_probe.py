"""lsgd_stream_probe (the benchmark's measurement aid) moves exactly the bytes it says it moves."""
import pytest
import torch

import paper_1905_10395_amd as L

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("n", [2, 510, 512, 100_002, 3_000_000])
def test_stream_probe_kinds(n):
    gen = torch.Generator(device=DEV).manual_seed(n)
    a = torch.randn(n, device=DEV, generator=gen)
    b = torch.randn(n, device=DEV, generator=gen)
    c = torch.randn(n, device=DEV, generator=gen)
    a0, b0, c0 = a.clone(), b.clone(), c.clone()
    L.stream_probe(L.PROBE_READ, a, b)
    torch.cuda.synchronize()
    assert torch.equal(a, a0) and torch.equal(b, b0)
    L.stream_probe(L.PROBE_COPY, a, c)
    torch.cuda.synchronize()
    assert torch.equal(c, a0) and torch.equal(a, a0)
    c.copy_(c0)
    L.stream_probe(L.PROBE_UPDATE, a, b, c)
    torch.cuda.synchronize()
    m = 0.9 * c0.double() + b0.double()
    torch.testing.assert_close(c.double(), m, rtol=1e-6, atol=1e-7)
    torch.testing.assert_close(a.double(), a0.double() - 1e-3 * m, rtol=1e-6, atol=1e-7)
    assert torch.equal(b, b0)


def test_stream_probe_rejects_bad_arguments():
    a = torch.zeros(7, device=DEV)
    with pytest.raises(L.LsgdError, match="even"):
        L.stream_probe(L.PROBE_COPY, a, a.clone())
    a = torch.zeros(8, device=DEV)
    with pytest.raises(L.LsgdError, match="kind"):
        L.stream_probe(9, a, a.clone())
    with pytest.raises(L.LsgdError, match="NULL"):
        L.stream_probe(L.PROBE_UPDATE, a, a.clone())
