"""The plain streaming kernels that serve as bandwidth yardsticks must compute what their header says, on sizes
that are not multiples of their tiles (a yardstick that skipped or repeated elements would move the ceiling)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [4, 1028, 8 * 4 * 256 * 4, 8 * 4 * 256 * 4 + 12, 5_000_004])
def test_probes(n):
    import paper_1708_02983_amd as hip
    g = torch.Generator(device="cuda"); g.manual_seed(n)
    b, c, d = (torch.randn(n + 8, device="cuda", generator=g) for _ in range(3))
    a = torch.full((n + 8,), float("nan"), device="cuda")
    a2 = torch.full((n + 8,), float("nan"), device="cuda")
    hip.stream_copy(a[:n], b[:n])
    assert torch.equal(a[:n], b[:n]) and bool(torch.isnan(a[n:]).all())
    a.fill_(float("nan"))
    hip.stream_triad(a[:n], b[:n], c[:n], 0.5)
    assert torch.equal(a[:n], torch.addcmul(b[:n], c[:n], torch.tensor(0.5, device="cuda"))) or \
        torch.allclose(a[:n], b[:n] + 0.5 * c[:n], rtol=0, atol=1e-6)
    assert bool(torch.isnan(a[n:]).all())
    a.fill_(float("nan"))
    hip.stream_mix32(a[:n], a2[:n], b[:n], c[:n], d[:n], 0.5)
    assert torch.allclose(a[:n], b[:n] + 0.5 * c[:n], rtol=0, atol=1e-6)
    assert torch.allclose(a2[:n], c[:n] + 0.5 * d[:n], rtol=0, atol=1e-6)
    assert bool(torch.isnan(a[n:]).all()) and bool(torch.isnan(a2[n:]).all())
