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


@pytest.mark.parametrize("lds_fetch", [0, 1, 2], ids=["registers", "lds", "lds+global_feed"])
def test_mfma_probe_does_the_flops_it_claims(lds_fetch):
    """Every pass of the matrix-core yardstick adds the 64x64 product A^T B of its slab to the accumulators (values
    are multiples of 1/32, so a few passes are exact): out must hold iters x that product in every block, in the
    accumulator layout of the 32x32x2 instruction, and the call must report blocks x 4 x iters x 16 x 4096 flops."""
    import paper_1708_02983_amd as hip
    iters, per_cu = 3, 1
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out = torch.full((per_cu * cus * 4096 + 5,), float("nan"), device="cuda")
    src = torch.randn(5 * 4096 + 100, device="cuda") if lds_fetch == 2 else None     # five pieces and a remainder
    flops = hip.mfma_probe(out, iters, lds_fetch, per_cu, src=src)
    assert flops == per_cu * cus * 4 * iters * 16 * 4096
    val = lambda i: ((i * 37 + 11) % 64 - 32) / 32.0
    A = np.array([[val(k * 64 + m) for m in range(64)] for k in range(32)])
    B = np.array([[val(1000 + k * 64 + n) for n in range(64)] for k in range(32)])
    C = iters * (A.T @ B)
    expect = np.empty((256, 16))
    for t in range(256):
        wave, lane = t // 64, t % 64
        for r in range(16):
            expect[t, r] = C[(wave >> 1) * 32 + 8 * (r // 4) + 4 * (lane // 32) + r % 4, (wave & 1) * 32 + lane % 32]
    got = out.cpu().numpy()
    assert np.isnan(got[per_cu * cus * 4096:]).all()
    got = got[:per_cu * cus * 4096].reshape(-1, 16, 256)            # [block][register][thread]
    for b in (0, 1, got.shape[0] // 2, got.shape[0] - 1):
        np.testing.assert_array_equal(got[b].T.astype(np.float64), expect)
    with pytest.raises(hip.EasgdError):
        hip.mfma_probe(out[:100], iters, lds_fetch, per_cu, src=src)
    with pytest.raises(hip.EasgdError):
        hip.mfma_probe(out, iters, 2, per_cu)                       # mode 2 without a source
