"""The measurement helpers of the library do what their declarations say: the copy copies, the
triad is one fused multiply-add per element, the matrix-core probe runs to completion and writes
one finite value per thread; bad arguments come back as errors, not launches."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    from paper_2311_04499_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


@pytest.mark.parametrize("n", [4, 64 * 4 + 4, 1_000_000])
def test_copy_and_triad(B, n):
    g = torch.Generator(device=DEV)
    g.manual_seed(n)
    b = torch.randn(n, generator=g, device=DEV)
    c = torch.randn(n, generator=g, device=DEV)
    a = torch.full((n + 4,), float("nan"), device=DEV)
    B.covap_probe_copy(a, b, 4 * n)
    torch.cuda.synchronize()
    assert torch.equal(a[:n], b) and bool(torch.isnan(a[n:]).all())          # nothing past the end
    B.covap_probe_triad(a, b, c, 0.5, n)
    torch.cuda.synchronize()
    want = np.float32(0.5) * c.cpu().numpy().astype(np.float64) + b.cpu().numpy().astype(np.float64)
    assert np.array_equal(a[:n].cpu().numpy(), want.astype(np.float32))      # one rounding: 0.5 * c is exact
    assert bool(torch.isnan(a[n:]).all())
    with pytest.raises(B.CovapError):
        B.covap_probe_copy(a, b, 4 * n - 2)                                   # not a multiple of 16 bytes
    with pytest.raises(B.CovapError):
        B.covap_probe_triad(a, b, c, 0.5, n - 1)


def test_matrix_core_probe(B):
    out = torch.full((8 * 256 + 16,), float("nan"), device=DEV)
    for iters, lds in ((0, 0), (10, 0), (100, 65536)):
        out.fill_(float("nan"))
        B.covap_probe_mfma(out, 8, iters, lds)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out[:8 * 256]).all()) and bool(torch.isnan(out[8 * 256:]).all())
        if iters == 0:
            assert not bool(out[:8 * 256].any())
    with pytest.raises(ValueError):
        B.covap_probe_mfma(out[:100], 8, 1)                                   # the binding checks the buffer
    with pytest.raises(B.CovapError):
        B.covap_probe_mfma(out, 0, 1)
    with pytest.raises(B.CovapError):
        B.covap_probe_mfma(out, 8, -1)
    with pytest.raises(B.CovapError):
        B.covap_probe_mfma(out, 8, 1, 1 << 20)
    torch.cuda.synchronize()
