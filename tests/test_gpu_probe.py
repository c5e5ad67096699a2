"""The MFMA-rate measurement hook runs and returns a rate a gfx950 can have."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("waves", [1, 2])
def test_mfma_rate_probe_returns_a_plausible_rate(waves):
    from paper_2503_22796_amd import binding as B
    g = torch.Generator(device="cpu").manual_seed(3)
    data = torch.randn(1 << 16, generator=g).to(torch.bfloat16).to("cuda:0")
    tflops, ms = B.difa_probe_mfma_rate(data, waves_per_simd=waves, rounds=4000)
    assert ms > 0
    # 256 compute units x 4 SIMDs, one 32x32x16 MFMA per 32 clocks at no more than 2.4 GHz
    assert 200.0 < tflops < 2600.0, tflops
