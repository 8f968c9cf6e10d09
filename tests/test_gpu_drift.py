"""GPU parity of the inter-layer representation drift (Eq. 1) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import tsa_oracle as orc
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tsa():
    from paper_2602_03216_amd import binding
    binding.load_library(build_if_missing=False)
    return binding


@pytest.mark.parametrize("n_tokens,width,eps", [(1, 8, 0.0), (7, 136, 1e-6), (1000, 4096, 1e-6), (16385, 3584, 1e-3), (65, 8192, 0.5)])
def test_layer_drift(tsa, n_tokens, width, eps):
    r = np.random.Generator(np.random.PCG64(800 + n_tokens))
    hin = gu.rand_bits(r, (n_tokens, width))
    hout = orc.f64_to_bf16(orc.bf16_to_f64(hin) + 0.3 * r.standard_normal((n_tokens, width)))
    out = torch.full((1,), -1.0, dtype=torch.float32, device=gu.DEV)
    a, b = gu.to_dev(hin), gu.to_dev(hout)
    tsa.tsa_layer_drift(a, b, eps, out)
    first = out.item()
    tsa.tsa_layer_drift(a, b, eps, out)
    torch.cuda.synchronize()
    want = orc.layer_drift(orc.bf16_to_f64(hin), orc.bf16_to_f64(hout), eps)
    assert out.item() == first                      # deterministic
    assert abs(out.item() - want) <= 2e-6 * abs(want) + 1e-9
    # unchanged hidden state: drift exactly zero
    tsa.tsa_layer_drift(a, a, eps, out)
    assert out.item() == 0.0
