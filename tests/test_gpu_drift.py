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


def test_mfma_probe_runs_and_reports_clocks(tsa):
    """The roofline calibration loop: queues, finishes, and reports a plausible shader clock."""
    ops = torch.zeros(1 << 15, dtype=torch.bfloat16, device=gu.DEV)
    blocks = 64
    sink = torch.empty(blocks * 256, dtype=torch.float32, device=gu.DEV)
    clocks = torch.zeros(2, dtype=torch.int64, device=gu.DEV)
    flops, khz = tsa.tsa_mfma_probe(ops, 1000, blocks, sink, clocks)
    torch.cuda.synchronize()
    assert flops == blocks * 4 * 1000 * 8 * 2 * 32 * 32 * 16 and khz > 0
    cyc, ticks = (int(v) for v in clocks.cpu())
    mhz = cyc / (ticks / (khz * 1e3)) / 1e6
    assert cyc >= 1000 * 8 * 16 and 500 < mhz < 3500
    assert not sink.isnan().any() and float(sink.abs().max()) == 0.0      # zero operands: zero accumulators


def test_mix_and_read_probes_run(tsa):
    """The instruction-mix and read-bandwidth calibration loops: they queue, finish and leave finite results."""
    ops = (torch.randn(1 << 15, device=gu.DEV) * 0.5).to(torch.bfloat16)
    blocks = 64
    sink = torch.empty(blocks * 256, dtype=torch.float32, device=gu.DEV)
    for mix, per_iter in ((0, 16), (1, 16), (2, 8), (3, 8)):
        sink.fill_(float("nan"))
        flops = tsa.tsa_mix_probe(mix, ops, 50, blocks, sink)
        torch.cuda.synchronize()
        assert flops == blocks * 4 * 50 * per_iter * 2 * 32 * 32 * 16
        assert not sink.isnan().any()                      # every thread wrote its accumulator sum
    src = torch.arange(1 << 20, dtype=torch.int32, device=gu.DEV)
    word = torch.zeros(1, dtype=torch.int32, device=gu.DEV)
    tsa.tsa_read_probe(src, word)
    torch.cuda.synchronize()
