"""Helpers shared by the GPU parity tests: host <-> device marshalling of bf16 bit patterns
and the tolerances of the parity bar."""
import numpy as np
import torch

from oracle import tsa_oracle as orc

DEV = "cuda:0"
# parity bar for bf16 outputs (max-abs / mean-abs against the oracle's bf16-rounded result)
MAX_ABS, MEAN_ABS = 2e-2, 2e-3
# fp32 scores: bf16 products are exact, the difference is fp32 accumulation order and exp2
SCORE_RTOL, SCORE_ATOL = 3e-5, 1e-10


def to_dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 tensor on the GPU."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def from_dev(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns on the host."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def rand_bits(rng, shape, scale=1.0):
    return orc.f64_to_bf16(rng.standard_normal(shape) * scale)


def assert_output_close(got_bits, want_bits, what=""):
    err = np.abs(orc.bf16_to_f64(got_bits) - orc.bf16_to_f64(want_bits))
    assert np.isfinite(err).all(), what
    assert err.max() <= MAX_ABS, "%s max-abs %.4g" % (what, err.max())
    assert err.mean() <= MEAN_ABS, "%s mean-abs %.4g" % (what, err.mean())
    return err.max(), err.mean()


def assert_scores_close(got, want, what=""):
    got = np.asarray(got, dtype=np.float64)
    bad = np.abs(got - want) > SCORE_RTOL * np.abs(want) + SCORE_ATOL
    assert not bad.any(), "%s: %d scores off, worst rel %.3g" % (
        what, bad.sum(), np.max(np.abs(got - want) / np.maximum(np.abs(want), 1e-30)))
