"""tsa_select_static (the selection with its scratch in a static device array of the library, for
callers that cannot allocate) against tsa_select, through the C ABI: index sets and inverse maps bit
for bit, on two calls in a row that share the array, the second with a smaller input."""
import ctypes

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


def _both(tsa, s_np, k, **kw):
    B, Hq, L = s_np.shape
    Hkv = kw.pop("Hkv", Hq)
    desc = tsa.make_desc(B, Hq, Hkv, L, 128, min(64, L), **kw)
    Hs = Hkv if desc.group_mode else Hq
    s = torch.from_numpy(s_np).to(gu.DEV)
    out = []
    for static in (False, True):
        idx = torch.full((B, Hs, k), -7, dtype=torch.int32, device=gu.DEV)
        inv = torch.full((B, Hs, L), -7, dtype=torch.int32, device=gu.DEV)
        if static:
            tsa.tsa_select_static(desc, s, k, idx, inv)
        else:
            tsa.tsa_select(desc, s, k, idx, inv, tsa.alloc_workspace(desc, k, gu.DEV))
        torch.cuda.synchronize()
        out.append((idx.cpu().numpy(), inv.cpu().numpy()))
    assert np.array_equal(out[0][0], out[1][0]) and np.array_equal(out[0][1], out[1][1])
    return out[1]


def test_static_scratch_selection_equals_the_workspace_form_on_two_calls_in_a_row(tsa):
    r = np.random.Generator(np.random.PCG64(77))
    # first call: long rows (the sliced kernels), many ties; second call, smaller: short rows (one launch per row)
    s1 = (r.integers(0, 50, size=(2, 6, 40001)) / 64.0).astype(np.float32)
    idx, inv = _both(tsa, s1, 9000)
    widx, winv = orc.select(s1.astype(np.float64), 9000)
    assert np.array_equal(idx, widx) and np.array_equal(inv, winv)
    s2 = r.random((1, 3, 1500)).astype(np.float32)
    idx, inv = _both(tsa, s2, 400, force_first=2, force_last=3)
    widx, winv = orc.select(s2.astype(np.float64), 400, 2, 3)
    assert np.array_equal(idx, widx) and np.array_equal(inv, winv)
    # group mode (the group sums live in the scratch too), then a long row again after the short ones
    s3 = (np.floor(r.random((1, 8, 20000)) * 4096) / 4096).astype(np.float32)
    idx, inv = _both(tsa, s3, 700, Hkv=2, group_mode=1)
    widx, winv = orc.select(orc.group_scores(s3.astype(np.float64), 4), 700)
    assert np.array_equal(idx, widx) and np.array_equal(inv, winv)
    _both(tsa, s1[:1, :2, :17000].copy(), 17000)


def test_static_scratch_selection_rejects_what_does_not_fit(tsa):
    lib = tsa.load_library()
    cap = lib.tsa_select_static_capacity()
    assert cap >= 1 << 20
    # group mode keeps B * Hkv * L float32 sums in the scratch: choose L so that they alone exceed the capacity
    L = cap // 4 // 2 + 4096
    desc = tsa.make_desc(1, 4, 2, L, 128, 64, group_mode=1)
    s = torch.zeros((1, 4, L), dtype=torch.float32, device=gu.DEV)
    idx = torch.zeros((1, 2, 8), dtype=torch.int32, device=gu.DEV)
    with pytest.raises(tsa.TsaError) as e:
        tsa.tsa_select_static(desc, s, 8, idx, None)
    assert e.value.code == tsa.TSA_ERR_UNSUPPORTED and "static" in str(e.value)
