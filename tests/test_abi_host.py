"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and validates arguments before launching anything."""
import ctypes
import os
import re

import pytest

from oracle import tsa_oracle as orc
from paper_2602_03216_amd import binding as tsa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return tsa.load_library()


def test_every_declared_symbol_is_exported(lib):
    declared = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):       # tsa.h (the method) and tsa_bench.h (measurement support)
        header = open(os.path.join(ROOT, "include", name)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared |= set(re.findall(r"\b(tsa_[a-z_]+)\s*\(", header))
    assert declared == set(tsa.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_desc_struct_matches_header(lib):
    assert ctypes.sizeof(tsa.tsa_desc) == 120
    assert lib.tsa_version() == 10


def test_keep_count_matches_oracle_rule(lib):
    for L in (1, 2, 10, 1024, 8192, 32768, 65536, 131072, 100003):
        for tau in (0.0, 0.3, 0.5, 0.75, 0.9, 0.999, 1.0):
            assert tsa.tsa_keep_count(L, tau) == orc.keep_count(L, tau)
    assert tsa.tsa_keep_count(0, 0.5) == 0 and tsa.tsa_keep_count(10, 1.5) == 0 and tsa.tsa_keep_count(10, -0.1) == 0


def test_workspace_bytes(lib):
    d = tsa.make_desc(1, 32, 8, 131072, 128)
    n = tsa.tsa_workspace_bytes(d, 32768)
    # at least the scores, the two index maps and the V tiles
    assert n >= 32 * 131072 * 4 * 2 + 32 * 32768 * 4 + 32 * 32768 * 128 * 2
    assert n >= tsa.tsa_attend_workspace_bytes(d, 32768, 32)
    assert tsa.tsa_workspace_bytes(d, 0) == 0 and tsa.tsa_workspace_bytes(d, 131073) == 0
    assert tsa.tsa_workspace_bytes(tsa.make_desc(1, 32, 7, 1024, 128), 16) == 0
    assert "multiple" in tsa.tsa_last_error()
    assert tsa.tsa_workspace_bytes(tsa.make_desc(1, 4, 4, 1024, 96), 16) == 0
    assert tsa.tsa_workspace_bytes(tsa.make_desc(1, 1, 1, 1 << 23, 128), 16) == 0      # a head of 2 GiB: 32-bit offsets end here
    assert tsa.tsa_workspace_bytes(tsa.make_desc(1, 1, 1, (1 << 23) - 1, 128), 16) > 0
    assert tsa.tsa_workspace_bytes(tsa.make_desc(1, 4, 4, 32, 64, last_q=64), 16) == 0
    g1 = tsa.tsa_workspace_bytes(tsa.make_desc(1, 32, 8, 4096, 128, group_mode=1), 1024)
    g0 = tsa.tsa_workspace_bytes(tsa.make_desc(1, 32, 8, 4096, 128, group_mode=0), 1024)
    assert 0 < g1 < g0


def test_entry_points_reject_bad_arguments_before_any_launch(lib):
    d = tsa.make_desc(1, 4, 4, 1024, 64)
    dp = ctypes.byref(d)
    fake = ctypes.c_void_p(0x1000)       # aligned, never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1004)
    assert lib.tsa_score(dp, None, fake, fake, fake, 1 << 30, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_score(dp, odd, fake, fake, fake, 1 << 30, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_score(dp, fake, fake, fake, None, 0, None) == tsa.TSA_ERR_WORKSPACE
    assert lib.tsa_score(dp, fake, fake, fake, fake, 16, None) == tsa.TSA_ERR_WORKSPACE
    assert lib.tsa_select(dp, fake, 0, fake, fake, None, 0, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_select(dp, fake, 1025, fake, fake, None, 0, None) == tsa.TSA_ERR_ARG
    forced = tsa.make_desc(1, 4, 4, 1024, 64, force_first=4, force_last=7)       # 11 always-kept tokens need k_keep >= 11
    assert lib.tsa_select(ctypes.byref(forced), fake, 10, fake, fake, fake, 1 << 30, None) == tsa.TSA_ERR_ARG
    assert "force_first" in tsa.tsa_last_error()
    assert lib.tsa_forward(ctypes.byref(forced), fake, fake, fake, 10, None, 0, 0, fake, None, None, fake, 1 << 40, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_forward_dynamic(ctypes.byref(forced), fake, fake, fake, 0.01, 10, None, 0, 0, fake, None, None, None, fake, 1 << 40, None) == tsa.TSA_ERR_ARG
    # the general scorer takes 1..128 query rows whatever desc.last_q says
    assert lib.tsa_score_queries_workspace_bytes(dp, 0) == 0 and lib.tsa_score_queries_workspace_bytes(dp, 129) == 0
    assert lib.tsa_score_queries_workspace_bytes(dp, 100) >= lib.tsa_score_queries_workspace_bytes(dp, 3) > 0
    assert lib.tsa_copy_probe(fake, fake, 24, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_read_probe(fake, 24, fake, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_mix_probe(4, fake, 10, 8, fake, None, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_mix_probe(1, fake, 0, 8, fake, None, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_compress(dp, fake, fake, fake, None, 16, fake, fake, fake, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_attend(dp, fake, fake, fake, 0, 4, None, 0, 0, fake, None, fake, 1 << 30, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_attend(dp, fake, fake, fake, 16, 3, None, 0, 0, fake, None, fake, 1 << 30, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_attend(dp, fake, fake, fake, 256, 4, fake, 32, 3, fake, None, fake, 1 << 30, None) == tsa.TSA_ERR_UNSUPPORTED    # blocks of 64, 128, 256 only
    assert lib.tsa_attend(dp, fake, fake, fake, 256, 4, None, 0, 0, fake, None, fake, 64, None) == tsa.TSA_ERR_WORKSPACE
    assert tsa.tsa_attend_workspace_bytes(d, 100, 4) == 4 * 128 * 64 * 2 and tsa.tsa_attend_workspace_bytes(d, 100, 3) == 0
    assert lib.tsa_decompress(dp, fake, fake, fake, 16, None, None, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_forward(dp, fake, fake, fake, 16, None, 0, 0, fake, None, None, fake, 64, None) == tsa.TSA_ERR_WORKSPACE
    assert "workspace" in tsa.tsa_last_error()
    bad = tsa.make_desc(1, 4, 4, 1024, 64, pool_w=4)
    assert lib.tsa_score(ctypes.byref(bad), fake, fake, fake, fake, 1 << 30, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_coverage_budget(dp, fake, 1.5, fake, fake, 1 << 30, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_coverage_budget(dp, fake, 0.01, None, fake, 1 << 30, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_score(None, fake, fake, fake, fake, 1 << 30, None) == tsa.TSA_ERR_ARG
    # the layer with the budget decided on the device
    assert lib.tsa_forward_dynamic(dp, fake, fake, fake, 0.01, 0, None, 0, 0, fake, None, None, None, fake, 1 << 40, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_forward_dynamic(dp, fake, fake, fake, 1.5, 16, None, 0, 0, fake, None, None, None, fake, 1 << 40, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_forward_dynamic(dp, fake, fake, fake, 0.01, 16, None, 0, 0, None, None, None, None, fake, 1 << 40, None) == tsa.TSA_ERR_ARG
    assert lib.tsa_forward_dynamic(dp, fake, fake, fake, 0.01, 16, None, 0, 0, fake, None, None, None, fake, 64, None) == tsa.TSA_ERR_WORKSPACE
    assert lib.tsa_forward_dynamic_workspace_bytes(dp, 0) == 0
    assert lib.tsa_forward_dynamic_workspace_bytes(dp, 16) > lib.tsa_workspace_bytes(dp, 16)
