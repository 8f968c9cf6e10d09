"""Host-side checks of the synthetic input generator and of the margin helper."""
import numpy as np

from oracle import tsa_oracle as orc
from paper_2602_03216_amd import inputs as gen
from tests.margin import enforce_margin, RHO


def test_generator_is_deterministic_and_shaped():
    a = gen.make_inputs(1)
    b = gen.make_inputs(1)
    assert a.Q.shape == (1, 4, 1024, 64) and a.K.shape == (1, 4, 1024, 64) and a.Q.dtype == np.uint16
    assert np.array_equal(a.Q, b.Q) and np.array_equal(a.K, b.K) and np.array_equal(a.V, b.V)
    c = gen.make_inputs(1, seed=5)
    assert not np.array_equal(a.Q, c.Q)
    assert all(len(p) == 64 and p.max() < 1024 - 64 for p in a.planted)
    assert not np.array_equal(a.planted[0], a.planted[1])


def test_bf16_rounding_of_generator_matches_oracle_rounding():
    x = np.random.Generator(np.random.PCG64(3)).standard_normal(100000).astype(np.float32)
    assert np.array_equal(gen.f32_to_bf16_bits(x), orc.f64_to_bf16(x.astype(np.float64)))


def test_config1_planted_tokens_are_selected_and_margin_holds():
    inp = gen.make_inputs(1)
    s, margin = enforce_margin(inp, [256])
    assert margin >= RHO
    idx, _ = orc.select(s, 256)
    for h in range(4):
        assert np.isin(inp.planted[h], idx[0, h]).all()


def test_reduced_gqa_recipe_with_sinks():
    inp = gen.make_inputs(3, L=2048)
    assert inp.Q.shape == (1, 32, 2048, 128) and inp.K.shape == (1, 8, 2048, 128)
    ks = [orc.keep_count(2048, t) for t in (0.5, 0.75, 0.9)]
    s, margin = enforce_margin(inp, ks)
    assert margin >= RHO
    idx, _ = orc.select(s, ks[-1])
    assert np.all(idx[0, :, :4] == np.arange(4))          # the four sink tokens are kept by every head
    rec = np.mean([np.isin(inp.planted[h], idx[0, h]).mean() for h in range(32)])
    assert rec > 0.9


def test_sink_window_block_list_matches_the_pair_predicate():
    """The generator's block list lists key block kb for query block qb exactly when kb <= qb and
    (kb is a sink block or qb - kb <= window / block): checked pair by pair, and against the
    list the oracle builds for its own attention."""
    for Lc, bs, win, ns in ((1000, 128, 256, 1), (4096, 128, 4096, 1), (777, 64, 128, 2), (130, 128, 512, 1)):
        bl = gen.sink_window_block_list(Lc, bs, win, ns)
        nb = (Lc + bs - 1) // bs
        assert bl.shape[0] == nb
        for qb in range(nb):
            row = [int(v) for v in bl[qb] if v >= 0]
            assert row == sorted(set(row))
            want = [kb for kb in range(nb) if kb <= qb and (kb < ns or qb - kb <= win // bs)]
            assert row == want
        ref = orc.lambda_block_list(Lc, bs, win, ns)
        assert all([v for v in a if v >= 0] == [v for v in b if v >= 0] for a, b in zip(bl.tolist(), ref.tolist()))
