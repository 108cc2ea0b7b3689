"""gbmw_backtrack_static, the plan read-back for callers that must not allocate device memory:
its staging block is a fixed array inside the library's device image.  Through the C ABI, two
calls in a row on one context (the second with fewer queries, so that it runs over what the
first left in the block), against gbmw_backtrack on the same queries and against the oracle;
then a second context on the same GPU, and the size limit."""
import ctypes as ct

import numpy as np
import pytest

import gbmw_inputs as gi
import oracle
import pins

pytestmark = pytest.mark.gpu


def _raw_static(g, ctx, qi, qe):
    """The entry point on the raw symbol: plain pointers and sizes."""
    lib = ct.CDLL(g.LIB_PATH)
    fn = lib.gbmw_backtrack_static
    fn.argtypes = [ct.c_void_p, ct.c_int32] + [ct.c_void_p] * 5
    fn.restype = ct.c_int
    nq, Lmax = len(qi), g.gbmw_max_layers(ctx)
    plan = np.full((nq, Lmax), 0xAB, np.uint8)
    cost = np.full(nq, np.nan, np.float32)
    mem = np.full(nq, -99, np.int32)
    rc = fn(ctx.handle, nq, qi.ctypes.data, qe.ctypes.data, plan.ctypes.data, cost.ctypes.data, mem.ctypes.data)
    return rc, plan, cost, mem


def _same(a, b):
    for x, y in zip(a, b):
        assert np.array_equal(np.ascontiguousarray(x).view(np.uint8), np.ascontiguousarray(y).view(np.uint8))


@pytest.mark.parametrize("flags", [0, 16], ids=["records", "lazy-argmin"])
def test_static_backtrack_matches_the_allocating_one(flags):
    import paper_2307_02031_amd as g
    p = gi.stack([gi.random_instance(3300 + i, L, 11, 2500, M_rng=(1, 400)) for i, L in enumerate([9, 4, 1, 7])], "static")
    ctx = g.gbmw_dp_solve_batched(p.L, p.c, p.M, p.R, p.S, p.E, flags=flags)
    g.gbmw_synchronize(ctx)
    st = gi.Stream(3400)
    # first call: 3000 queries (incl. infeasible budgets); second: 37 queries, other instances first
    for nq, seed_shift in ((3000, 0), (37, 1)):
        qi = np.ascontiguousarray((st.integers(nq, 0, p.B - 1) + seed_shift) % p.B, dtype=np.int32)
        qe = np.ascontiguousarray(st.integers(nq, 0, p.E), dtype=np.int32)
        print(f"static backtrack: {nq} queries, flags={flags}", flush=True)
        rc, plan, cost, mem = _raw_static(g, ctx, qi, qe)
        assert rc == g.GBMW_OK, g.gbmw_last_error()
        _same((plan, cost, mem), g.gbmw_backtrack(ctx, qi, qe))
        _same((plan, cost, mem), g.gbmw_backtrack_static(ctx, qi, qe))
        # and against the oracle, on a sample
        refs = [oracle.solve_problem(p, b, keep_C=False, keep_A=True) for b in range(p.B)]
        for i in range(0, nq, max(1, nq // 60)):
            b, Lb = int(qi[i]), int(p.L[int(qi[i])])
            rp, rc_, rm = refs[b].backtrack(int(qe[i]))
            if np.isinf(rc_):
                assert np.isinf(cost[i]) and mem[i] == -1 and np.all(plan[i] == 255)
            else:
                assert np.array_equal(plan[i, :Lb], rp) and np.all(plan[i, Lb:] == 255)
                assert pins.bits(cost[i]) == pins.bits(rc_) and int(mem[i]) == rm
    # another context on the same GPU shares the block
    p2 = gi.random_instance(3500, 5, 6, 300, M_rng=(1, 60))
    ctx2 = g.gbmw_dp_solve_batched(p2.L, p2.c, p2.M, p2.R, p2.S, p2.E, flags=flags)
    qi = np.zeros(50, np.int32); qe = np.ascontiguousarray(np.arange(251, 301), dtype=np.int32)
    _same(g.gbmw_backtrack_static(ctx2, qi, qe), g.gbmw_backtrack(ctx2, qi, qe))
    qi = np.ascontiguousarray(np.arange(8) % p.B, dtype=np.int32); qe = np.full(8, p.E, np.int32)
    _same(g.gbmw_backtrack_static(ctx, qi, qe), g.gbmw_backtrack(ctx, qi, qe))
    g.gbmw_destroy(ctx2)
    g.gbmw_destroy(ctx)


def test_static_backtrack_limit_and_errors():
    import paper_2307_02031_amd as g
    p = gi.random_instance(3600, 6, 5, 200, M_rng=(1, 30))
    ctx = g.gbmw_dp_solve_batched(p.L, p.c, p.M, p.R, p.S, p.E)
    Lmax = g.gbmw_max_layers(ctx)
    fits = g.GBMW_STATIC_SCRATCH_BYTES // (16 + Lmax)
    for nq, ok in ((fits, True), (fits + 1, False)):
        qi = np.zeros(nq, np.int32); qe = np.full(nq, p.E, np.int32)
        rc, plan, cost, mem = _raw_static(g, ctx, qi, qe)
        if ok:
            assert rc == g.GBMW_OK, g.gbmw_last_error()
            ref = g.gbmw_backtrack(ctx, qi[:1], qe[:1])
            assert np.all(plan == ref[0][0]) and np.all(cost == ref[1][0]) and np.all(mem == ref[2][0])
        else:
            assert rc == g.GBMW_ERR_UNSUPPORTED and "static block" in g.gbmw_last_error()
            assert np.all(plan == 0xAB) and np.all(mem == -99)        # nothing was written
    with pytest.raises(g.GbmwError):
        g.gbmw_backtrack_static(ctx, [1], [0])                          # no such instance
    with pytest.raises(g.GbmwError):
        g.gbmw_backtrack_static(ctx, [0], [p.E + 1])
    plan, cost, mem = g.gbmw_backtrack_static(ctx, np.zeros(0, np.int32), np.zeros(0, np.int32))
    assert plan.shape == (0, Lmax)
    g.gbmw_destroy(ctx)
