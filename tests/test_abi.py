"""The C-ABI boundary without a GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching the device."""
import ctypes as ct
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "gbmw.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gbmw_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2307_02031_amd as g
    names = _declared()
    assert "gbmw_dp_solve_batched" in names and "gbmw_backtrack" in names
    for n in names:
        assert hasattr(g._lib, n), f"{n} declared in gbmw.h but not exported"
    assert sorted(g.EXPORTS) == names
    assert "gfx950" in g.gbmw_version()


def test_binding_has_the_same_names():
    import paper_2307_02031_amd as g
    for n in _declared():
        assert callable(getattr(g, n)), n


def test_no_cpu_fallback_in_the_product_package():
    """The product never imports the oracle (and the oracle never imports it)."""
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2307_02031_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower(), f"{f} mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            assert "paper_2307_02031_amd" not in open(os.path.join(ROOT, "oracle", f)).read()


def _problem(g, L, c, M, R, S, E, space=0):
    L = np.ascontiguousarray(L, np.int32)
    p = g.gbmw_problem(len(L), S, E, L.ctypes.data, c.ctypes.data, M.ctypes.data, R.ctypes.data, space, None)
    p._keep = (L, c, M, R)
    return p


def test_argument_errors_are_reported_without_a_device():
    import paper_2307_02031_amd as g
    c = np.ones((2, 3), np.float32)
    M = np.ones((2, 3), np.int32)
    R = np.zeros((2, 3, 3), np.float32)
    h = ct.c_void_p(None)

    def status(p, flags=0):
        return g._lib.gbmw_dp_solve_batched(ct.byref(p), flags, ct.byref(h))

    assert g._lib.gbmw_dp_solve_batched(None, 0, ct.byref(h)) == g.GBMW_ERR_INVALID_ARG
    assert "null" in g.gbmw_last_error()
    assert status(_problem(g, [2], c, M, R, 0, 10)) == g.GBMW_ERR_INVALID_ARG       # S = 0
    assert status(_problem(g, [2], c, M, R, 257, 10)) == g.GBMW_ERR_INVALID_ARG     # S > 256
    assert status(_problem(g, [2], c, M, R, 3, -1)) == g.GBMW_ERR_INVALID_ARG       # E < 0
    assert status(_problem(g, [0], c, M, R, 3, 10)) == g.GBMW_ERR_INVALID_ARG       # L < 1
    assert status(_problem(g, [2], c, M, R, 3, 10, space=7)) == g.GBMW_ERR_INVALID_ARG
    assert status(_problem(g, [2], c, M, R, 3, 10), flags=2048) == g.GBMW_ERR_INVALID_ARG
    bad = c.copy(); bad[1, 2] = np.nan
    assert status(_problem(g, [2], bad, M, R, 3, 10)) == g.GBMW_ERR_INVALID_ARG
    assert "c[5]" in g.gbmw_last_error()
    bad = c.copy(); bad[0, 0] = -1.0
    assert status(_problem(g, [2], bad, M, R, 3, 10)) == g.GBMW_ERR_INVALID_ARG
    badM = M.copy(); badM[1, 0] = -3
    assert status(_problem(g, [2], c, badM, R, 3, 10)) == g.GBMW_ERR_INVALID_ARG
    badR = R.copy(); badR[1, 0, 1] = -np.inf
    assert status(_problem(g, [2], c, M, badR, 3, 10)) == g.GBMW_ERR_INVALID_ARG
    okR = R.copy(); okR[0, :, :] = np.nan          # the l == 0 slab is ignored
    st = status(_problem(g, [2], c, M, okR, 3, 10))
    assert st != g.GBMW_ERR_INVALID_ARG
    assert h.value is None or st == g.GBMW_OK
    if h.value:
        g._lib.gbmw_destroy(h)
    # calls on a null context
    assert g._lib.gbmw_synchronize(None) == g.GBMW_ERR_INVALID_ARG
    assert g._lib.gbmw_get_best(None, None, None) == g.GBMW_ERR_INVALID_ARG
    assert g._lib.gbmw_max_layers(None) == 0
    g._lib.gbmw_destroy(None)


def test_without_a_gpu_the_solve_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    import paper_2307_02031_amd as g
    c = np.ones((2, 3), np.float32)
    with pytest.raises(g.GbmwError) as ei:
        g.gbmw_dp_solve_batched([2], c, np.ones((2, 3), np.int32), np.zeros((2, 3, 3), np.float32), 3, 10)
    assert ei.value.status in (g.GBMW_ERR_DEVICE, g.GBMW_ERR_OOM)


def test_partition_search_rejects_bad_arguments_before_touching_the_device():
    import paper_2307_02031_amd as g
    import gbmw_inputs as gi
    mod = gi.uniform_pipeline_model(6, 2, 100, [2, 4], p_t=[3, 3])

    def status(max_iter=8, flags=0, **over):
        a = dict(P=[2], Lm=[6], m=[2], c=mod.c, c_nosync=mod.c_ns, R=mod.R, M=mod.M.reshape(12, 1),
                 p0=mod.p0, p_t=mod.p_t, S=1, E=100, O_b=None, O_ms=None)
        a.update(over)
        try:
            g.gbmw_partition_search(a["P"], a["Lm"], a["m"], a["c"], a["c_nosync"], a["R"], a["M"], a["p0"],
                                    a["p_t"], a["S"], a["E"], max_iter=max_iter, flags=flags,
                                    O_b=a["O_b"], O_ms=a["O_ms"])
        except g.GbmwError as e:
            return e.status, str(e)
        return g.GBMW_OK, ""

    for kw, word in [(dict(p0=np.array([2, 5])), "sums to"), (dict(p0=np.array([0, 6])), "empty"),
                     (dict(p_t=np.array([6, 0])), "empty"), (dict(m=[0]), "m[0]"), (dict(E=-1), "E="),
                     (dict(max_iter=0), "max_iter"), (dict(flags=1), "flag"),
                     (dict(c=-mod.c), "c[0]"), (dict(c_nosync=mod.c_ns * np.nan), "c_nosync[0]"),
                     (dict(M=-mod.M.reshape(12, 1)), "M[0]"),
                     (dict(O_b=np.zeros((12, 1), np.int32)), "go together"),
                     (dict(O_b=-np.ones((12, 1), np.int32), O_ms=np.zeros((12, 1), np.int32)), "O_b[0]"),
                     (dict(O_b=np.zeros((12, 1), np.int32), O_ms=mod.M.reshape(12, 1) + 1), "O_ms[0]"),
                     (dict(O_b=np.zeros((12, 1), np.int32), O_ms=-np.ones((12, 1), np.int32)), "O_ms[0]")]:
        st, msg = status(**kw)
        assert st == g.GBMW_ERR_INVALID_ARG and word in msg, (kw, st, msg)
    badR = mod.R.copy(); badR[1, 0, 0] = -1.0
    assert status(R=badR)[0] == g.GBMW_ERR_INVALID_ARG
    st, msg = status(P=[7], M=np.ones((42, 1), np.int32), p0=np.ones(7, np.int32), p_t=None)   # more stages than layers
    assert st == g.GBMW_ERR_INVALID_ARG and "Lm[0]" in msg
    assert g._lib.gbmw_partition_search(None, 0, None, None) == g.GBMW_ERR_INVALID_ARG
