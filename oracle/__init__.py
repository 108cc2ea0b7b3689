"""ctypes front end of the plain-C CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It imports nothing from the GPU package and the GPU package
imports nothing from here.  See gbmw_oracle.c for what is computed and for the
arithmetic contract (Section 4.1.2, Eq. 3 and Appendix A of the paper).

All tables use the logical layout [l][e][s] (s fastest); a batch is handled by
looping over its instances.
"""
from __future__ import annotations

import ctypes as ct
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gbmw_oracle.c")
_LIB = os.path.join(_HERE, "libgbmw_oracle.so")
CFLAGS = ["-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
          "-fno-fast-math", "-fexcess-precision=standard", "-Wall", "-Wextra"]

_lib = None


def build(force: bool = False) -> str:
    """Compile gbmw_oracle.c with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", *CFLAGS, _SRC, "-o", tmp, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _bind(path: str):
    """Load one build of the oracle and declare its prototypes."""
    lib = ct.CDLL(path)
    f32p, i32p, u8p, i64p = (ct.POINTER(ct.c_float), ct.POINTER(ct.c_int32),
                             ct.POINTER(ct.c_uint8), ct.POINTER(ct.c_int64))
    lib.gbmw_oracle_plan_cost.argtypes = [ct.c_int, ct.c_int, f32p, i32p, f32p, u8p, f32p, i64p]
    lib.gbmw_oracle_plan_cost.restype = None
    lib.gbmw_oracle_bruteforce.argtypes = [ct.c_int, ct.c_int, ct.c_int, f32p, i32p, f32p,
                                           f32p, i64p, ct.c_int, u8p, ct.c_int64]
    lib.gbmw_oracle_bruteforce.restype = ct.c_int64
    lib.gbmw_oracle_solve.argtypes = [ct.c_int, ct.c_int, ct.c_int, f32p, i32p, f32p,
                                      f32p, u8p, f32p, f32p, u8p, ct.c_int]
    lib.gbmw_oracle_solve.restype = ct.c_int
    lib.gbmw_oracle_backtrack.argtypes = [ct.c_int, ct.c_int, ct.c_int, i32p, u8p, f32p, u8p,
                                          ct.c_int, u8p, f32p, i64p]
    lib.gbmw_oracle_backtrack.restype = None
    lib.gbmw_oracle_max_threads.restype = ct.c_int
    lib.gbmw_oracle_e_all.argtypes = [ct.c_int, ct.c_int, i32p, i32p, i32p, u8p]
    lib.gbmw_oracle_e_all.restype = ct.c_int64
    lib.gbmw_oracle_select_budget.argtypes = [ct.c_int, ct.c_int, ct.c_int, i32p, u8p, f32p, u8p,
                                              i32p, i32p, i32p, ct.POINTER(ct.c_int32), f32p, u8p, i64p]
    lib.gbmw_oracle_select_budget.restype = None
    lib.gbmw_oracle_pipeline_cost.argtypes = [ct.c_int, ct.c_int, f32p, f32p]
    lib.gbmw_oracle_pipeline_cost.restype = ct.c_float
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build())
    return _lib


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(ct.POINTER(ty))


def _chk(a, dtype, shape):
    assert a.dtype == dtype and a.flags.c_contiguous and a.shape == shape, (a.dtype, a.shape, shape)
    return a


def max_threads() -> int:
    return int(_load().gbmw_oracle_max_threads())


def plan_cost(c, M, R, plan):
    """(cost float32, mem int) of one plan by the plain definition."""
    L, S = c.shape
    plan = np.ascontiguousarray(plan, dtype=np.uint8)
    assert L >= 1 and plan.shape == (L,) and int(plan.max()) < S, "not a plan of this instance"
    cost, mem = ct.c_float(), ct.c_int64()
    _load().gbmw_oracle_plan_cost(L, S, _p(_chk(c, np.float32, (L, S)), ct.c_float),
                                  _p(_chk(M, np.int32, (L, S)), ct.c_int32),
                                  _p(_chk(R, np.float32, (L, S, S)), ct.c_float),
                                  _p(plan, ct.c_uint8), ct.byref(cost), ct.byref(mem))
    return np.float32(cost.value), int(mem.value)


def bruteforce(c, M, R, E, e_q=-1, limit=1 << 26):
    """opt[E+1], nopt[E+1], first optimal plan at e_q (or None)."""
    L, S = c.shape
    opt = np.empty(E + 1, np.float32)
    nopt = np.empty(E + 1, np.int64)
    plan = np.empty(L, np.uint8)
    n = _load().gbmw_oracle_bruteforce(L, S, E, _p(_chk(c, np.float32, (L, S)), ct.c_float),
                                       _p(_chk(M, np.int32, (L, S)), ct.c_int32),
                                       _p(_chk(R, np.float32, (L, S, S)), ct.c_float),
                                       _p(opt, ct.c_float), _p(nopt, ct.c_int64), int(e_q),
                                       _p(plan, ct.c_uint8), int(limit))
    if n < 0:
        raise ValueError("S^L exceeds the enumeration limit")
    return opt, nopt, (plan if e_q >= 0 else None)


class Solution:
    """Tables of one instance: C [L][E+1][S] f32 (or None), A [L][E+1][S] u8
    (or None), T (or None), best [E+1] f32, best_s [E+1] u8."""

    def __init__(self, L, S, E, M, C, A, T, best, best_s):
        self.L, self.S, self.E, self.M = L, S, E, M
        self.C, self.A, self.T, self.best, self.best_s = C, A, T, best, best_s

    def backtrack(self, e_q: int):
        assert self.A is not None and 0 <= e_q <= self.E
        plan = np.empty(self.L, np.uint8)
        cost, mem = ct.c_float(), ct.c_int64()
        _load().gbmw_oracle_backtrack(self.L, self.S, self.E, _p(self.M, ct.c_int32),
                                      _p(self.A, ct.c_uint8), _p(self.best, ct.c_float),
                                      _p(self.best_s, ct.c_uint8), int(e_q),
                                      _p(plan, ct.c_uint8), ct.byref(cost), ct.byref(mem))
        return plan, np.float32(cost.value), int(mem.value)


def e_all(Of, Ob, Oms, plan) -> int:
    """Overall memory of one plan (Eq. 2)."""
    L, S = Of.shape
    plan = np.ascontiguousarray(plan, dtype=np.uint8)
    return int(_load().gbmw_oracle_e_all(L, S, _p(_chk(Of, np.int32, (L, S)), ct.c_int32),
                                         _p(_chk(Ob, np.int32, (L, S)), ct.c_int32),
                                         _p(_chk(Oms, np.int32, (L, S)), ct.c_int32), _p(plan, ct.c_uint8)))


def pipeline_cost(m: int, C, Cns) -> np.float32:
    """Eq. 5 / Eq. 8: (m - 1) * max Cns + sum C over the stages."""
    C = np.ascontiguousarray(C, np.float32)
    Cns = np.ascontiguousarray(Cns, np.float32)
    assert C.shape == Cns.shape and C.ndim == 1 and len(C) >= 1
    return np.float32(_load().gbmw_oracle_pipeline_cost(len(C), int(m), _p(C, ct.c_float), _p(Cns, ct.c_float)))


def select_budget(sol: "Solution", Of, Ob, Oms):
    """Algorithm 3's outer loop on a solved instance whose M was Of + Oms:
    (e_opt, cost, plan, e_all)."""
    L, S = Of.shape
    assert sol.A is not None and np.array_equal(sol.M, Of + Oms)
    e_opt, cost, ea = ct.c_int32(), ct.c_float(), ct.c_int64()
    plan = np.empty(L, np.uint8)
    _load().gbmw_oracle_select_budget(L, S, sol.E, _p(sol.M, ct.c_int32), _p(sol.A, ct.c_uint8),
                                      _p(sol.best, ct.c_float), _p(sol.best_s, ct.c_uint8),
                                      _p(_chk(Of, np.int32, (L, S)), ct.c_int32),
                                      _p(_chk(Ob, np.int32, (L, S)), ct.c_int32),
                                      _p(_chk(Oms, np.int32, (L, S)), ct.c_int32),
                                      ct.byref(e_opt), ct.byref(cost), _p(plan, ct.c_uint8), ct.byref(ea))
    return int(e_opt.value), np.float32(cost.value), plan, int(ea.value)


def solve(c, M, R, E, keep_C=True, keep_A=True, keep_T=False, nthreads=1) -> Solution:
    """Run the recurrence for one instance (c [L][S], M [L][S], R [L][S][S])."""
    L, S = c.shape
    _chk(c, np.float32, (L, S)); _chk(M, np.int32, (L, S)); _chk(R, np.float32, (L, S, S))
    C = np.empty((L, E + 1, S), np.float32) if keep_C else None
    A = np.empty((L, E + 1, S), np.uint8) if keep_A else None
    T = np.full((L, E + 1, S), np.nan, np.float32) if keep_T else None
    best = np.empty(E + 1, np.float32)
    best_s = np.empty(E + 1, np.uint8)
    rc = _load().gbmw_oracle_solve(L, S, E, _p(c, ct.c_float), _p(M, ct.c_int32), _p(R, ct.c_float),
                                   _p(C, ct.c_float), _p(A, ct.c_uint8), _p(T, ct.c_float),
                                   _p(best, ct.c_float), _p(best_s, ct.c_uint8), int(nthreads))
    if rc != 0:
        raise RuntimeError("oracle: bad sizes or out of memory")
    return Solution(L, S, E, M, C, A, T, best, best_s)


def solve_problem(prob, b: int, **kw) -> Solution:
    """Instance b of a batched problem (anything with L, c, M, R, E, offsets)."""
    o, n = int(prob.offsets[b]), int(prob.L[b])
    return solve(prob.c[o:o + n], prob.M[o:o + n], prob.R[o:o + n], prob.E, **kw)
