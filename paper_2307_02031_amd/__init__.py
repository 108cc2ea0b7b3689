"""Python binding of libgbmw.so, the gfx950 library for the batched layer-wise
strategy search (Section 4.1.2, Eq. 3 and Appendix A of the paper).

The functions here have the names of the C entry points in include/gbmw.h and
only marshal arguments: every step of the search runs in the library's HIP
kernels.  There is no CPU fallback -- if the library has not been built
(``python -m paper_2307_02031_amd.build``) importing this package raises.

PyTorch is used for device memory and streams only: device-resident inputs are
torch CUDA tensors whose ``data_ptr()`` is handed to the library, and work is
enqueued on ``torch.cuda.current_stream()`` unless a stream is given.
"""
from __future__ import annotations

import ctypes as ct
import os

import numpy as np
import torch  # imported first so that the library binds to the same HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgbmw.so")

GBMW_OK, GBMW_ERR_INVALID_ARG, GBMW_ERR_UNSUPPORTED, GBMW_ERR_OOM, GBMW_ERR_DEVICE = range(5)
GBMW_PTR_HOST, GBMW_PTR_DEVICE = 0, 1
GBMW_FLAG_KEEP_ALL_C = 1
GBMW_FLAG_TIME_KERNELS = 2
GBMW_FLAG_ONE_STREAM = 4
GBMW_FLAG_RESOLVE_ALL = 8
GBMW_FLAG_LAZY_ARGMIN = 16
GBMW_FLAG_DENSE_ARITHMETIC = 32
GBMW_FLAG_COUNT_WORK = 64
GBMW_FLAG_LAYER_LAUNCHES = 128
GBMW_FLAG_TEST_WAIT_GIVES_UP = 256
GBMW_FLAG_COOPERATIVE_LAUNCH = 512
GBMW_MAX_S = 256
GBMW_STATIC_SCRATCH_BYTES = 1 << 20

EXPORTS = [
    "gbmw_dp_solve_batched", "gbmw_backtrack", "gbmw_backtrack_static", "gbmw_select_forward_budget", "gbmw_pipeline_cost",
    "gbmw_partition_search", "gbmw_enumerate_strategies", "gbmw_cost_model",
    "gbmw_max_layers", "gbmw_get_best",
    "gbmw_export_tables", "gbmw_synchronize", "gbmw_last_solve_ms", "gbmw_last_solve_work", "gbmw_destroy",
    "gbmw_last_error", "gbmw_version",
]


class gbmw_problem(ct.Structure):
    _fields_ = [("B", ct.c_int32), ("S", ct.c_int32), ("E", ct.c_int32),
                ("L", ct.c_void_p), ("c", ct.c_void_p), ("M", ct.c_void_p), ("R", ct.c_void_p),
                ("ptr_space", ct.c_int32), ("stream", ct.c_void_p)]


class gbmw_partition_problem(ct.Structure):
    _fields_ = [("n_chain", ct.c_int32), ("S", ct.c_int32), ("E", ct.c_int32), ("max_iter", ct.c_int32),
                ("P", ct.c_void_p), ("Lm", ct.c_void_p), ("m", ct.c_void_p), ("c", ct.c_void_p),
                ("c_nosync", ct.c_void_p), ("R", ct.c_void_p), ("M", ct.c_void_p), ("p0", ct.c_void_p),
                ("p_t", ct.c_void_p), ("stream", ct.c_void_p), ("batch_size", ct.c_void_p),
                ("batch_group", ct.c_void_p), ("O_b", ct.c_void_p), ("O_ms", ct.c_void_p)]


class gbmw_partition_result(ct.Structure):
    _fields_ = [("n_iter", ct.c_void_p), ("O_t", ct.c_void_p), ("p", ct.c_void_p), ("cost", ct.c_void_p),
                ("C", ct.c_void_p), ("Cns", ct.c_void_p), ("O", ct.c_void_p), ("alpha_t", ct.c_void_p),
                ("alpha_m", ct.c_void_p), ("strat", ct.c_void_p),
                ("rounds", ct.c_int32), ("stage_solves", ct.c_int32), ("cell_updates", ct.c_int64),
                ("device_ms", ct.c_float), ("tpt", ct.c_float), ("tpt_group", ct.c_int32),
                ("tpt_pair", ct.c_int32)]


class gbmw_strategy(ct.Structure):
    _fields_ = [("n_levels", ct.c_int32), ("kind", ct.c_int32 * 3), ("degree", ct.c_int32 * 3), ("ckpt", ct.c_int32)]


class gbmw_hardware(ct.Structure):
    _fields_ = [("rate", ct.c_double), ("bw_in", ct.c_double), ("bw_out", ct.c_double),
                ("param_bytes", ct.c_double), ("state_bytes", ct.c_double), ("slow", ct.c_double),
                ("unit_bytes", ct.c_double), ("island", ct.c_int32)]


STRATEGY_DTYPE = np.dtype([("n_levels", np.int32), ("kind", np.int32, 3), ("degree", np.int32, 3), ("ckpt", np.int32)])
GBMW_DP, GBMW_SDP, GBMW_TP = 1, 2, 3


class GbmwError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"gbmw status {status}: {message}")
        self.status = status


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2307_02031_amd.build` "
                      "(there is no CPU fallback)")
_lib = ct.CDLL(LIB_PATH)
_lib.gbmw_dp_solve_batched.argtypes = [ct.POINTER(gbmw_problem), ct.c_uint32, ct.POINTER(ct.c_void_p)]
_lib.gbmw_dp_solve_batched.restype = ct.c_int
_lib.gbmw_backtrack.argtypes = [ct.c_void_p, ct.c_int32] + [ct.c_void_p] * 5
_lib.gbmw_backtrack.restype = ct.c_int
_lib.gbmw_backtrack_static.argtypes = [ct.c_void_p, ct.c_int32] + [ct.c_void_p] * 5
_lib.gbmw_backtrack_static.restype = ct.c_int
_lib.gbmw_select_forward_budget.argtypes = [ct.c_void_p] * 8
_lib.gbmw_select_forward_budget.restype = ct.c_int
_lib.gbmw_pipeline_cost.argtypes = [ct.c_void_p, ct.c_int32] + [ct.c_void_p] * 8
_lib.gbmw_pipeline_cost.restype = ct.c_int
_lib.gbmw_partition_search.argtypes = [ct.POINTER(gbmw_partition_problem), ct.c_uint32,
                                       ct.POINTER(gbmw_partition_result), ct.POINTER(ct.c_void_p)]
_lib.gbmw_partition_search.restype = ct.c_int
_lib.gbmw_enumerate_strategies.argtypes = [ct.c_int32, ct.c_int32, ct.c_int32, ct.c_void_p, ct.c_int32]
_lib.gbmw_enumerate_strategies.restype = ct.c_int32
_lib.gbmw_cost_model.argtypes = [ct.c_void_p, ct.c_int32, ct.c_void_p, ct.c_int32, ct.POINTER(gbmw_hardware),
                                 ct.c_double, ct.c_int32, ct.c_int32] + [ct.c_void_p] * 8
_lib.gbmw_cost_model.restype = ct.c_int
_lib.gbmw_max_layers.argtypes = [ct.c_void_p]
_lib.gbmw_max_layers.restype = ct.c_int32
_lib.gbmw_get_best.argtypes = [ct.c_void_p, ct.c_void_p, ct.c_void_p]
_lib.gbmw_get_best.restype = ct.c_int
_lib.gbmw_export_tables.argtypes = [ct.c_void_p, ct.c_int32, ct.c_int32, ct.c_int32, ct.c_void_p, ct.c_void_p]
_lib.gbmw_export_tables.restype = ct.c_int
_lib.gbmw_synchronize.argtypes = [ct.c_void_p]
_lib.gbmw_synchronize.restype = ct.c_int
_lib.gbmw_last_solve_ms.argtypes = [ct.c_void_p, ct.POINTER(ct.c_float), ct.POINTER(ct.c_float),
                                    ct.POINTER(ct.c_int32)]
_lib.gbmw_last_solve_ms.restype = ct.c_int
_lib.gbmw_last_solve_work.argtypes = [ct.c_void_p, ct.c_int32, ct.POINTER(ct.c_uint64)]
_lib.gbmw_last_solve_work.restype = ct.c_int
_lib.gbmw_destroy.argtypes = [ct.c_void_p]
_lib.gbmw_destroy.restype = None
_lib.gbmw_last_error.restype = ct.c_char_p
_lib.gbmw_version.restype = ct.c_char_p


def gbmw_last_error() -> str:
    return _lib.gbmw_last_error().decode()


def gbmw_version() -> str:
    return _lib.gbmw_version().decode()


def _check(status: int):
    if status != GBMW_OK:
        raise GbmwError(status, gbmw_last_error())


class Context:
    """Owner of a gbmw_ctx*; keeps the arrays handed to the library alive."""

    def __init__(self):
        self.handle = ct.c_void_p(None)
        self.B = self.S = self.E = 0
        self.L = None
        self._keep = ()

    def __del__(self):
        try:
            gbmw_destroy(self)
        except Exception:
            pass


def _ptr(a):
    if isinstance(a, torch.Tensor):
        return a.data_ptr()
    return a.ctypes.data


def gbmw_dp_solve_batched(L, c, M, R, S: int, E: int, flags: int = 0, ctx: Context | None = None,
                          stream: int | None = None) -> Context:
    """Enqueue the table fill for B = len(L) instances.

    c [sumL][S] f32, M [sumL][S] i32, R [sumL][S][S] f32: either all numpy
    arrays (host) or all torch CUDA tensors (device, used in place).  Returns
    the context (a new one unless ``ctx`` is given)."""
    L = np.ascontiguousarray(L, dtype=np.int32)
    on_dev = isinstance(c, torch.Tensor)
    if on_dev:
        assert all(isinstance(x, torch.Tensor) and x.is_cuda and x.is_contiguous() for x in (c, M, R))
        assert c.dtype == torch.float32 and M.dtype == torch.int32 and R.dtype == torch.float32
    else:
        c = np.ascontiguousarray(c, dtype=np.float32)
        M = np.ascontiguousarray(M, dtype=np.int32)
        R = np.ascontiguousarray(R, dtype=np.float32)
    sumL = int(L.sum())
    assert tuple(c.shape) == (sumL, S) and tuple(M.shape) == (sumL, S) and tuple(R.shape) == (sumL, S, S)
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
    p = gbmw_problem(len(L), S, E, L.ctypes.data, _ptr(c), _ptr(M), _ptr(R),
                     GBMW_PTR_DEVICE if on_dev else GBMW_PTR_HOST, stream)
    if ctx is None:
        ctx = Context()
    _check(_lib.gbmw_dp_solve_batched(ct.byref(p), flags, ct.byref(ctx.handle)))
    ctx.B, ctx.S, ctx.E, ctx.L = len(L), S, E, L
    ctx._keep = (L, c, M, R)
    return ctx


def gbmw_synchronize(ctx: Context) -> None:
    _check(_lib.gbmw_synchronize(ctx.handle))


def gbmw_max_layers(ctx: Context) -> int:
    return int(_lib.gbmw_max_layers(ctx.handle))


def gbmw_get_best(ctx: Context):
    """best [B][E+1] float32, best_s [B][E+1] uint8 (host arrays)."""
    best = np.empty((ctx.B, ctx.E + 1), np.float32)
    best_s = np.empty((ctx.B, ctx.E + 1), np.uint8)
    _check(_lib.gbmw_get_best(ctx.handle, best.ctypes.data, best_s.ctypes.data))
    return best, best_s


def gbmw_backtrack(ctx: Context, q_instance, q_e):
    """plan [nq][Lmax] uint8 (0xFF padded), cost [nq] float32, mem_used [nq] int32."""
    qi = np.ascontiguousarray(q_instance, dtype=np.int32)
    qe = np.ascontiguousarray(q_e, dtype=np.int32)
    assert qi.shape == qe.shape and qi.ndim == 1
    nq, Lmax = len(qi), gbmw_max_layers(ctx)
    plan = np.empty((nq, Lmax), np.uint8)
    cost = np.empty(nq, np.float32)
    mem = np.empty(nq, np.int32)
    _check(_lib.gbmw_backtrack(ctx.handle, nq, qi.ctypes.data, qe.ctypes.data, plan.ctypes.data,
                               cost.ctypes.data, mem.ctypes.data))
    return plan, cost, mem


def gbmw_backtrack_static(ctx: Context, q_instance, q_e):
    """gbmw_backtrack through the library's fixed staging block (no device allocation)."""
    qi = np.ascontiguousarray(q_instance, dtype=np.int32)
    qe = np.ascontiguousarray(q_e, dtype=np.int32)
    assert qi.shape == qe.shape and qi.ndim == 1
    nq, Lmax = len(qi), gbmw_max_layers(ctx)
    plan = np.empty((nq, Lmax), np.uint8)
    cost = np.empty(nq, np.float32)
    mem = np.empty(nq, np.int32)
    _check(_lib.gbmw_backtrack_static(ctx.handle, nq, qi.ctypes.data, qe.ctypes.data, plan.ctypes.data,
                                      cost.ctypes.data, mem.ctypes.data))
    return plan, cost, mem


def gbmw_select_forward_budget(ctx: Context, O_f, O_b, O_ms):
    """Algorithm 3's outer loop: e_opt [B] int32, cost [B] float32, plan [B][Lmax] uint8,
    e_all [B] int32 (host arrays)."""
    sumL = int(ctx.L.sum())
    arrs = [np.ascontiguousarray(a, dtype=np.int32) for a in (O_f, O_b, O_ms)]
    assert all(a.shape == (sumL, ctx.S) for a in arrs)
    Lmax = gbmw_max_layers(ctx)
    e_opt = np.empty(ctx.B, np.int32)
    cost = np.empty(ctx.B, np.float32)
    plan = np.empty((ctx.B, Lmax), np.uint8)
    e_all = np.empty(ctx.B, np.int32)
    _check(_lib.gbmw_select_forward_budget(ctx.handle, arrs[0].ctypes.data, arrs[1].ctypes.data,
                                           arrs[2].ctypes.data, e_opt.ctypes.data, cost.ctypes.data,
                                           plan.ctypes.data, e_all.ctypes.data))
    return e_opt, cost, plan, e_all


def gbmw_pipeline_cost(ctx: Context, stage_begin, stage_instance, stage_e, microbatches, c_nosync=None):
    """Eq. 5 / Eq. 8: cost [n_pipe], stage_cost [n_stage], stage_cost_nosync [n_stage] (float32)."""
    sb = np.ascontiguousarray(stage_begin, dtype=np.int32)
    si = np.ascontiguousarray(stage_instance, dtype=np.int32)
    se = np.ascontiguousarray(stage_e, dtype=np.int32)
    mb = np.ascontiguousarray(microbatches, dtype=np.int32)
    n_pipe = len(mb)
    assert sb.shape == (n_pipe + 1,) and si.shape == se.shape == (int(sb[-1]),)
    cns = None if c_nosync is None else np.ascontiguousarray(c_nosync, dtype=np.float32)
    if cns is not None:
        assert cns.shape == (int(ctx.L.sum()), ctx.S)
    cost = np.empty(n_pipe, np.float32)
    sc = np.empty(len(si), np.float32)
    scn = np.empty(len(si), np.float32)
    _check(_lib.gbmw_pipeline_cost(ctx.handle, n_pipe, sb.ctypes.data, si.ctypes.data, se.ctypes.data,
                                   mb.ctypes.data, None if cns is None else cns.ctypes.data,
                                   cost.ctypes.data, sc.ctypes.data, scn.ctypes.data))
    return cost, sc, scn


def gbmw_partition_search(P, Lm, m, c, c_nosync, R, M, p0, p_t, S: int, E: int, max_iter: int = 64,
                          flags: int = 0, ctx: Context | None = None, stream: int | None = None,
                          batch_size=None, batch_group=None, O_b=None, O_ms=None):
    """Algorithm 2's inner loop for n_chain = len(P) pairs (host numpy arrays, the
    pairs' rows concatenated; c_nosync and p_t may be None; O_b and O_ms, shaped like M,
    switch the stage searches to Appendix A's forward-budget selection).  Returns (result dict,
    ctx): n_iter, O_t [n]; p, C, Cns, O [n][max_iter][Pmax]; cost, alpha_t, alpha_m
    [n][max_iter]; strat [n][Lmmax]; rounds, stage_solves, cell_updates, device_ms."""
    i32 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.int32)
    f32 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.float32)
    P, Lm, m, M, p0, p_t = (i32(a) for a in (P, Lm, m, M, p0, p_t))
    c, c_nosync, R, batch_size = (f32(a) for a in (c, c_nosync, R, batch_size))
    batch_group, O_b, O_ms = i32(batch_group), i32(O_b), i32(O_ms)
    n, sumLm, sumP = len(P), int(Lm.sum()), int(P.sum())
    sumPL = int((P.astype(np.int64) * Lm).sum())
    assert Lm.shape == m.shape == (n,) and c.shape == (sumLm, S) and R.shape == (sumLm, S, S)
    assert M.shape == (sumPL, S) and p0.shape == (sumP,)
    assert c_nosync is None or c_nosync.shape == c.shape
    assert p_t is None or p_t.shape == p0.shape
    assert (O_b is None or O_b.shape == M.shape) and (O_ms is None or O_ms.shape == M.shape)
    Pmax, Lmmax = int(P.max()), int(Lm.max())
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
    ptr = lambda a: None if a is None else a.ctypes.data
    q = gbmw_partition_problem(n, S, E, max_iter, ptr(P), ptr(Lm), ptr(m), ptr(c), ptr(c_nosync), ptr(R),
                               ptr(M), ptr(p0), ptr(p_t), stream, ptr(batch_size), ptr(batch_group),
                               ptr(O_b), ptr(O_ms))
    mi = max(1, max_iter)
    res = dict(n_iter=np.zeros(n, np.int32), O_t=np.zeros(n, np.int32),
               p=np.zeros((n, mi, Pmax), np.int32), cost=np.zeros((n, mi), np.float32),
               C=np.zeros((n, mi, Pmax), np.float32), Cns=np.zeros((n, mi, Pmax), np.float32),
               O=np.zeros((n, mi, Pmax), np.int32), alpha_t=np.zeros((n, mi), np.float32),
               alpha_m=np.zeros((n, mi), np.float32), strat=np.zeros((n, Lmmax), np.uint8))
    out = gbmw_partition_result(*[res[k].ctypes.data for k in ("n_iter", "O_t", "p", "cost", "C", "Cns", "O",
                                                               "alpha_t", "alpha_m", "strat")], 0, 0, 0, 0.0, 0.0, -1, -1)
    if ctx is None:
        ctx = Context()
    _check(_lib.gbmw_partition_search(ct.byref(q), flags, ct.byref(out), ct.byref(ctx.handle)))
    ctx.B = ctx.S = ctx.E = 0
    ctx.L, ctx._keep = None, ()
    res.update(rounds=out.rounds, stage_solves=out.stage_solves, cell_updates=out.cell_updates,
               device_ms=out.device_ms, tpt=np.float32(out.tpt), tpt_group=out.tpt_group, tpt_pair=out.tpt_pair)
    return res, ctx


def gbmw_enumerate_strategies(group_size: int, with_ckpt: bool = True, takeaway3: bool = True) -> np.ndarray:
    """Structured array (STRATEGY_DTYPE) of the candidate strategies of one layer."""
    n = _lib.gbmw_enumerate_strategies(group_size, int(with_ckpt), int(takeaway3), None, 0)
    if n < 0:
        raise GbmwError(GBMW_ERR_INVALID_ARG, gbmw_last_error())
    out = np.zeros(n, STRATEGY_DTYPE)
    assert STRATEGY_DTYPE.itemsize == ct.sizeof(gbmw_strategy)
    _lib.gbmw_enumerate_strategies(group_size, int(with_ckpt), int(takeaway3), out.ctypes.data, n)
    return out


def gbmw_cost_model(layers, strategies, hw: dict, Bm: float, P: int, device: bool = False,
                    stream: int | None = None) -> dict:
    """c, c_nosync [L][S] f32; O_f, O_b, O_ms [L][S] i32; M [P][L][S] i32; R [L][S][S] f32 --
    numpy arrays, or torch CUDA tensors if ``device``.  layers: float64 [L][4] (params,
    flops, bnd, intm); strategies: STRATEGY_DTYPE array."""
    layers = np.ascontiguousarray(layers, dtype=np.float64)
    strategies = np.ascontiguousarray(strategies, dtype=STRATEGY_DTYPE)
    L, S = len(layers), len(strategies)
    assert layers.shape == (L, 4)
    h = gbmw_hardware(hw["rate"], hw["bw_in"], hw["bw_out"], hw["param_bytes"], hw["state_bytes"], hw["slow"],
                      hw["unit_bytes"], hw["island"])
    shapes = dict(c=((L, S), np.float32), c_nosync=((L, S), np.float32), O_f=((L, S), np.int32),
                  O_b=((L, S), np.int32), O_ms=((L, S), np.int32), M=((P, L, S), np.int32), R=((L, S, S), np.float32))
    if device:
        tdt = {np.float32: torch.float32, np.int32: torch.int32}
        out = {k: torch.empty(sh, dtype=tdt[dt], device="cuda") for k, (sh, dt) in shapes.items()}
    else:
        out = {k: np.empty(sh, dt) for k, (sh, dt) in shapes.items()}
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
    _check(_lib.gbmw_cost_model(layers.ctypes.data, L, strategies.ctypes.data, S, ct.byref(h), float(Bm), P,
                                GBMW_PTR_DEVICE if device else GBMW_PTR_HOST,
                                *[_ptr(out[k]) for k in ("c", "c_nosync", "O_f", "O_b", "O_ms", "M", "R")], stream))
    return out


def gbmw_export_tables(ctx: Context, instance: int, l0: int = 0, l1: int | None = None,
                       want_C: bool = True, want_A: bool = True):
    """C [l1-l0][E+1][S] float32 and A [l1-l0][E+1][S] uint8 (None if not wanted)."""
    if l1 is None:
        l1 = int(ctx.L[instance])
    n = max(0, l1 - l0)
    C = np.empty((n, ctx.E + 1, ctx.S), np.float32) if want_C else None
    A = np.empty((n, ctx.E + 1, ctx.S), np.uint8) if want_A else None
    _check(_lib.gbmw_export_tables(ctx.handle, instance, l0, l1,
                                   C.ctypes.data if want_C else None,
                                   A.ctypes.data if want_A else None))
    return C, A


def gbmw_last_solve_ms(ctx: Context):
    """(total_ms, minplus_ms, minplus_launches) of the last solve."""
    a, b, n = ct.c_float(), ct.c_float(), ct.c_int32()
    _check(_lib.gbmw_last_solve_ms(ctx.handle, ct.byref(a), ct.byref(b), ct.byref(n)))
    return a.value, b.value, n.value


def gbmw_last_solve_work(ctx: Context, launch: int = -1):
    """(wide workgroups, run waves by summary, run waves by value, dense rows) of the last counted
    solve: of one min-plus launch, or summed over all (launch = -1)."""
    w = (ct.c_uint64 * 4)()
    _check(_lib.gbmw_last_solve_work(ctx.handle, launch, w))
    return tuple(int(x) for x in w)


def gbmw_destroy(ctx: Context) -> None:
    if ctx.handle:
        _lib.gbmw_destroy(ctx.handle)
        ctx.handle = ct.c_void_p(None)
        ctx._keep = ()
