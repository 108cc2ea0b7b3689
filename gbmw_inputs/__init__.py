"""Seeded synthetic inputs for the layer-wise strategy search (data only).

This module produces the *problem statements* the search consumes -- per-layer
execution cost c(l, s), forward memory M(l, s) = O_f + O_ms in budget units,
transformation cost R(l, s', s) and the forward budget E (Section 4.1.2, Eq. 3
of the paper) -- for a batch of independent (pipeline stage x PP degree x batch
size x partition) searches (Algorithm 1 / Algorithm 2 call the search once per
stage).  It contains none of the search's arithmetic: no recurrence, no min, no
backtracking.  Both the CPU oracle's tests and the GPU library's tests draw
their inputs here, so the two sides see identical bits.

Everything is generated from a counter-based 64-bit mixer written out below, so
the values do not depend on numpy's generator implementation or version.

Memory layout of a :class:`Problem` (all C-contiguous):
    L  int32 [B]            layers per instance
    c  float32 [sumL][S]    rows of instance b start at off_b = L[0]+..+L[b-1]
    M  int32   [sumL][S]
    R  float32 [sumL][S][S] R[off_b + l][s_prev][s]; the l == 0 slab is unused
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass

import numpy as np

__all__ = [
    "Problem", "Stream", "make_config", "random_instance", "stack", "split_memory",
    "CONFIG_NAMES", "PipelineModel", "random_pipeline_model", "structured_pipeline_model",
    "uniform_pipeline_model", "with_memory_split", "proportional_partition", "TABLE1", "table1_layers", "default_hardware",
]

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser applied element-wise to uint64 values."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


class Stream:
    """Counter-based random stream: value i of stream (seed, lane) is a pure
    function of (seed, lane, i)."""

    def __init__(self, seed: int, lane: int = 0):
        with np.errstate(over="ignore"):
            k = _mix(np.array([seed], dtype=np.uint64) * _GOLD + np.uint64(0x1234567))
            k = _mix(k ^ (np.array([lane], dtype=np.uint64) * _M2 + np.uint64(0x89ABCDEF)))
        self._key = k[0]
        self._ctr = 0

    def bits(self, n: int) -> np.ndarray:
        ctr = np.arange(self._ctr, self._ctr + n, dtype=np.uint64)
        self._ctr += n
        with np.errstate(over="ignore"):
            return _mix(self._key + ctr * _GOLD)

    def unit(self, n: int) -> np.ndarray:
        """n values in [0, 1) with 24 random bits each (exact in float32)."""
        return (self.bits(n) >> np.uint64(40)).astype(np.float64) * (1.0 / (1 << 24))

    def uniform(self, n: int, lo: float, hi: float) -> np.ndarray:
        """float32 values in [lo, hi): lo + (hi - lo) * u evaluated in float64,
        rounded once to float32 and clipped just below hi."""
        v = (lo + (hi - lo) * self.unit(n)).astype(np.float32)
        top = np.nextafter(np.float32(hi), np.float32(lo))
        return np.minimum(v, top)

    def integers(self, n: int, lo: int, hi: int) -> np.ndarray:
        """int64 values uniform on {lo, ..., hi} (inclusive)."""
        span = np.uint64(hi - lo + 1)
        r = ((self.bits(n) >> np.uint64(32)) * span) >> np.uint64(32)
        return r.astype(np.int64) + lo


@dataclass
class Problem:
    B: int
    S: int
    E: int
    L: np.ndarray
    c: np.ndarray
    M: np.ndarray
    R: np.ndarray
    name: str = ""

    def __post_init__(self):
        self.L = np.ascontiguousarray(self.L, dtype=np.int32)
        self.c = np.ascontiguousarray(self.c, dtype=np.float32)
        self.M = np.ascontiguousarray(self.M, dtype=np.int32)
        self.R = np.ascontiguousarray(self.R, dtype=np.float32)
        sumL = int(self.L.sum())
        assert self.L.shape == (self.B,)
        assert self.c.shape == (sumL, self.S), self.c.shape
        assert self.M.shape == (sumL, self.S), self.M.shape
        assert self.R.shape == (sumL, self.S, self.S), self.R.shape

    @property
    def sumL(self) -> int:
        return int(self.L.sum())

    @property
    def offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.L)[:-1]]).astype(np.int64)

    def instance(self, b: int) -> "Problem":
        """The b-th instance as a B == 1 problem (views, no copy)."""
        o = int(self.offsets[b])
        n = int(self.L[b])
        return Problem(1, self.S, self.E, self.L[b:b + 1], self.c[o:o + n],
                       self.M[o:o + n], self.R[o:o + n], f"{self.name}[{b}]")

    def nominal_updates(self) -> int:
        """sum_b L_b * E * S * S  (the metric's B.L.E.S.S')."""
        return int(self.L.astype(np.int64).sum()) * self.E * self.S * self.S

    def executed_updates(self) -> int:
        """sum_b (L_b - 1) * (E + 1) * S * S: layer 0 has no contraction and the
        table has rows e = 0..E."""
        return int((self.L.astype(np.int64) - 1).sum()) * (self.E + 1) * self.S * self.S


def stack(problems, name: str = "") -> Problem:
    """Concatenate single- or multi-instance problems that share S and E."""
    S, E = problems[0].S, problems[0].E
    assert all(p.S == S and p.E == E for p in problems)
    return Problem(
        B=sum(p.B for p in problems), S=S, E=E,
        L=np.concatenate([p.L for p in problems]),
        c=np.concatenate([p.c for p in problems]),
        M=np.concatenate([p.M for p in problems]),
        R=np.concatenate([p.R for p in problems]), name=name)


def _zero_diag(R: np.ndarray) -> np.ndarray:
    S = R.shape[-1]
    R[..., np.arange(S), np.arange(S)] = 0.0
    return R


def _uniform_instance(st: Stream, L: int, S: int, c_rng, M_rng, R_rng) -> tuple:
    """Draw order: all c (l-major, s-minor), then all M, then all R (l, s', s)."""
    c = st.uniform(L * S, *c_rng).reshape(L, S)
    M = st.integers(L * S, *M_rng).reshape(L, S)
    R = _zero_diag(st.uniform(L * S * S, *R_rng).reshape(L, S, S))
    return c, M, R


def random_instance(seed: int, L: int, S: int, E: int, c_rng=(1.0, 10.0),
                    M_rng=(1, 32), R_rng=(0.0, 2.0), name: str = "") -> Problem:
    c, M, R = _uniform_instance(Stream(seed), L, S, c_rng, M_rng, R_rng)
    return Problem(1, S, E, np.array([L]), c, M, R, name or f"rand{seed}")


# --------------------------------------------------------------------------
# Structured instances: 22 base strategies x {no checkpointing, checkpointing}
# (the paper's 8-GPU strategy set has 22 entries without and 44 with
# activation checkpointing, Section 3.2 / Section 7.3).
# --------------------------------------------------------------------------
def _round_half_away(x: np.ndarray) -> np.ndarray:
    return np.sign(x) * np.floor(np.abs(x) + 0.5)


def _structured_instance(st: Stream, L: int, S: int, act_scale: float = 1.0,
                         cost_scale: float = 1.0) -> tuple:
    """Strategy s = (j, k): base j = s mod 22, k = s div 22 (1 = checkpointing).
    shard_j = 2^(j mod 4).  Memory: half of Mbase_l is model state, half is
    activation (scaled by act_scale); checkpointing halves the activation part;
    both parts divide by shard_j.  Cost: cbase_l * (1/shard_j + 0.02*(j div 4)),
    +25% under checkpointing.  R is zero between strategies with the same base
    j (they share a data layout) and U[0, 5) otherwise."""
    assert S % 22 == 0 and S // 22 in (1, 2)
    s = np.arange(S)
    j, k = s % 22, s // 22
    shard = (2.0 ** (j % 4))
    Mbase = st.integers(L, 512, 4096).astype(np.float64)
    cbase = st.uniform(L, 5.0, 50.0).astype(np.float64) * cost_scale
    state = Mbase[:, None] / 2.0
    act = (Mbase[:, None] / 2.0) * act_scale * np.where(k == 1, 0.5, 1.0)[None, :]
    M = np.maximum(1.0, _round_half_away((state + act) / shard[None, :])).astype(np.int64)
    c = (cbase[:, None] * (1.0 / shard + 0.02 * (j // 4))[None, :]
         * np.where(k == 1, 1.25, 1.0)[None, :]).astype(np.float32)
    R = st.uniform(L * S * S, 0.0, 5.0).reshape(L, S, S)
    same = (j[:, None] == j[None, :])
    R[:, same] = 0.0
    return c, M, R


CONFIG_NAMES = {
    1: "cfg1 single L=4 S=4 E=256",
    2: "cfg2 single BERT-Large-shaped L=24 S=22 E=8192",
    3: "cfg3 single structured L=32 S=44 E=16384",
    4: "cfg4 batched B=64 L~U[6,24] S=44 E=32768",
    5: "cfg5 large batched B=16 L=96 S=64 E=65536",
}


def make_config(k: int, B: int | None = None) -> Problem:
    """The five benchmark workloads.  ``B`` truncates the batched configs (4, 5)
    to their first B instances (instances are generated independently, so the
    prefix is identical to the prefix of the full batch)."""
    if k == 1:
        c, M, R = _uniform_instance(Stream(0), 4, 4, (1.0, 10.0), (1, 32), (0.0, 2.0))
        return Problem(1, 4, 256, np.array([4]), c, M, R, CONFIG_NAMES[1])
    if k == 2:
        c, M, R = _uniform_instance(Stream(1), 24, 22, (5.0, 50.0), (64, 1024), (0.0, 5.0))
        return Problem(1, 22, 8192, np.array([24]), c, M, R, CONFIG_NAMES[2])
    if k == 3:
        c, M, R = _structured_instance(Stream(2), 32, 44)
        return Problem(1, 44, 16384, np.array([32]), c, M, R, CONFIG_NAMES[3])
    if k == 4:
        nB = 64 if B is None else B
        Ls = Stream(3, lane=1 << 20).integers(64, 6, 24)
        parts = []
        for b in range(nB):
            q = (b // 4) % 4            # batch-size index; b = (p*4 + q)*4 + r
            scale = (2.0 ** q) / 4.0
            c, M, R = _structured_instance(Stream(3, lane=b), int(Ls[b]), 44,
                                           act_scale=scale, cost_scale=scale)
            parts.append(Problem(1, 44, 32768, np.array([Ls[b]]), c, M, R))
        return stack(parts, CONFIG_NAMES[4] if nB == 64 else f"cfg4[:{nB}]")
    if k == 5:
        nB = 16 if B is None else B
        parts = []
        for b in range(nB):
            c, M, R = _uniform_instance(Stream(4, lane=b), 96, 64, (1.0, 100.0),
                                        (128, 2048), (0.0, 10.0))
            parts.append(Problem(1, 64, 65536, np.array([96]), c, M, R))
        return stack(parts, CONFIG_NAMES[5] if nB == 16 else f"cfg5[:{nB}]")
    raise ValueError(f"unknown config {k}")


def split_memory(p: Problem, seed: int, ob_max: int | None = None):
    """Synthetic O_f, O_b, O_ms [sumL][S] int32 for the overall-memory check of
    Algorithm 3, with O_f + O_ms == M: the model-state share of each M is a
    uniform fraction, O_b ~ U{0..ob_max} (default: the largest M)."""
    st = Stream(seed, lane=77)
    n, S = p.M.shape
    frac = st.unit(n * S).reshape(n, S)
    Oms = np.floor(p.M.astype(np.float64) * frac).astype(np.int32)
    Of = (p.M - Oms).astype(np.int32)
    hi = max(1, int(p.M.max())) if ob_max is None else ob_max
    Ob = st.integers(n * S, 0, hi).reshape(n, S).astype(np.int32)
    return np.ascontiguousarray(Of), np.ascontiguousarray(Ob), np.ascontiguousarray(Oms)


# --------------------------------------------------------------------------
# Whole models cut into pipeline stages (inputs of Algorithm 2's partition
# loop).  The memory of a layer depends on the stage it sits in: under 1F1B
# stage i of P keeps the activations of P - i micro-batches (Section 4.2.1).
# --------------------------------------------------------------------------
@dataclass
class PipelineModel:
    """One (batch size, PP degree) pair: Lm layers, P stages, m micro-batches.
    c, c_ns float32 [Lm][S]; R float32 [Lm][S][S]; M int32 [P][Lm][S];
    p0, p_t int32 [P] (initial and time-balanced partition: layers per stage).
    Ob, Oms: optional int32 [P][Lm][S] (backward activations and model states,
    the latter a part of M) for stage searches with the overall-memory check of
    Appendix A."""
    S: int
    E: int
    P: int
    m: int
    c: np.ndarray
    c_ns: np.ndarray
    R: np.ndarray
    M: np.ndarray
    p0: np.ndarray
    p_t: np.ndarray | None
    name: str = ""
    Ob: np.ndarray | None = None
    Oms: np.ndarray | None = None

    def __post_init__(self):
        self.c = np.ascontiguousarray(self.c, dtype=np.float32)
        self.c_ns = np.ascontiguousarray(self.c_ns, dtype=np.float32)
        self.R = np.ascontiguousarray(self.R, dtype=np.float32)
        self.M = np.ascontiguousarray(self.M, dtype=np.int32)
        self.p0 = np.ascontiguousarray(self.p0, dtype=np.int32)
        if self.p_t is not None:
            self.p_t = np.ascontiguousarray(self.p_t, dtype=np.int32)
        Lm = self.c.shape[0]
        assert self.c.shape == (Lm, self.S) and self.c_ns.shape == (Lm, self.S)
        assert self.R.shape == (Lm, self.S, self.S) and self.M.shape == (self.P, Lm, self.S)
        for p in (self.p0, self.p_t):
            assert p is None or (p.shape == (self.P,) and p.min() >= 1 and int(p.sum()) == Lm)

    @property
    def Lm(self) -> int:
        return self.c.shape[0]

    def as_dict(self) -> dict:
        d = dict(c=self.c, c_ns=self.c_ns, R=self.R, M=self.M)
        if self.Ob is not None:
            d.update(Ob=self.Ob, Oms=self.Oms)
        return d


def with_memory_split(mod: PipelineModel, seed: int, ob_max: int | None = None) -> PipelineModel:
    """The same model with synthetic O_b and O_ms tables [P][Lm][S]: the
    model-state share of every M entry is a uniform fraction of it (so that
    0 <= O_ms <= M), O_b ~ U{0..ob_max} (default: the largest M of the last
    stage), drawn per stage as well so that no two stages share a table."""
    st = Stream(seed, lane=78)
    frac = st.unit(mod.M.size).reshape(mod.M.shape)
    Oms = np.floor(mod.M.astype(np.float64) * frac).astype(np.int32)
    hi = max(1, int(mod.M[-1].max())) if ob_max is None else ob_max
    Ob = st.integers(mod.M.size, 0, hi).reshape(mod.M.shape).astype(np.int32)
    return dataclasses.replace(mod, Ob=np.ascontiguousarray(Ob), Oms=np.ascontiguousarray(Oms),
                               name=mod.name + "+split")


def proportional_partition(Lm: int, weights) -> np.ndarray:
    """Layer counts proportional to the weights, each at least 1, summing to Lm
    (largest remainders first, the earlier stage on a tie)."""
    w = np.asarray(weights, np.float64)
    P = len(w)
    assert Lm >= P
    share = (Lm - P) * w / w.sum()
    p = np.floor(share).astype(np.int64)
    rest = Lm - P - int(p.sum())
    order = sorted(range(P), key=lambda i: (-(share[i] - p[i]), i))
    for i in order[:rest]:
        p[i] += 1
    return (p + 1).astype(np.int32)


def _stage_memory(state, act, P):
    """M[i] = state + act * (P - i), rounded half away from zero, at least 1."""
    inflight = np.arange(P, 0, -1, dtype=np.float64)
    M = state[None] + act[None] * inflight[:, None, None]
    return np.maximum(1.0, _round_half_away(M)).astype(np.int64)


def random_pipeline_model(seed: int, Lm: int, S: int, P: int, E: int, m: int = 4,
                          c_rng=(1.0, 10.0), M_rng=(1, 8), R_rng=(0.0, 2.0),
                          with_pt: bool = True, skew: bool = False, name: str = "") -> PipelineModel:
    """Unstructured model: c, state and activation memory, R uniform;
    c_ns = c * U[0.5, 1); p0 favours deep stages (weights 1..P; with skew: one
    layer per stage and all the others on the last), p_t is even."""
    st = Stream(seed, lane=5)
    c = st.uniform(Lm * S, *c_rng).reshape(Lm, S)
    c_ns = (c.astype(np.float64) * st.uniform(Lm * S, 0.5, 1.0).reshape(Lm, S)).astype(np.float32)
    state = st.integers(Lm * S, *M_rng).reshape(Lm, S).astype(np.float64)
    act = st.integers(Lm * S, *M_rng).reshape(Lm, S).astype(np.float64) / 2.0
    R = _zero_diag(st.uniform(Lm * S * S, *R_rng).reshape(Lm, S, S))
    M = _stage_memory(state, act, P)
    p0 = proportional_partition(Lm, [0.0] * (P - 1) + [1.0] if skew else np.arange(1, P + 1))
    p_t = proportional_partition(Lm, np.ones(P)) if with_pt else None
    return PipelineModel(S, E, P, m, c, c_ns, R, M, p0, p_t, name or f"pipe-rand{seed}")


def structured_pipeline_model(seed: int, Lm: int, P: int, E: int, m: int = 8, S: int = 44,
                              act_scale: float = 1.0, name: str = "") -> PipelineModel:
    """The 22/44-strategy layer model of _structured_instance as a whole model:
    state = Mbase/8, activation per in-flight micro-batch = Mbase/2 * act_scale
    (halved under checkpointing), both divided by shard_j; c_ns = 0.8 c for the
    data-parallel-heavy bases (j mod 4 < 2), c otherwise.  p0 puts more layers
    on deep stages (weights 1/(P - i), inverse to the micro-batches in flight),
    p_t is the even split."""
    st = Stream(seed, lane=6)
    c, _, R = _structured_instance(st, Lm, S)
    s = np.arange(S)
    j, k = s % 22, s // 22
    shard = 2.0 ** (j % 4)
    Mbase = Stream(seed, lane=7).integers(Lm, 512, 4096).astype(np.float64)
    state = (Mbase[:, None] / 8.0) / shard[None, :]
    act = (Mbase[:, None] / 2.0) * act_scale * np.where(k == 1, 0.5, 1.0)[None, :] / shard[None, :]
    M = _stage_memory(state, act, P)
    c_ns = (c.astype(np.float64) * np.where(j % 4 < 2, 0.8, 1.0)[None, :]).astype(np.float32)
    w = 1.0 / np.arange(P, 0, -1)
    return PipelineModel(S, E, P, m, c, c_ns, R, M, proportional_partition(Lm, w),
                         proportional_partition(Lm, np.ones(P)), name or f"pipe-struct{seed}")


def uniform_pipeline_model(Lm: int, P: int, E: int, p0, cost: float = 2.0, r: float = 0.5,
                           mem=None, m: int = 2, p_t=None) -> PipelineModel:
    """S = 1, every layer alike: time cost, transformation r, memory mem[i] per
    layer in stage i (default 1).  A stage of n layers then takes exactly
    n*cost + (n-1)*r (dyadic values) and mem[i]*n memory."""
    mem = [1] * P if mem is None else mem
    c = np.full((Lm, 1), cost, np.float32)
    R = np.full((Lm, 1, 1), r, np.float32)
    M = np.array([[[mem[i]]] * Lm for i in range(P)], np.int32)
    return PipelineModel(1, E, P, m, c, c * np.float32(0.5), R, M, np.array(p0), p_t, "pipe-uniform")


# --------------------------------------------------------------------------
# Layer shapes for the analytic cost model: rows of the paper's model table
# (Table 1: layers, hidden size, parameters, activation bytes per sample), cut
# into equal layers.  Shapes only: the cost model itself lives elsewhere.
# --------------------------------------------------------------------------
TABLE1 = {
    # name: (layers, hidden, parameters, activation MB per sample, tokens per sample)
    "BERT-Huge-32": (32, 1280, 672e6, 3149.39, 512),
    "BERT-Huge-48": (48, 1280, 987e6, 4657.51, 512),
    "BERT-xHuge": (128, 2560, 10.2e9, 24210.05, 512),
    "ViT-Huge-32": (32, 1280, 632e6, 646.5, 197),
    "GPT3-15B": (48, 5120, 15.4e9, 32889.04, 2048),
}


def table1_layers(name: str, layers: int | None = None) -> np.ndarray:
    """float64 [L][4]: parameters, forward FLOPs per sample, boundary and
    intermediate activation bytes per sample of each layer.  A layer holds
    1/L of the parameters and of the activations; forward FLOPs = 2 x parameters
    x tokens; the boundary activation is tokens x hidden x 2 bytes.  ``layers``
    repeats the model's layer that many times instead (the paper's search-time
    figure varies the depth of one architecture)."""
    L, hidden, params, act_mb, tokens = TABLE1[name]
    p = params / L
    act = act_mb * 2.0 ** 20 / L
    bnd = float(tokens * hidden * 2)
    assert bnd < act
    row = [p, 2.0 * p * tokens, bnd, act - bnd]
    return np.ascontiguousarray(np.tile(np.array(row, np.float64), (L if layers is None else layers, 1)))


def default_hardware(unit_mb: float = 8.0) -> dict:
    """A100-class node of 8 devices in NVLink islands of 8, as in the paper's
    testbed description: numbers are round figures, not measurements."""
    return dict(rate=150e12, bw_in=150e9, bw_out=12.5e9, param_bytes=2.0, state_bytes=16.0, slow=1.3,
                unit_bytes=unit_mb * 2.0 ** 20, island=8)
