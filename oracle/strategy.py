"""Candidate hybrid-parallelism strategies of one layer (Section 3.2: the
decision trees, their construction rules and Takeaway #3) and a small analytic
cost model in the spirit of Section 5 that turns layer shapes into the search's
inputs c, c_nosync, O_f, O_b, O_ms, M and R -- TEST INFRASTRUCTURE ONLY (see the
package docstring for who may import this).

What the paper fixes and this file follows:
  * a tree's levels are distinct paradigms out of DP, SDP, TP with degrees from
    {2, 4, 8, ...} whose product is the device-group size; the order of the
    levels matters; every tree exists with and without CKPT (Section 3.2 rules);
  * Takeaway #3 removes the trees that hold both DP and SDP;
  * per-layer communication volumes 2(N-1)/N (DP all-reduce) and 3(N-1)/N (SDP:
    two all-gathers and a reduce-scatter) of the parameter bytes (Takeaway #3);
  * backward computation = twice the forward; CKPT adds one more forward (and,
    with TP, its all-reduce); overlapped computation and communication slow each
    other down by 1.3x (Section 5);
  * CKPT keeps only the boundary activations in the forward pass and needs the
    intermediate ones during backward (Section 3.1);
  * O_f, O_b, O_ms and E_all as in Eq. 2.
Everything else (which tensors TP replicates, the transformation cost, the
bandwidth a level sees, bytes per parameter) is this build's choice, stated in
the functions below.  All arithmetic is fp64 in the order written; times are
rounded to fp32 and memories to integer units at the end.
"""
from __future__ import annotations

import itertools
import math

import numpy as np

DP, SDP, TP = 1, 2, 3
NAMES = {DP: "DP", SDP: "SDP", TP: "TP"}


def _factorisations(g):
    """Ordered tuples of factors from {2, 4, 8, ...} with product g."""
    if g == 1:
        return [()]
    out = []
    d = 2
    while d <= g:
        if g % d == 0:
            out += [(d,) + rest for rest in _factorisations(g // d)]
        d *= 2
    return out


def enumerate_strategies(g, ckpt=True, takeaway3=True):
    """All trees for a device group of g devices (g a power of two), outer level
    first: list of (levels, ckpt_flag) with levels = ((paradigm, degree), ...).
    Order: fewer levels first; then degrees lexicographically; then paradigms
    lexicographically (DP < SDP < TP); all trees without CKPT, then all with."""
    assert g >= 1 and g & (g - 1) == 0
    trees = []
    for degs in sorted(_factorisations(g), key=lambda t: (len(t), t)):
        if len(degs) > 3:
            continue                         # three paradigms: at most three levels
        for kinds in itertools.permutations((DP, SDP, TP), len(degs)):
            if takeaway3 and DP in kinds and SDP in kinds:
                continue
            trees.append(tuple(zip(kinds, degs)))
    out = [(t, 0) for t in trees]
    if ckpt:
        out += [(t, 1) for t in trees]
    return out


def describe(levels, ckpt):
    s = "-".join(f"{NAMES[k]}{d}" for k, d in levels) or "single"
    return s + ("+CKPT" if ckpt else "")


def degrees(levels):
    """(dp, sdp, tp, span_dp, span_sdp, span_tp): degree of each paradigm (1 if
    absent) and the number of consecutive devices its groups stretch over: its
    own degree times the degrees of the levels inside it."""
    deg = {DP: 1, SDP: 1, TP: 1}
    span = {DP: 1, SDP: 1, TP: 1}
    inner = 1
    for k, d in reversed(levels):
        deg[k] = d
        span[k] = d * inner
        inner *= d
    return deg[DP], deg[SDP], deg[TP], span[DP], span[SDP], span[TP]


def layout_key(levels):
    """How the activations of a layer are laid out over the group: batch-split
    levels (DP and SDP alike) and TP levels, outer first."""
    return tuple(("B" if k in (DP, SDP) else "T", d) for k, d in levels)


def overlap(a, b, slow):
    """Two activities started together, each slowed by `slow` while both run:
    the shorter ends after slow*min, by then the longer has min of its own work
    behind it: total = slow*min + (max - min)."""
    lo, hi = (a, b) if a <= b else (b, a)
    return slow * lo + (hi - lo)


def layer_costs(layer, levels, ckpt, hw, Bm):
    """One (layer, strategy): dict(c, c_ns, ms, act_f, act_b) in seconds / bytes (fp64).
    layer: dict(params, flops, bnd, int); hw: dict(rate, bw_in, bw_out, island,
    param_bytes, state_bytes, slow)."""
    dp, sdp, tp, sp_dp, sp_sdp, sp_tp = degrees(levels)
    bw = lambda span: hw["bw_in"] if span <= hw["island"] else hw["bw_out"]
    lb = Bm / (dp * sdp)                                   # samples per device
    t_f = lb * layer["flops"] / tp / hw["rate"]
    t_b = 2.0 * t_f
    tp_ar = 2.0 * (tp - 1) / tp * (lb * layer["bnd"]) / bw(sp_tp) if tp > 1 else 0.0
    pbytes = layer["params"] * hw["param_bytes"] / tp
    sdp_ag = (sdp - 1) / sdp * pbytes / bw(sp_sdp) if sdp > 1 else 0.0      # one all-gather
    dp_ar = 2.0 * (dp - 1) / dp * pbytes / bw(sp_dp) if dp > 1 else 0.0
    fwd = t_f + tp_ar + sdp_ag
    bwd = t_b + tp_ar
    if ckpt:
        bwd = bwd + (t_f + tp_ar)                          # recomputation, with TP's all-reduce
    sync = dp_ar + sdp_ag                                  # gradient all-reduce / reduce-scatter
    c = fwd + overlap(bwd, sdp_ag + sync, hw["slow"])      # SDP gathers the parameters again for backward
    c_ns = fwd + overlap(bwd, sdp_ag, hw["slow"])
    ms = layer["params"] * hw["state_bytes"] / (tp * sdp)
    if ckpt:
        act_f, act_b = lb * layer["bnd"], lb * (layer["int"] / tp)
    else:
        act_f, act_b = lb * (layer["bnd"] + layer["int"] / tp), 0.0
    return dict(c=c, c_ns=c_ns, ms=ms, act_f=act_f, act_b=act_b)


def transform_cost(bnd_prev, lev_prev, lev, hw, Bm):
    """Slice-Gather between neighbouring layers: nothing if the two layouts are
    the same; otherwise the boundary activations of the micro-batch are
    re-distributed over the slow links: the difference of the per-device shares
    if the batch-split degrees differ, one share if only the order differs."""
    if layout_key(lev_prev) == layout_key(lev):
        return 0.0
    dp0, sdp0, *_ = degrees(lev_prev)
    dp1, sdp1, *_ = degrees(lev)
    b0, b1 = dp0 * sdp0, dp1 * sdp1
    share = abs(1.0 / b1 - 1.0 / b0) if b0 != b1 else 1.0 / b1
    return Bm * bnd_prev * share / hw["bw_out"]


def units(x, unit):
    return int(math.ceil(x / unit))


def cost_model(layers, strategies, hw, Bm, P, unit):
    """The search's inputs for one pipeline stage group: c, c_ns f32 [L][S];
    O_f, O_b, O_ms i32 [L][S]; M i32 [P][L][S] with M[i] = O_ms + (P - i) * O_f
    (stage i of a 1F1B pipeline holds the forward activations of P - i
    micro-batches); R f32 [L][S][S] (R[l][s'][s], layer 0's slab zero)."""
    L, S = len(layers), len(strategies)
    c = np.zeros((L, S), np.float32); c_ns = np.zeros((L, S), np.float32)
    Of = np.zeros((L, S), np.int32); Ob = np.zeros((L, S), np.int32); Oms = np.zeros((L, S), np.int32)
    R = np.zeros((L, S, S), np.float32)
    for l, layer in enumerate(layers):
        for s, (lev, ck) in enumerate(strategies):
            v = layer_costs(layer, lev, ck, hw, Bm)
            c[l, s], c_ns[l, s] = np.float32(v["c"]), np.float32(v["c_ns"])
            Of[l, s], Ob[l, s], Oms[l, s] = units(v["act_f"], unit), units(v["act_b"], unit), units(v["ms"], unit)
            if l > 0:
                for sp, (levp, _) in enumerate(strategies):
                    R[l, sp, s] = np.float32(transform_cost(layers[l - 1]["bnd"], levp, lev, hw, Bm))
    M = np.stack([Oms + (P - i) * Of for i in range(P)]).astype(np.int32)
    return dict(c=c, c_ns=c_ns, O_f=Of, O_b=Ob, O_ms=Oms, M=M, R=R)
