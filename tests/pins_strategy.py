"""Pins of the oracle's strategy enumerator and analytic cost model: the counts
the paper states, an enumeration written a second way, the paper's Takeaway #3
argument, a hand-worked fixture and structural properties.  Each pin takes the
module under test so that the mutation tests can hand in a broken copy."""
import itertools
import json
import os

import numpy as np

import gbmw_inputs as gi
import pins


def pin_counts(st):
    """Section 3.2: 8 GPUs under PP 1/2/4/8 -> groups of 8/4/2/1: 34 trees (68 with
    CKPT); after Takeaway #3: 22 (44), i.e. 11 / 7 / 3 / 1 per group."""
    groups = (8, 4, 2, 1)
    assert [len(st.enumerate_strategies(g, ckpt=False, takeaway3=False)) for g in groups] == [21, 9, 3, 1]
    assert sum(len(st.enumerate_strategies(g, ckpt=True, takeaway3=False)) for g in groups) == 68
    assert [len(st.enumerate_strategies(g, ckpt=False, takeaway3=True)) for g in groups] == [11, 7, 3, 1]
    assert sum(len(st.enumerate_strategies(g, ckpt=True, takeaway3=True)) for g in groups) == 44


def brute_trees(g, takeaway3):
    """Every sequence of up to three (paradigm, degree) levels, filtered by the
    construction rules."""
    degs = [d for d in (2 ** k for k in range(1, 21)) if d <= g]
    out = set()
    for n in range(0, 4):
        for kinds in itertools.product((1, 2, 3), repeat=n):
            if len(set(kinds)) != n:
                continue                                 # no paradigm twice
            if takeaway3 and 1 in kinds and 2 in kinds:
                continue
            for ds in itertools.product(degs, repeat=n):
                if int(np.prod(ds, dtype=np.int64)) == g:
                    out.add(tuple(zip(kinds, ds)))
    return out


def pin_enumeration(st):
    for g in (1, 2, 4, 8, 16, 32):
        for t3 in (False, True):
            got = st.enumerate_strategies(g, ckpt=True, takeaway3=t3)
            trees = [t for t, ck in got if ck == 0]
            assert [t for t, ck in got if ck == 1] == trees and len(got) == 2 * len(trees)
            assert [ck for _, ck in got] == [0] * len(trees) + [1] * len(trees)
            assert len(set(trees)) == len(trees) and set(trees) == brute_trees(g, t3), (g, t3)
            # documented order
            key = lambda t: (len(t), tuple(d for _, d in t), tuple(k for k, _ in t))
            assert trees == sorted(trees, key=key)
            assert st.enumerate_strategies(g, ckpt=False, takeaway3=t3) == [(t, 0) for t in trees]


def _hw(g):
    return dict(g["hw"])


def pin_fixture(st):
    with open(os.path.join(pins.GOLDEN, "worked_example_cost_model.json")) as f:
        g = json.load(f)
    hw, layer, Bm = _hw(g), g["layer"], g["Bm"]
    for case in g["cases"]:
        lev = tuple(tuple(x) for x in case["levels"])
        v = st.layer_costs(layer, lev, case["ckpt"], hw, Bm)
        for k in ("c", "c_ns", "ms", "act_f", "act_b"):
            assert v[k] == case[k], (case["levels"], k, v[k], case[k])
        assert [st.units(v[k], hw["unit_bytes"]) for k in ("ms", "act_f", "act_b")] == case["units"]
    # memory is rounded UP to whole units (a plan must not be credited memory it does not have)
    assert [st.units(x, 3.0 * 2 ** 20) for x in (0.0, 1.0, 3.0 * 2 ** 20, 5.0 * 2 ** 20)] == [0, 1, 1, 2]
    for t in g["transforms"]:
        a, b = (tuple(tuple(x) for x in t[k]) for k in ("prev", "next"))
        assert st.transform_cost(layer["bnd"], a, b, hw, Bm) == t["R"], t
    # the table form agrees with the single-entry form, M follows Eq. 2's split, R[0] is zero
    strategies = [(tuple(tuple(x) for x in c["levels"]), c["ckpt"]) for c in g["cases"]]
    tab = st.cost_model([layer, layer], strategies, hw, Bm, 3, hw["unit_bytes"])
    for s, case in enumerate(g["cases"]):
        assert float(tab["c"][1, s]) == case["c"] and float(tab["c_ns"][0, s]) == case["c_ns"]
        assert [int(tab[k][1, s]) for k in ("O_ms", "O_f", "O_b")] == case["units"]
        for i in range(3):
            assert int(tab["M"][i, 0, s]) == case["units"][0] + (3 - i) * case["units"][1]
    assert not tab["R"][0].any()
    assert float(tab["R"][1, 0, 1]) == 0.01171875 and float(tab["R"][1, 0, 2]) == 0.015625
    assert float(tab["R"][1, 1, 0]) == 0.01171875 and float(tab["R"][1, 0, 0]) == 0.0


def pin_takeaway3(st):
    """The paper's argument for Takeaway #3, on the model: with communication only
    (no FLOPs, no activations, one bandwidth) N1-way DP inside/outside N2-way SDP
    costs pbytes/bw * [2(N1-1)/N1 + 3(N2-1)/N2], more than N-way SDP's 3(N-1)/N, and
    holds N/N2 times the model state."""
    hw = dict(rate=1.0, bw_in=1.0, bw_out=1.0, param_bytes=1.0, state_bytes=1.0, slow=1.3, unit_bytes=1.0, island=1)
    layer = dict(params=1024.0, flops=0.0, bnd=0.0, int=0.0)
    for N in (4, 8, 16):
        pure = st.layer_costs(layer, ((2, N),), 0, hw, 1.0)
        assert abs(pure["c"] - 1024.0 * 3 * (N - 1) / N) < 1e-9 and pure["ms"] == 1024.0 / N
        assert abs(pure["c_ns"] - 1024.0 * 2 * (N - 1) / N) < 1e-9     # no reduce-scatter without gradient sync
        dp = st.layer_costs(layer, ((1, N),), 0, hw, 1.0)
        assert abs(dp["c"] - 1024.0 * 2 * (N - 1) / N) < 1e-9 and dp["ms"] == 1024.0 and dp["c_ns"] == 0.0
        N1 = 2
        while N1 < N:
            N2 = N // N1
            for lev in (((1, N1), (2, N2)), ((2, N2), (1, N1))):
                mix = st.layer_costs(layer, lev, 0, hw, 1.0)
                want = 1024.0 * (2 * (N1 - 1) / N1 + 3 * (N2 - 1) / N2)
                assert abs(mix["c"] - want) < 1e-9 and mix["c"] > pure["c"] and mix["ms"] == 1024.0 / N2 > pure["ms"]
            N1 *= 2


def pin_properties(st):
    """Computation only (infinite bandwidth is not allowed, so: zero bytes):
    backward = 2 x forward, CKPT adds one forward: c = 3 t_f, 4 t_f with CKPT, and
    t_f = Bm * flops / (group size) / rate for every tree of the group.  Memory:
    CKPT moves the intermediate activations from O_f to O_b and changes nothing
    else; M[i] - M[i+1] = O_f; times never decrease when the slowdown grows."""
    hw = gi.default_hardware()
    layers = gi.table1_layers("BERT-Huge-32")
    layer = dict(params=0.0, flops=float(layers[0, 1]), bnd=0.0, int=0.0)
    for g in (1, 2, 8):
        for lev, ck in st.enumerate_strategies(g):
            v = st.layer_costs(layer, lev, ck, hw, 16.0)
            t_f = 16.0 * layer["flops"] / g / hw["rate"]
            assert abs(v["c"] - (4 if ck else 3) * t_f) <= 1e-12 * t_f and v["c_ns"] == v["c"]
    full = dict(params=float(layers[0, 0]), flops=float(layers[0, 1]), bnd=float(layers[0, 2]), int=float(layers[0, 3]))
    strategies = st.enumerate_strategies(8)
    n = len(strategies) // 2
    for s in range(n):
        a = st.layer_costs(full, strategies[s][0], 0, hw, 16.0)
        b = st.layer_costs(full, strategies[s + n][0], 1, hw, 16.0)
        assert strategies[s][0] == strategies[s + n][0]
        assert a["ms"] == b["ms"] and a["act_b"] == 0.0 and b["c"] > a["c"]
        assert abs((b["act_f"] + b["act_b"]) - a["act_f"]) <= 1e-9 * a["act_f"]
        slower = st.layer_costs(full, strategies[s][0], 0, dict(hw, slow=1.6), 16.0)
        assert slower["c"] >= a["c"] and slower["c_ns"] >= a["c_ns"] >= 0 and a["c"] >= a["c_ns"]
    tab = st.cost_model([full] * 3, strategies, hw, 16.0, 4, hw["unit_bytes"])
    assert np.array_equal(tab["M"][:-1] - tab["M"][1:], np.broadcast_to(tab["O_f"], (3,) + tab["O_f"].shape))
    assert np.array_equal(tab["M"][-1], tab["O_f"] + tab["O_ms"])       # the last stage: Eq. 3's M = O_f + O_ms
    R = tab["R"][1]
    assert np.array_equal(R, R.T) and not np.diag(R).any() and (R >= 0).all()
    # permutations matter: TP across islands is slower than TP inside one
    hw4 = dict(hw, island=4)
    inner = st.layer_costs(full, ((1, 2), (3, 4)), 0, hw4, 16.0)["c"]
    outer = st.layer_costs(full, ((3, 4), (1, 2)), 0, hw4, 16.0)["c"]
    assert outer > inner


def run_all(st):
    pin_counts(st)
    pin_enumeration(st)
    pin_fixture(st)
    pin_takeaway3(st)
    pin_properties(st)
