"""The oracle's strategy enumerator and cost model against their pins, the
pins against planted mistakes, and the library's host-side enumerator against
the oracle's.  CPU only."""
import importlib.util
import os

import pytest

import oracle
import oracle.strategy
import pins_strategy as ps

SRC = open(os.path.join(os.path.dirname(oracle.__file__), "strategy.py")).read()


def test_counts_of_the_paper():
    ps.pin_counts(oracle.strategy)


def test_enumeration_against_a_second_enumeration():
    ps.pin_enumeration(oracle.strategy)


def test_worked_example():
    ps.pin_fixture(oracle.strategy)


def test_takeaway3_argument_and_properties():
    ps.pin_takeaway3(oracle.strategy)
    ps.pin_properties(oracle.strategy)


def test_library_enumerator_matches(tmp_path):
    """gbmw_enumerate_strategies is host code: checked here without a GPU."""
    import paper_2307_02031_amd as g
    for gs in (1, 2, 4, 8, 16, 64):
        for ck in (False, True):
            for t3 in (False, True):
                got = g.gbmw_enumerate_strategies(gs, ck, t3)
                ref = oracle.strategy.enumerate_strategies(gs, ckpt=ck, takeaway3=t3)
                as_tuples = [(tuple((int(k), int(d)) for k, d in zip(s["kind"][:s["n_levels"]], s["degree"][:s["n_levels"]])),
                              int(s["ckpt"])) for s in got]
                assert as_tuples == ref, (gs, ck, t3)
                assert all(not s["kind"][s["n_levels"]:].any() and not s["degree"][s["n_levels"]:].any() for s in got)
    assert g._lib.gbmw_enumerate_strategies(6, 1, 1, None, 0) == -1
    assert g._lib.gbmw_enumerate_strategies(0, 1, 1, None, 0) == -1
    assert "power of two" in g.gbmw_last_error()


MUTANTS = [
    ("a paradigm may repeat", [("for kinds in itertools.permutations((DP, SDP, TP), len(degs)):", "for kinds in itertools.product((DP, SDP, TP), repeat=len(degs)):")]),
    ("Takeaway #3 drops DP with TP instead", [("if takeaway3 and DP in kinds and SDP in kinds:", "if takeaway3 and DP in kinds and TP in kinds:")]),
    ("degree 1 levels allowed", [("    d = 2\n    while d <= g:", "    d = 1 if g > 1 else 2\n    while d <= g and len(str(d)) < 3:")]),
    ("order of levels ignored (combinations)", [("for kinds in itertools.permutations((DP, SDP, TP), len(degs)):", "for kinds in itertools.combinations((DP, SDP, TP), len(degs)):")]),
    ("span measured from the outside", [("    for k, d in reversed(levels):", "    for k, d in levels:")]),
    ("backward as long as forward", [("t_b = 2.0 * t_f", "t_b = 1.0 * t_f")]),
    ("CKPT without recomputation", [("        bwd = bwd + (t_f + tp_ar)", "        bwd = bwd")]),
    ("CKPT recomputation without TP's all-reduce", [("        bwd = bwd + (t_f + tp_ar)", "        bwd = bwd + t_f")]),
    ("DP volume (N-1)/N", [("dp_ar = 2.0 * (dp - 1) / dp * pbytes", "dp_ar = 1.0 * (dp - 1) / dp * pbytes")]),
    ("SDP moves 2(N-1)/N", [("    c = fwd + overlap(bwd, sdp_ag + sync, hw[\"slow\"])", "    c = fwd + overlap(bwd, sync, hw[\"slow\"])")]),
    ("gradient sync kept in c_ns", [("    c_ns = fwd + overlap(bwd, sdp_ag, hw[\"slow\"])", "    c_ns = fwd + overlap(bwd, sdp_ag + sync, hw[\"slow\"])")]),
    ("overlap is a plain maximum", [("    return slow * lo + (hi - lo)", "    return hi")]),
    ("overlap is a plain sum", [("    return slow * lo + (hi - lo)", "    return lo + hi")]),
    ("slowdown on the longer activity", [("    return slow * lo + (hi - lo)", "    return slow * hi + (hi - lo)")]),
    ("SDP does not shard the model state", [('ms = layer["params"] * hw["state_bytes"] / (tp * sdp)', 'ms = layer["params"] * hw["state_bytes"] / tp')]),
    ("DP shards the model state", [('ms = layer["params"] * hw["state_bytes"] / (tp * sdp)', 'ms = layer["params"] * hw["state_bytes"] / (tp * sdp * dp)')]),
    ("CKPT keeps the intermediates in forward", [('        act_f, act_b = lb * layer["bnd"], lb * (layer["int"] / tp)', '        act_f, act_b = lb * (layer["bnd"] + layer["int"] / tp), lb * (layer["int"] / tp)')]),
    ("no backward memory under CKPT", [('        act_f, act_b = lb * layer["bnd"], lb * (layer["int"] / tp)', '        act_f, act_b = lb * layer["bnd"], 0.0')]),
    ("batch not split by SDP", [("    lb = Bm / (dp * sdp)", "    lb = Bm / dp")]),
    ("units rounded down", [("    return int(math.ceil(x / unit))", "    return int(math.floor(x / unit))")]),
    ("stage i keeps i + 1 micro-batches", [("M = np.stack([Oms + (P - i) * Of for i in range(P)])", "M = np.stack([Oms + (i + 1) * Of for i in range(P)])")]),
    ("R from the layer's own boundary", [("transform_cost(layers[l - 1][\"bnd\"], levp, lev, hw, Bm)", "transform_cost(layers[l][\"bnd\"] * 2, levp, lev, hw, Bm)")]),
    ("same batch split is always free", [("    share = abs(1.0 / b1 - 1.0 / b0) if b0 != b1 else 1.0 / b1", "    share = abs(1.0 / b1 - 1.0 / b0)")]),
    ("fast links everywhere", [('    bw = lambda span: hw["bw_in"] if span <= hw["island"] else hw["bw_out"]', '    bw = lambda span: hw["bw_in"]')]),
]


def _load(tmp_path, name, text):
    path = tmp_path / f"{name}.py"
    path.write_text(text)
    spec = importlib.util.spec_from_file_location(f"oracle.{name}", str(path))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_unmodified_copy_passes(tmp_path):
    ps.run_all(_load(tmp_path, "strategy_copy", SRC))


@pytest.mark.parametrize("name,edits", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, edits, tmp_path):
    text = SRC
    for old, new in edits:
        assert text.count(old) == 1, f"mutation anchor not unique/present: {old!r}"
        text = text.replace(old, new)
    mod = _load(tmp_path, "strategy_mut", text)
    with pytest.raises((AssertionError, IndexError, ValueError, RuntimeError, ZeroDivisionError)):
        ps.run_all(mod)
