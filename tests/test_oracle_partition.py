"""The oracle's pipeline-partition search (Algorithm 2's inner loop) against its
pins, and the pins against planted mistakes.  CPU only."""
import importlib.util
import os

import pytest

import oracle
import oracle.bmw
import pins_partition as pp

SRC_PATH = os.path.join(os.path.dirname(oracle.__file__), "bmw.py")
SRC = open(SRC_PATH).read()


def test_fixture():
    pp.pin_fixture(oracle.bmw)


def test_uniform_closed_forms():
    pp.pin_uniform_two_stages(oracle.bmw)
    pp.pin_uniform_memory_limits(oracle.bmw)
    pp.pin_uniform_three_stages(oracle.bmw)


def test_properties_and_stage_bruteforce():
    pp.pin_properties(oracle.bmw)


def test_alg3_stage_searches_in_the_loop():
    pp.pin_alg3_in_loop(oracle.bmw)


def test_throughput():
    pp.pin_throughput(oracle.bmw)


# ---------------------------------------------------------------- mutants
# (name, [(old, new), ...]); every `old` must occur exactly once in the source
MUTANTS = [
    ("limit 1 dropped", [("if not (Ck <= Cmax and Ok <= E and Ok <= O_t)", "if not (Ok <= E and Ok <= O_t)")]),
    ("limit 1 strict", [("if not (Ck <= Cmax and", "if not (Ck < Cmax and")]),
    ("limit 2 dropped", [("if not (Ck <= Cmax and Ok <= E and Ok <= O_t)", "if not (Ck <= Cmax and Ok <= O_t)")]),
    ("limit 3 dropped", [("if not (Ck <= Cmax and Ok <= E and Ok <= O_t)", "if not (Ck <= Cmax and Ok <= E)")]),
    ("limit 3 strict", [("Ok <= E and Ok <= O_t)", "Ok <= E and Ok < O_t)")]),
    ("limit 1 against the pipeline's maximum of Cns", [("validate(model, q, strat, C[i], E, O_t)", "validate(model, q, strat, max(Cns), E, O_t)")]),
    ("fastest stage gives the layer away", [("i = int(np.argmax(C))", "i = int(np.argmin(C))")]),
    ("last maximum is the slowest stage", [("i = int(np.argmax(C))", "i = len(C) - 1 - int(np.argmax(C[::-1]))")]),
    ("slower neighbour takes the layer", [("j = min(cand, key=lambda k: (C[k], k))", "j = max(cand, key=lambda k: (C[k], -k))")]),
    ("later neighbour on a tie", [("j = min(cand, key=lambda k: (C[k], k))", "j = min(cand, key=lambda k: (C[k], -k))")]),
    ("always the earlier neighbour", [("j = min(cand, key=lambda k: (C[k], k))", "j = cand[0]")]),
    ("one-layer stage may give its layer", [("if not cand or p[i] < 2:", "if not cand or p[i] < 1:")]),
    ("searched partitions are searched again", [("if q is None or q in seen:", "if q is None:")]),
    ("stage memory of the wrong stage", [('M = np.ascontiguousarray(model["M"][i][sl])', 'M = np.ascontiguousarray(model["M"][0][sl])')]),
    ("search uses stage 0's memory", [('np.ascontiguousarray(model["M"][i][sl]),\n', 'np.ascontiguousarray(model["M"][0][sl]),\n')]),
    ("O_t is the smallest stage memory of p_t", [("O_t = int(max(O))", "O_t = int(min(O))")]),
    ("O_t from an infeasible p_t", [("        if not np.isinf(cost):\n            O_t = int(max(O))", "        O_t = int(max(O))")]),
    ("plan read at e = E - 1", [("sol.backtrack(E)", "sol.backtrack(E - 1)")]),
    ("Cns charged with gradient synchronisation", [('Cns, _ = plan_cost(np.ascontiguousarray(model["c_ns"][sl])', 'Cns, _ = plan_cost(np.ascontiguousarray(model["c"][sl])')]),
    ("stage starts off by one", [("a.append(a[-1] + int(n))", "a.append(a[-1] + int(n) - (1 if len(a) > 1 else 0))")]),
    ("alpha_t without the 1 -", [("np.float32(np.float32(1) - np.float32(np.float32(max(C)) / tot))", "np.float32(np.float32(max(C)) / tot)")]),
    ("alpha_m from the smallest stage", [("float(max(int(x) for x in O)) / float(so)", "float(min(int(x) for x in O)) / float(so)")]),
    ("loop goes on after an infeasible search", [("        if not feasible:\n            break\n", "")]),
    ("max_iter ignored", [("while Q and len(trace) < max_iter:", "while Q:")]),
    ("throughput keeps going after out-of-memory", [("        if np.isinf(c_opt):\n            break", "        if np.isinf(c_opt):\n            continue")]),
    ("Algorithm 3: plan read at e = E although its overall memory does not fit",
     [("_, cost, plan, mem = select_budget(sol, Of, Ob, Oms)", "plan, cost, mem = sol.backtrack(E)")]),
    ("Algorithm 3: stage memory is the forward memory, not E_all",
     [("_, cost, plan, mem = select_budget(sol, Of, Ob, Oms)", "_, cost, plan, _ = select_budget(sol, Of, Ob, Oms); mem = int(sum(model[\"M\"][i][a + k][plan[k]] for k in range(n)))")]),
    ("Algorithm 3: validate checks the forward memory only",
     [("        O = e_all(Of, Ob, Oms, strat[sl])\n", "        O = O\n")]),
    ("Algorithm 3: backward activations of stage 0",
     [('Ob = np.ascontiguousarray(model["Ob"][i][sl])', 'Ob = np.ascontiguousarray(model["Ob"][0][sl])')]),
    ("Algorithm 3: model states of stage 0",
     [('Oms = np.ascontiguousarray(model["Oms"][i][sl])', 'Oms = np.ascontiguousarray(model["Oms"][0][sl])')]),
    ("Algorithm 3: O_f taken as all of M",
     [('Of = np.ascontiguousarray(model["M"][i][sl] - Oms)', 'Of = np.ascontiguousarray(model["M"][i][sl])')]),
    ("throughput takes the worst degree", [("c_opt = np.float32(min(", "c_opt = np.float32(max(")]),
]


def _load(tmp_path, name, text):
    """A copy of the module, inside the oracle package so that its relative
    imports resolve, from a temporary file."""
    path = tmp_path / f"{name}.py"
    path.write_text(text)
    spec = importlib.util.spec_from_file_location(f"oracle.{name}", str(path))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_unmodified_copy_passes(tmp_path):
    pp.run_all(_load(tmp_path, "bmw_copy", SRC))


@pytest.mark.parametrize("name,edits", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, edits, tmp_path):
    text = SRC
    for old, new in edits:
        assert text.count(old) == 1, f"mutation anchor not unique/present: {old!r}"
        text = text.replace(old, new)
    mod = _load(tmp_path, "bmw_mut", text)
    with pytest.raises((AssertionError, IndexError, ValueError, RuntimeError)):
        pp.run_all(mod)
