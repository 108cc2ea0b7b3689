"""The oracle's Algorithm 3 outer loop (E_all, b_up window, first failure stops)
against a hand-worked fixture, the definition of Eq. 2 written out in Python and
the bounds E_f <= E_all <= E_f + b_up.  CPU only."""
import os
import subprocess

import numpy as np
import pytest

import oracle
import pins
from test_oracle_pins import solve


def test_worked_example():
    pins.pin_select_golden(solve, oracle.select_budget, oracle.e_all)


def test_properties_and_python_rewrite():
    pins.pin_select_properties(solve, oracle.select_budget, oracle.e_all)


SRC = open(os.path.join(os.path.dirname(oracle.__file__), "gbmw_oracle.c")).read()
MUTANTS = [
    ("backward term of the wrong layer", "int64_t here = fwd + Ob[(size_t)i * S + s];",
     "int64_t here = fwd + Ob[(size_t)(i > 0 ? i - 1 : 0) * S + s];"),
    ("model states left out", "return peak + ms;", "return peak;"),
    ("forward prefix excludes the layer itself",
     "        fwd += Of[(size_t)i * S + s];\n        ms += Oms[(size_t)i * S + s];\n        int64_t here = fwd + Ob[(size_t)i * S + s];",
     "        ms += Oms[(size_t)i * S + s];\n        int64_t here = fwd + Ob[(size_t)i * S + s];\n        fwd += Of[(size_t)i * S + s];"),
    ("min instead of max over layers", "if (i == 0 || here > peak) peak = here;", "if (i == 0 || here < peak) peak = here;"),
    ("strict budget check", "Oms, cur) <= E) opt = e;", "Oms, cur) < E) opt = e;"),
    ("no stop at the first failure", "        else break;\n    }\n    free(cur);", "    }\n    free(cur);"),
    ("window starts one too late", "for (int64_t e = opt + 1; e <= E; ++e) {", "for (int64_t e = opt + 2; e <= E; ++e) {"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new, tmp_path, monkeypatch):
    assert SRC.count(old) == 1, old
    src = tmp_path / "mut.c"
    lib = tmp_path / "mut.so"
    src.write_text(SRC.replace(old, new))
    subprocess.run(["gcc", *oracle.CFLAGS, str(src), "-o", str(lib), "-lm"], check=True)
    monkeypatch.setattr(oracle, "_lib", oracle._bind(str(lib)))
    with pytest.raises(AssertionError):
        pins.pin_select_golden(solve, oracle.select_budget, oracle.e_all)
        pins.pin_select_properties(solve, oracle.select_budget, oracle.e_all)
