"""Do the pins have teeth?  Each case plants ONE plausible mistake in a copy of
the oracle's C source (on the CPU, in a temporary build), and the pins must
reject it.  The unmodified source must pass the very same call."""
import os
import subprocess

import numpy as np
import pytest

import oracle
import pins

SRC = open(os.path.join(os.path.dirname(oracle.__file__), "gbmw_oracle.c")).read()

# (name, [(old, new), ...]); every `old` must occur exactly once in the source
MUTANTS = [
    ("transposed R operand",
     [("Cp[(size_t)e * S + sp] + Rl[(size_t)sp * S + s]", "Cp[(size_t)e * S + sp] + Rl[(size_t)s * S + sp]")]),
    ("dropped layer cost c(l,s)",
     [("Tl[(size_t)ep * S + s] + cl[s] : INFINITY", "Tl[(size_t)ep * S + s] : INFINITY")]),
    ("dropped transformation cost R",
     [("Cp[(size_t)e * S + sp] + Rl[(size_t)sp * S + s]", "Cp[(size_t)e * S + sp]")]),
    ("shift off by one (exact fit refused)",
     [("(ep >= 0) ? Tl", "(ep > 0) ? Tl")]),
    ("base case off by one",
     [("((int64_t)e >= (int64_t)M[s]) ? c[s]", "((int64_t)e > (int64_t)M[s]) ? c[s]")]),
    ("ties to the highest predecessor",
     [("if (x < t) { t = x; a = sp; }", "if (x <= t) { t = x; a = sp; }")]),
    ("ties to the highest final strategy",
     [("if (x < t) { t = x; a = s; }", "if (x <= t) { t = x; a = s; }")]),
    ("R of the wrong layer",
     [("const float *Rl = R + (size_t)l * S * S;", "const float *Rl = R + (size_t)(l - 1) * S * S;")]),
    ("M of the wrong layer",
     [("const int32_t *Ml = M + (size_t)l * S;", "const int32_t *Ml = M + (size_t)(l - 1) * S;")]),
    ("c of the wrong layer",
     [("const float *cl = c + (size_t)l * S;", "const float *cl = c + (size_t)(l - 1) * S;")]),
    ("additions reassociated to C + (R + c)",
     [("Cp[(size_t)e * S + sp] + Rl[(size_t)sp * S + s]", "Cp[(size_t)e * S + sp] + (Rl[(size_t)sp * S + s] + cl[s])"),
      ("Tl[(size_t)ep * S + s] + cl[s] : INFINITY", "Tl[(size_t)ep * S + s] : INFINITY")]),
    ("backtrack reads the record before paying the layer's memory",
     [("        e -= M[(size_t)l * S + s];            /* budget left for layers < l */\n"
       "        s = A[(size_t)l * slab + (size_t)e * S + s];",
       "        { int s_old = s; s = A[(size_t)l * slab + (size_t)e * S + s];\n"
       "          e -= M[(size_t)l * S + s_old]; }")]),
    ("max instead of min over predecessors",
     [("float t = INFINITY;\n                int a = 0;\n                for (int sp = 0; sp < S; ++sp) {\n"
       "                    float x = Cp[(size_t)e * S + sp] + Rl[(size_t)sp * S + s];\n"
       "                    if (x < t) { t = x; a = sp; }",
       "float t = -INFINITY;\n                int a = 0;\n                for (int sp = 0; sp < S; ++sp) {\n"
       "                    float x = Cp[(size_t)e * S + sp] + Rl[(size_t)sp * S + s];\n"
       "                    if (x > t) { t = x; a = sp; }")]),
]


def _build(tmp_path, name, text):
    src = tmp_path / f"{name}.c"
    lib = tmp_path / f"{name}.so"
    src.write_text(text)
    subprocess.run(["gcc", *oracle.CFLAGS, str(src), "-o", str(lib), "-lm"], check=True)
    return oracle._bind(str(lib))


def _solver_for(lib, monkeypatch):
    monkeypatch.setattr(oracle, "_lib", lib)

    def solve(c, M, R, E):
        return oracle.solve(np.ascontiguousarray(c, np.float32), np.ascontiguousarray(M, np.int32),
                            np.ascontiguousarray(R, np.float32), E, keep_T=True)
    return solve


def test_unmodified_copy_passes(tmp_path, monkeypatch):
    pins.run_all_pins(_solver_for(_build(tmp_path, "orig", SRC), monkeypatch))


@pytest.mark.parametrize("name,edits", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, edits, tmp_path, monkeypatch):
    text = SRC
    for old, new in edits:
        assert text.count(old) == 1, f"mutation anchor not unique/present: {old!r}"
        text = text.replace(old, new)
    solve = _solver_for(_build(tmp_path, "mut", text), monkeypatch)
    with pytest.raises(AssertionError):
        pins.run_all_pins(solve)
