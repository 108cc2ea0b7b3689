"""The oracle's C source under AddressSanitizer and UndefinedBehaviorSanitizer (host only):
a second build of gbmw_oracle.c with -fsanitize=address,undefined runs every pin of the table
solve, the brute force, the backtrack, Algorithm 3's loop and the pipeline cost, plus a
multi-threaded solve, in a child process (the sanitizer runtime has to be the first library a
process loads).  Any out-of-bounds access, signed overflow or misaligned access ends the child
with a report and a non-zero status."""
import os
import subprocess
import sys

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)

CHILD = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {here!r})
import numpy as np
import oracle, pins, gbmw_inputs as gi
oracle._lib = oracle._bind({lib!r})
from test_oracle_pins import solve
pins.run_all_pins(solve)
pins.pin_select_golden(solve, oracle.select_budget, oracle.e_all)
pins.pin_select_properties(solve, oracle.select_budget, oracle.e_all)
import test_oracle_pipeline as tp
tp.test_worked_example()
# OpenMP rows, ragged sizes, memories beyond the budget, +inf costs
p = gi.random_instance(977, 5, 7, 333, M_rng=(0, 400))
p.c[1, 2] = np.inf
a = oracle.solve(p.c, p.M, p.R, p.E, nthreads=4)
b = oracle.solve(p.c, p.M, p.R, p.E, nthreads=1)
assert np.array_equal(a.C.view(np.uint32), b.C.view(np.uint32)) and np.array_equal(a.A, b.A)
for e in (0, 1, 200, 333):
    a.backtrack(e)
opt, nopt, plan = oracle.bruteforce(p.c[:4, :4].copy(), p.M[:4, :4].copy(), p.R[:4, :4, :4].copy(), 333, e_q=333)
print("sanitized oracle: all pins passed")
"""


SRC = os.path.join(ROOT, "oracle", "gbmw_oracle.c")


def _run_sanitized(tmp_path, source_text, child):
    src = tmp_path / "gbmw_oracle_san.c"
    src.write_text(source_text)
    lib = tmp_path / "libgbmw_oracle_san.so"
    flags = [f for f in oracle.CFLAGS if f != "-O2"] + ["-O1", "-g", "-fsanitize=address,undefined",
                                                        "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    subprocess.run(["gcc", *flags, str(src), "-o", str(lib), "-lm"], check=True)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()
    assert os.path.isabs(asan), "gcc has no libasan.so"
    env = dict(os.environ)
    # the sanitizer runtime goes in front of whatever is preloaded already
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    return subprocess.run([sys.executable, "-c", child.format(root=ROOT, here=HERE, lib=str(lib))], env=env,
                          capture_output=True, text=True, timeout=600)


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    r = _run_sanitized(tmp_path, open(SRC).read(), CHILD)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "all pins passed" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]


PROBE = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {here!r})
import oracle, gbmw_inputs as gi
oracle._lib = oracle._bind({lib!r})
p = gi.random_instance(978, 3, 4, 50, M_rng=(1, 9))
oracle.solve(p.c, p.M, p.R, p.E, keep_C=False, keep_T=False)
print("finished")
"""


def test_the_sanitized_build_catches_a_planted_out_of_bounds_read(tmp_path):
    """The leg above has teeth: a copy of the source whose shift reads one row below the
    product's first row (budget -1) is stopped by AddressSanitizer; the unmodified source runs
    the same call to its end."""
    text = open(SRC).read()
    old, new = "(ep >= 0) ? Tl", "(ep >= -1) ? Tl"
    assert text.count(old) == 1
    good = _run_sanitized(tmp_path, text, PROBE)
    assert good.returncode == 0 and "finished" in good.stdout, good.stderr[-3000:]
    bad = _run_sanitized(tmp_path, text.replace(old, new), PROBE)
    assert bad.returncode != 0 and "AddressSanitizer" in bad.stderr, bad.stderr[-3000:]
