"""Do the pins notice a mistake?  Each entry of oracle_mutant_list plants one plausible mistake in a copy of the
oracle (never in the repository's files); the pin tests then run against that copy in a child process and must
fail.  A copy without a mistake must pass, so a failure comes from the pins and not from the harness.  Only pins
are run (tests that compare the library with the oracle are deselected): the point is that the oracle is held by
something other than the code it checks.  CPU only."""
import concurrent.futures as cf
import os
import py_compile
import shutil
import subprocess
import sys
import tempfile
from pathlib import Path

from oracle_mutant_list import C_MUTANTS, PY_MUTANTS

ROOT = Path(__file__).resolve().parents[1]
FILES = ("__init__.py", "astraea_oracle.c", "budget_search.py")


def _run_pins(mutant):
    """Returns (name, outcome): 'killed' / 'survived' / a description of a harness problem."""
    name, fname, old, new, target = mutant
    tmp = Path(tempfile.mkdtemp(prefix="oracle_mutant_"))
    try:
        pkg = tmp / "oracle"
        pkg.mkdir()
        for f in FILES:
            shutil.copy(ROOT / "oracle" / f, pkg / f)
        if fname is not None:
            src = (pkg / fname).read_text()
            if src.count(old) != 1:
                return name, f"text to replace occurs {src.count(old)} times"
            (pkg / fname).write_text(src.replace(old, new))
        # the planted mistake must still be a program: build it here, so that a pin can only fail on a value
        try:
            py_compile.compile(str(pkg / "budget_search.py"), cfile=str(tmp / "bs.pyc"), doraise=True)
        except py_compile.PyCompileError as e:
            return name, "does not compile: " + str(e)[-300:]
        cc = subprocess.run(["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
                             "-shared", "-o", str(pkg / "liboracle.so"), str(pkg / "astraea_oracle.c"), "-lm"],
                            capture_output=True, text=True)
        if cc.returncode != 0:
            return name, "does not compile: " + cc.stderr[-300:]
        env = dict(os.environ, ASTRAEA_TEST_ORACLE_ROOT=str(tmp), OMP_NUM_THREADS="1")
        r = subprocess.run([sys.executable, "-m", "pytest", str(ROOT / "tests" / target), "-x", "-q", "-m", "not gpu",
                            "-k", "not test_library_", "-p", "no:cacheprovider"],
                           env=env, capture_output=True, text=True, cwd=ROOT, timeout=600)
        if r.returncode == 0:
            return name, "survived"
        if r.returncode == 1 and " failed" in r.stdout:
            return name, "killed"
        return name, f"pytest exit {r.returncode}: " + (r.stdout + r.stderr)[-300:]
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def test_every_planted_mistake_fails_a_pin():
    controls = [("control (pins)", None, None, None, "test_oracle_pins.py"),
                ("control (search)", None, None, None, "test_budget_search.py")]
    with cf.ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        results = dict(ex.map(_run_pins, controls + C_MUTANTS + PY_MUTANTS))
    for name, _, _, _, _ in controls:
        assert results.pop(name) == "survived", f"{name}: the unchanged copy must pass"
    not_killed = {n: v for n, v in results.items() if v != "killed"}
    assert not not_killed, not_killed
    assert len(results) == len(C_MUTANTS) + len(PY_MUTANTS)          # names are unique
