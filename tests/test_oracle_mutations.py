"""The pins must reject a mistaken oracle (CPU only).

For every planted mistake of tests/oracle_mutants.py the pin tests (tests/test_oracle_*.py
except this file) are run in a child interpreter against the rewritten oracle; at least one
of them has to fail with an assertion.  A mistake that passes all pins is a gap in the pins.
The unchanged oracle is run the same way as the control.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from tests import oracle_mutants as M

ROOT = M.ROOT
PIN_FILES = sorted(os.path.join("tests", f) for f in os.listdir(os.path.join(ROOT, "tests"))
                   if f.startswith("test_oracle_") and f.endswith(".py") and f != "test_oracle_mutations.py")


def _run_pins(mutant):
    env = dict(os.environ)
    env.pop("VFM_ORACLE_MUTANT", None)
    if mutant:
        env["VFM_ORACLE_MUTANT"] = mutant
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES],
                          cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


@pytest.fixture(scope="module")
def verdicts():
    names = [None] + sorted(M.MUTANTS)
    with ThreadPoolExecutor(max_workers=4) as pool:
        return dict(zip(names, pool.map(_run_pins, names)))


def test_every_mutant_applies():
    for name in M.MUTANTS:
        assert M.mutated_source(name) != open(M.ORACLE_SRC).read(), name


def test_unchanged_oracle_passes_in_the_child(verdicts):
    r = verdicts[None]
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name", sorted(M.MUTANTS))
def test_pins_reject_the_mistake(verdicts, name):
    r = verdicts[name]
    # pytest exit code 1 = tests ran and some failed (2.. = usage or collection trouble)
    assert r.returncode == 1 and " failed" in r.stdout, f"{name}: pins passed or did not run\n{r.stdout[-1500:]}"
