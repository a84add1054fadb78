"""The oracle's pins must fail when the oracle is wrong: every planted mistake of
`oracle_mutants.MUTANTS` (one altered spot each) is run against its pin files in a child process,
and the pins have to report a failure.  A mistake that survives means a pin is missing."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import oracle_mutants as M  # noqa: E402


@pytest.mark.parametrize("name", sorted(M.MUTANTS))
def test_mutant_applies_to_the_current_source(name):
    """Every altered spot exists exactly once in the oracle as it stands, and the result still compiles."""
    compile(M.mutated_source(name), "mutant", "exec")


def _run(name):
    env = dict(os.environ, BAKLAVA_ORACLE_MUTANT=name)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *M.MUTANTS[name][1]]
    r = subprocess.run(cmd, cwd=M.ROOT, env=env, capture_output=True, text=True, timeout=600)
    return name, r.returncode, (r.stdout + r.stderr)[-600:]


def test_every_planted_mistake_is_caught():
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(_run, sorted(M.MUTANTS)))
    survivors = [n for n, rc, _ in results if rc == 0]
    broken = [(n, rc, tail) for n, rc, tail in results if rc not in (0, 1)]
    assert not broken, f"pin runs that did not end in pass/fail: {broken}"
    assert not survivors, f"planted mistakes no pin noticed: {survivors}"
