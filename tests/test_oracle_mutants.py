"""The oracle's pins must notice a planted mistake: for every entry of
`oracle_mutants.MUTANTS` the pin files are re-run in a child process with that
mistake patched into the oracle, and at least one pin has to fail.  Unpatched,
the same command has to pass.  CPU only; the child processes run a few at a time."""

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle_mutants import MUTANTS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_sketch.py", "tests/test_oracle_scores.py", "tests/test_oracle_select.py",
             "tests/test_oracle_adaptive.py", "tests/test_oracle_quality.py", "tests/test_abi.py"]


def _run_pins(mutant):
    env = dict(os.environ)
    env.pop("CURDKV_ORACLE_MUTANT", None)
    env["OMP_NUM_THREADS"] = "1"
    if mutant:
        env["CURDKV_ORACLE_MUTANT"] = mutant
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *PIN_FILES]
    p = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    return p.returncode, p.stdout[-1500:]


@pytest.fixture(scope="module")
def outcomes():
    names = [None] + sorted(MUTANTS)
    workers = max(1, min(8, (os.cpu_count() or 2) - 1))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        return dict(zip(names, pool.map(_run_pins, names)))


def test_pins_pass_without_a_planted_mistake(outcomes):
    rc, out = outcomes[None]
    assert rc == 0, out


@pytest.mark.parametrize("mutant", sorted(MUTANTS))
def test_pins_notice(outcomes, mutant):
    rc, out = outcomes[mutant]
    assert rc == 1 and " failed" in out, f"no pin fails with the mistake '{mutant}' planted:\n{out}"
