"""Are the oracle's pins strong enough?  Every planted mistake of tests/_oracle_mutants.py must make at least
one of the oracle's CPU pin tests fail.  Each mistake gets a pytest session of its own (a child process with
PG_ORACLE_MUTANT set; conftest.py plants it before any test imports the oracle's functions).  CPU only."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle import pg_oracle as O
from tests._oracle_mutants import MUTANTS, plant

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_trloo.py", "tests/test_oracle_head_loss.py", "tests/test_oracle_stages.py",
             "tests/test_oracle_shard.py"]


def _run_pins(mutant):
    env = dict(os.environ, PYTHONDONTWRITEBYTECODE="1", OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1")
    if mutant:
        env["PG_ORACLE_MUTANT"] = mutant
    else:
        env.pop("PG_ORACLE_MUTANT", None)
    r = subprocess.run([sys.executable, "-m", "pytest", *PIN_FILES, "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    return mutant, r.returncode, r.stdout[-1500:]


def test_every_mutant_still_applies():
    """The expressions the mutants rewrite exist in the oracle as it stands (checked on a scratch copy)."""
    import types
    for name in MUTANTS:
        scratch = types.ModuleType("scratch_oracle")
        scratch.__dict__.update(O.__dict__)
        plant(scratch, name)
        fn = MUTANTS[name][0]
        assert scratch.__dict__[fn] is not O.__dict__[fn]


def test_pins_pass_unmutated_and_fail_for_every_planted_mistake():
    with ThreadPoolExecutor(max_workers=6) as pool:
        results = list(pool.map(_run_pins, [None] + sorted(MUTANTS)))
    clean = results[0]
    assert clean[1] == 0, "the pins must pass on the oracle as it stands:\n" + clean[2]
    survivors = [m for m, rc, _ in results[1:] if rc == 0]
    broken = [(m, out) for m, rc, out in results[1:] if rc not in (0, 1)]
    assert not broken, f"sessions that did not run to a verdict: {broken[:2]}"
    assert not survivors, f"planted mistakes no pin caught: {survivors}"
