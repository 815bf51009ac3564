"""Are the oracle's pins strong enough?  Each case plants ONE plausible mistake in the CPU oracle (a
dropped term, a wrong sign or index, a swapped operand, a misread rule -- see oracle_mutants.py) and
runs the pin tests of that oracle function in a fresh interpreter: they must fail.  The unmodified
oracle must pass the same files.  Everything here runs on the CPU; the HIP path is not involved."""
import os
import subprocess
import sys

import pytest

from oracle_mutants import MUTANTS, PIN_FILES

HERE = os.path.dirname(os.path.abspath(__file__))


def _run_pins(files, mutant=None):
    env = dict(os.environ)
    env.pop("SDLLM_ORACLE_MUTANT", None)
    if mutant:
        env["SDLLM_ORACLE_MUTANT"] = mutant
    env["PYTHONPATH"] = HERE + os.pathsep + env.get("PYTHONPATH", "")
    cmd = [sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider", "-p", "oracle_mutants",
           "-m", "not gpu"] + [os.path.join(HERE, f) for f in files]
    return subprocess.run(cmd, cwd=HERE, env=env, capture_output=True, text=True)


@pytest.mark.parametrize("sub", sorted(PIN_FILES))
def test_unmodified_oracle_passes_its_pins(sub):
    r = _run_pins(PIN_FILES[sub])
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    r = _run_pins(PIN_FILES[MUTANTS[name][0]], mutant=name)
    assert r.returncode == 1, f"no pin noticed the mistake '{name}':\n" + r.stdout[-1500:]
    assert "failed" in r.stdout
