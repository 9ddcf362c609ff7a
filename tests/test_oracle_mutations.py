"""Do the pins pin?  Every planted mistake in the CPU oracle must make at least one pin test fail (CPU only).

The pin files are re-run in child processes with one mutant of ``tests/mutants.py`` switched on.  A mutant
that survives means the oracle could carry that mistake unnoticed, and with it every parity claim.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from tests import mutants

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(target: str, mutant: str | None):
    env = dict(os.environ)
    env.pop(mutants.ENV, None)
    if mutant:
        env[mutants.ENV] = mutant
    env["OMP_NUM_THREADS"] = "1"
    proc = subprocess.run([sys.executable, "-m", "pytest", target, "-x", "-q", "-p", "no:cacheprovider"],
                          cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    return proc.returncode, proc.stdout[-1500:]


def test_every_mutant_has_a_target_and_the_pins_pass_unmutated():
    assert set(mutants.MUTANTS) == set(mutants.TARGETS)
    assert mutants.ENV not in os.environ, "the mutation switch must never be set for a normal run"


def test_every_planted_mistake_is_caught_by_a_pin():
    names = sorted(mutants.TARGETS)
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda n: _run(mutants.TARGETS[n], n), names))
    survivors = [n for n, (rc, _) in zip(names, results) if rc == 0]
    broken = [(n, out) for n, (rc, out) in zip(names, results) if rc not in (0, 1)]
    assert not broken, f"pin run did not complete under mutants: {broken[:2]}"
    assert not survivors, f"mutants that no pin caught: {survivors}"
