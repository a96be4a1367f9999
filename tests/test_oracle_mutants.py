"""The pins must have teeth: copies of the oracle with one planted mistake each must fail them.

Every mutant is the oracle's C source with a single textual change of the kind a slip would make
(a dropped term, a wrong sign, index, constant or inequality, swapped operands).  It is compiled
on the CPU into a temporary library and the whole pin suite (tests/test_oracle_pins.py) runs
against it in a child process; the suite must report failures.  The mistakes are planted in the
oracle only; no GPU is involved and the HIP path is never touched.
"""
import os
import subprocess
import sys

import pytest

from tests.mutants import MUTANTS, ROOT, build_mutant

def run_mutant(workdir, name):
    lib = build_mutant(workdir, name)
    env = dict(os.environ, RC_ORACLE_LIB=lib, OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return r.returncode, r.stdout[-1500:] + r.stderr[-500:]


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """Every mutant built and judged once, a few at a time (each run is a child process of a few seconds)."""
    from concurrent.futures import ThreadPoolExecutor
    workdir = str(tmp_path_factory.mktemp("mutants"))
    workers = max(1, min(8, len(os.sched_getaffinity(0))))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        futures = {m[0]: pool.submit(run_mutant, workdir, m[0]) for m in MUTANTS}
        return {name: f.result() for name, f in futures.items()}


def test_mutant_names_are_unique():
    assert len({m[0] for m in MUTANTS}) == len(MUTANTS)


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_pins_reject_mutant(outcomes, name):
    code, tail = outcomes[name]
    # 1 = some pin failed (what must happen); 0 = the mistake went unnoticed; anything else = the suite itself broke
    assert code == 1, f"mutant {name}: pin suite exit code {code}\n{tail}"
