"""The pins must catch planted mistakes: for every mutation in tests/oracle_mutations.py the pin suite is run
in a subprocess with the mutation applied to the oracle (CPU only) and has to FAIL."""
import os
import subprocess
import sys

import pytest

from tests.oracle_mutations import MUTATIONS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_detect_mutation(name):
    env = dict(os.environ, ORACLE_MUTATION=name)
    p = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert p.returncode != 0, f"the pins did not notice the planted mistake '{name}':\n{p.stdout[-2000:]}"
    assert "failed" in p.stdout or "error" in p.stdout.lower()


def test_unmutated_pins_pass_in_the_same_harness():
    env = {k: v for k, v in os.environ.items() if k != "ORACLE_MUTATION"}
    p = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert p.returncode == 0, p.stdout[-2000:]
