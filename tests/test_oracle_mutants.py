"""A few quick mutants of the oracle must be caught by its pins (the full list: tests/oracle_mutants.py).
The mistakes are planted in a temporary copy of the oracle source, on the CPU; nothing in the tree changes."""
import os
import shutil

import pytest

import oracle_mutants as om

QUICK = {
    "refine strict<": ["tests/test_oracle_tree.py"],
    "balance not periodic": ["tests/test_oracle_tree.py"],
    "lagrange sign": ["tests/test_oracle_stencils.py"],
    "d2 centre": ["tests/test_oracle_stencils.py"],
    "ko scale": ["tests/test_oracle_pipeline.py"],
}


@pytest.fixture(scope="module")
def box():
    tmp = om.sandbox()
    yield tmp
    shutil.rmtree(tmp, ignore_errors=True)


@pytest.mark.parametrize("name", sorted(QUICK))
def test_planted_mistake_is_caught(box, name):
    original = open(os.path.join(om.ROOT, "oracle", "octfd_oracle.c")).read()
    (m,) = [m for m in om.MUTANTS if m[0] == name]
    killed, by = om.run_mutant(box, original, *m, tests=QUICK[name])
    assert killed, "the pins do not notice: " + name
    assert by is not None


def test_the_unchanged_copy_passes(box):
    # control: a "mutant" that changes nothing must survive, or the kills above would prove nothing
    original = open(os.path.join(om.ROOT, "oracle", "octfd_oracle.c")).read()
    killed, by = om.run_mutant(box, original, "none", "#define NPT 8", "#define NPT 8", 1, tests=["tests/test_oracle_stencils.py"])
    assert not killed, by


def test_every_mutant_still_applies_to_the_oracle_source():
    original = open(os.path.join(om.ROOT, "oracle", "octfd_oracle.c")).read()
    for name, old, new, nth in om.MUTANTS:
        assert original.count(old) >= nth, name
        assert old != new
